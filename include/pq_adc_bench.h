/*
 * pq_adc_bench.h -- measurement aids of libpqadc.  Not part of the search API (pq_adc.h): these calls
 * exist so that a benchmark can time the scan kernel on the stream it is launched on and calibrate
 * hardware counters; nothing on the search path needs them.
 */
#ifndef PQ_ADC_BENCH_H
#define PQ_ADC_BENCH_H

#include "pq_adc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* When enabled, pq_adc_scan_topk, pq_derived_search and ivf_adc_search bracket their scan kernel (the
 * kernel that streams the codes; not the set-up and merge kernels around it) with HIP events on the
 * context's stream.  pq_last_scan_kernel_ms waits for that kernel and returns its duration. */
int pq_set_profiling(pq_ctx *ctx, int enable);
int pq_last_scan_kernel_ms(pq_ctx *ctx, float *ms);
/* What the profiled scan kernel was (waits for the stream).  name: a description of the kernel variant;
 * queries_per_pass: queries one pass over a chunk of codes serves; passes: passes over the whole code
 * array the launch makes (= groups of queries; 0 for inverted lists, where it varies per list);
 * parked_lanes: lanes (16 code bytes each) whose lower bounds let at least one (code, query) pair through
 * to the insert path; inserted_keys: (code, query) pairs that passed every test and were appended to a
 * candidate list (both 0 for kernels without these counters).  Any pointer may be NULL.  Valid until the
 * next call on the context. */
int pq_last_scan_info(pq_ctx *ctx, char *name, size_t name_bytes, int *queries_per_pass, int *passes,
                      uint64_t *parked_lanes, uint64_t *inserted_keys);
/* Plain device-to-device copy of `bytes` bytes (multiple of 16, both pointers 16-byte aligned) by one
 * kernel.  Its known traffic (bytes read + bytes written) calibrates the hardware counters that are
 * read for the scan kernels. */
int pq_calibration_copy(pq_ctx *ctx, const void *src, void *dst, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* PQ_ADC_BENCH_H */
