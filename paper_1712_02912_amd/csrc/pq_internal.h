// Internal declarations shared by the translation units of libpqadc (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "pq_adc.h"
#include "pq_adc_bench.h"

// Tuning and test switches (pq_set_option).  PQ_OPT_UNSET = the kernel's own default.
enum pq_option_id {
    PQ_OPT_SCAN_PRUNE = 0, PQ_OPT_SCAN_Q8, PQ_OPT_SCAN_FORCE_GENERAL, PQ_OPT_SCAN_BLOCKS, PQ_OPT_SCAN_ITEMS_PER_BLOCK,
    PQ_OPT_SCAN_HEAD, PQ_OPT_LUT_MFMA, PQ_OPT_IVF_PRUNE, PQ_OPT_IVF_WS_GIB, PQ_OPT_IVF_BLOCK_WAVES, PQ_OPT_SCAN_WIDE_SEED, PQ_OPT_IVF_SHORT_MAX, PQ_OPT_IVF_COARSE_F32, PQ_OPT_IVF_QUICK_CHUNK_ROWS, PQ_OPT_IVF_COARSE_F16, PQ_OPT_COUNT
};
constexpr int PQ_OPT_UNSET = -2147483647 - 1;

struct pq_ctx {
    int device;
    hipStream_t stream;
    void *ws;          // device workspace, grown on demand (or the fixed scratch of the call that allocates nothing)
    size_t ws_bytes;
    int ws_fixed;      // ws must not grow: a request beyond ws_bytes is an error
    void *lut_ws;      // Tables step of many tiles: operands as doubles and their norms, grown on demand
    size_t lut_ws_bytes;
    void *host_pin;    // 256 bytes of pinned host memory for the few words a call reads back
    hipStream_t aux_stream;          // ivf_adc_search: work that does not depend on the tables runs beside them
    hipEvent_t aux_fork, aux_join;
    int opt[PQ_OPT_COUNT];
    int num_cu;
    int profiling;              // bracket the scan kernel with events
    hipEvent_t ev_begin, ev_end;
    int ev_valid;
    // measurement aids (valid while profiling): the scan kernel last launched, and where its counters live in the workspace
    char last_scan_name[320];
    int last_scan_qpp, last_scan_passes;
    const unsigned long long *stat_parked;
    const uint32_t *stat_ncand;
    int stat_ncand_len;
    char err[512];
};

namespace pq {

// ---- host helpers -----------------------------------------------------------------
int fail(pq_ctx *ctx, int code, const char *fmt, ...);
int hip_fail(pq_ctx *ctx, hipError_t e, const char *what);
// Make the workspace at least `bytes` large; returns PQ_OK or an error already recorded.
int ws_reserve(pq_ctx *ctx, size_t bytes);

#define PQ_HIP(ctx, call)                                                \
    do {                                                                 \
        hipError_t e__ = (call);                                         \
        if (e__ != hipSuccess) return pq::hip_fail((ctx), e__, #call);   \
    } while (0)

// value of a switch, or dflt if it was never set
static inline int opt_int(const pq_ctx *ctx, int id, int dflt) { return ctx->opt[id] == PQ_OPT_UNSET ? dflt : ctx->opt[id]; }

// measurement aid: a scan kernel without counters of its own is about to be launched
static inline void note_plain_scan(pq_ctx *ctx, const char *name, int queries_per_pass, int passes) {
    snprintf(ctx->last_scan_name, sizeof(ctx->last_scan_name), "%s", name);
    ctx->last_scan_qpp = queries_per_pass;
    ctx->last_scan_passes = passes;
    ctx->stat_parked = nullptr;
    ctx->stat_ncand = nullptr;
    ctx->stat_ncand_len = 0;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- launchers implemented in the kernel files -------------------------------------
int launch_build_luts(pq_ctx *ctx, const float *queries, const float *codebooks, int nq, int d, int m, int k,
                      float *luts);
int launch_quantize_luts(pq_ctx *ctx, const float *luts, int nq, int m, int k, const float *qmax,
                         uint8_t *qluts, float *qmin_out, float *scale_out);
int launch_qmax_prescan(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const float *luts, int nq, int m,
                        int k, int init, int kq, float *qmax_out);
int launch_rerank(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const float *luts, int nq, int m, int k,
                  const int64_t *cand, int ncand, int topk, float *out_dist, int64_t *out_ids);
int launch_scan(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const void *luts, int lf, int nq, int m,
                int k, int topk, void *out_val, int64_t *out_ids);
int launch_rotate(pq_ctx *ctx, const float *vectors, const float *rot, int64_t n, int d, float *out);
// Approximate squared distances of nq vectors to k centroids of d dimensions on the fp32 matrix cores, each within
// coarse_f32_error(d) * (||y||^2 + ||c||^2) of the exact value; coarse_f32_usable says whether the shape is served.
float coarse_f32_error(int d);
bool coarse_f32_usable(pq_ctx *ctx, const float *queries, const float *cents, int nq, int d, int k, const float *out);
int launch_coarse_f32(pq_ctx *ctx, const float *queries, const float *cents, size_t cent_stride, int nq, int d, int k, float *out);
int coarse_filter_slots(int k);   // places per query that the filtering forms write
int launch_coarse_f32_filter(pq_ctx *ctx, const float *queries, const float *cents, int nq, int d, int k, const float *theta,
                             unsigned long long *slot_keys, unsigned long long *ov_keys, unsigned int *ov_cnt, int ov_cap);
// The same filtering pass on the fp16 matrix cores (operands split into two halves each), within coarse_split16_error(d) *
// (||y||^2 + ||c||^2); magnitudes outside 2^-40 .. 2^40 keep nothing.
float coarse_split16_error(int d);
int launch_coarse_split16_filter(pq_ctx *ctx, const float *queries, const float *cents, int nq, int d, int k, const float *theta,
                                 unsigned long long *slot_keys, unsigned long long *ov_keys, unsigned int *ov_cnt, int ov_cap);
int launch_encode(pq_ctx *ctx, const float *vectors, const float *codebooks, int64_t n, int d, int m, int k, int cf,
                  uint8_t *codes);
int launch_derived_search(pq_ctx *ctx, const uint16_t *codes16, int64_t n, const float *derived_codebooks,
                          const float *codebooks, int k, const float *queries, int nq, int d, int r2, int topk,
                          float *out_dist, int64_t *out_ids, uint32_t *bucket_out, int64_t *ncand_out,
                          int64_t *cand_ids_out, int64_t cand_cap);
int launch_ivf(pq_ctx *ctx, const ivf_lists *lists, const float *codebooks, int m, int k, int cf,
               const float *queries, int nq, int nprobe, int topk, float *out_dist, int64_t *out_ids,
               int32_t *probe_out, int init, int kprime);   // (init, kprime: Quick ADC over packed 4-bit codes only)

}  // namespace pq
