// C-ABI entry points of libpqadc: argument validation, context and workspace handling.
// The kernels and their launchers live in the other translation units.
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include "pq_internal.h"

namespace pq {

int fail(pq_ctx *ctx, int code, const char *fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

int hip_fail(pq_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, PQ_EHIP, "HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
}

int ws_reserve(pq_ctx *ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return PQ_OK;
    if (ctx->ws_fixed)
        return fail(ctx, PQ_ENOMEM, "this call needs %zu bytes of scratch memory, the fixed scratch of the entry point that "
                                    "allocates nothing holds %zu", bytes, ctx->ws_bytes);
    // kernels already enqueued may still use the old workspace
    PQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->ws) {
        PQ_HIP(ctx, hipFree(ctx->ws));
        ctx->ws = nullptr;
        ctx->ws_bytes = 0;
    }
    const size_t want = align_up(bytes + bytes / 4, (size_t)1 << 20);
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, PQ_ENOMEM, "workspace allocation of %zu bytes failed: %s", want, hipGetErrorString(e));
    }
    ctx->ws = p;
    ctx->ws_bytes = want;
    return PQ_OK;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Names of the switches of pq_set_option, in the order of pq_option_id; the environment variable of a
// switch is "PQ_" + its name in upper case and is read once, by pq_create.
static const char *const OPTION_NAMES[PQ_OPT_COUNT] = {"scan_prune", "scan_q8", "scan_force_general", "scan_blocks",
                                                       "scan_items_per_block", "scan_head", "lut_mfma", "ivf_prune",
                                                       "ivf_ws_gib", "ivf_block_waves", "scan_wide_seed", "ivf_short_max", "ivf_coarse_f32",
                                                       "ivf_quick_chunk_rows", "ivf_coarse_f16"};

static void options_from_environment(pq_ctx *ctx) {
    for (int i = 0; i < PQ_OPT_COUNT; ++i) {
        char var[64] = "PQ_";
        size_t at = 3;
        for (const char *c = OPTION_NAMES[i]; *c && at + 1 < sizeof(var); ++c) var[at++] = (char)(*c >= 'a' && *c <= 'z' ? *c - 32 : *c);
        var[at] = 0;
        const char *v = getenv(var);
        ctx->opt[i] = v && *v ? atoi(v) : PQ_OPT_UNSET;
    }
}

}  // namespace pq

// Scratch memory of pq_adc_scan_topk_noalloc: one copy per GPU the library runs on, held until the process
// ends.  The name is a host-side stand-in; host code uses the device address that hipGetSymbolAddress
// returns for the current device (fixed_scratch_of), never the name.
constexpr size_t FIXED_SCRATCH_BYTES = (size_t)PQ_NOALLOC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[FIXED_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void *g_fixed_scratch[MAX_DEVICES];   // per device, looked up once with that device current

namespace pq {
static int fixed_scratch_of(pq_ctx *ctx, void **out) {
    if (ctx->device < 0 || ctx->device >= MAX_DEVICES) return fail(ctx, PQ_EUNSUPPORTED, "device index %d above %d", ctx->device, MAX_DEVICES - 1);
    if (!g_fixed_scratch[ctx->device]) {
        int current = -1;
        PQ_HIP(ctx, hipGetDevice(&current));
        if (current != ctx->device) PQ_HIP(ctx, hipSetDevice(ctx->device));
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (current != ctx->device) (void)hipSetDevice(current);
        if (e != hipSuccess || !p) return hip_fail(ctx, e, "hipGetSymbolAddress(scratch)");
        g_fixed_scratch[ctx->device] = p;
    }
    *out = g_fixed_scratch[ctx->device];
    return PQ_OK;
}
}  // namespace pq

namespace pq {
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                               size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}
}  // namespace pq

using namespace pq;

extern "C" {

const char *pq_version(void) { return "pqadc-gfx950 0.1"; }

int pq_create(pq_ctx **out, int device, void *hip_stream) {
    if (!out) return PQ_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return PQ_EHIP;
    if (hipSetDevice(device) != hipSuccess) return PQ_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return PQ_EHIP;
    pq_ctx *ctx = (pq_ctx *)calloc(1, sizeof(pq_ctx));
    if (!ctx) return PQ_ENOMEM;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    strcpy(ctx->err, "no error");
    options_from_environment(ctx);
    // the address of this device's fixed scratch is looked up here, at set-up, so that
    // pq_adc_scan_topk_noalloc itself has nothing left to initialise
    void *fixed = nullptr;
    if (fixed_scratch_of(ctx, &fixed) != PQ_OK) {
        free(ctx);
        return PQ_EHIP;
    }
    *out = ctx;
    return PQ_OK;
}

int pq_set_option(pq_ctx *ctx, const char *name, int value) {
    if (!ctx || !name) return PQ_EINVAL;
    for (int i = 0; i < PQ_OPT_COUNT; ++i)
        if (strcmp(name, OPTION_NAMES[i]) == 0) {
            ctx->opt[i] = value;
            return PQ_OK;
        }
    return fail(ctx, PQ_EINVAL, "set_option: unknown option '%s'", name);
}

int pq_unset_option(pq_ctx *ctx, const char *name) { return pq_set_option(ctx, name, PQ_OPT_UNSET); }

int pq_destroy(pq_ctx *ctx) {
    if (!ctx) return PQ_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->lut_ws) (void)hipFree(ctx->lut_ws);
    if (ctx->host_pin) (void)hipHostFree(ctx->host_pin);
    if (ctx->aux_stream) {
        (void)hipStreamSynchronize(ctx->aux_stream);
        (void)hipStreamDestroy(ctx->aux_stream);
        (void)hipEventDestroy(ctx->aux_fork);
        (void)hipEventDestroy(ctx->aux_join);
    }
    if (ctx->ev_begin) (void)hipEventDestroy(ctx->ev_begin);
    if (ctx->ev_end) (void)hipEventDestroy(ctx->ev_end);
    free(ctx);
    return PQ_OK;
}

int pq_set_profiling(pq_ctx *ctx, int enable) {
    if (!ctx) return PQ_EINVAL;
    if (enable && !(ctx->ev_begin && ctx->ev_end)) {
        // both events or none: a failure must not leave half of the pair behind
        hipEvent_t b = nullptr, e = nullptr;
        hipError_t rc = hipEventCreate(&b);
        if (rc == hipSuccess) rc = hipEventCreate(&e);
        if (rc != hipSuccess) {
            if (b) (void)hipEventDestroy(b);
            return hip_fail(ctx, rc, "hipEventCreate");
        }
        ctx->ev_begin = b;
        ctx->ev_end = e;
    }
    ctx->profiling = enable ? 1 : 0;
    ctx->ev_valid = 0;
    return PQ_OK;
}

int pq_last_scan_kernel_ms(pq_ctx *ctx, float *ms) {
    if (!ctx || !ms) return PQ_EINVAL;
    if (!ctx->ev_valid) return fail(ctx, PQ_EINVAL, "no profiled scan kernel recorded");
    PQ_HIP(ctx, hipEventSynchronize(ctx->ev_end));
    PQ_HIP(ctx, hipEventElapsedTime(ms, ctx->ev_begin, ctx->ev_end));
    return PQ_OK;
}

int pq_last_scan_info(pq_ctx *ctx, char *name, size_t name_bytes, int *queries_per_pass, int *passes,
                      uint64_t *parked_lanes, uint64_t *inserted_keys) {
    if (!ctx) return PQ_EINVAL;
    if (!ctx->ev_valid) return fail(ctx, PQ_EINVAL, "no profiled scan kernel recorded");
    PQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (name && name_bytes > 0) snprintf(name, name_bytes, "%s", ctx->last_scan_name);
    if (queries_per_pass) *queries_per_pass = ctx->last_scan_qpp;
    if (passes) *passes = ctx->last_scan_passes;
    if (parked_lanes) {
        unsigned long long v[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        if (ctx->stat_parked) PQ_HIP(ctx, hipMemcpy(v, ctx->stat_parked, sizeof(v), hipMemcpyDeviceToHost));
        *parked_lanes = v[0];
#ifdef PQ_SCAN_TIMING
        fprintf(stderr, "scan phases (wave cycles x 1e6): setup %.1f loop %.1f flush %.1f refresh %.1f emit %.1f overflow %.1f\n",
                v[1] / 1e6, v[2] / 1e6, v[3] / 1e6, v[4] / 1e6, v[5] / 1e6, v[6] / 1e6);
        fprintf(stderr, "  item results sorted %llu, merged %llu, keys in them %llu\n", v[7], v[8], v[9]);
#endif
    }
    if (inserted_keys) {
        uint64_t total = 0;
        uint32_t buf[1024];
        for (int at = 0; ctx->stat_ncand && at < ctx->stat_ncand_len; at += 1024) {
            const int take = ctx->stat_ncand_len - at < 1024 ? ctx->stat_ncand_len - at : 1024;
            PQ_HIP(ctx, hipMemcpy(buf, ctx->stat_ncand + at, (size_t)take * 4, hipMemcpyDeviceToHost));
            for (int i = 0; i < take; ++i) total += buf[i];
        }
        *inserted_keys = total;
    }
    return PQ_OK;
}

int pq_calibration_copy(pq_ctx *ctx, const void *src, void *dst, size_t bytes) {
    if (!ctx) return PQ_EINVAL;
    if (!src || !dst || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst))
        return fail(ctx, PQ_EINVAL, "calibration_copy: need 16-byte aligned pointers and size");
    if (bytes == 0) return PQ_OK;
    calibration_copy_kernel<<<ctx->num_cu * 16, 256, 0, ctx->stream>>>((const uint4 *)src, (uint4 *)dst, bytes / 16);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

const char *pq_last_error(const pq_ctx *ctx) { return ctx ? ctx->err : "null context"; }

int pq_build_luts(pq_ctx *ctx, const float *queries, const float *codebooks, int nq, int d, int m, int k,
                  float *luts) {
    if (!ctx) return PQ_EINVAL;
    if (nq < 0 || d <= 0 || m <= 0 || k <= 0) return fail(ctx, PQ_EINVAL, "build_luts: sizes must be positive");
    if (d % m != 0) return fail(ctx, PQ_ESHAPE, "build_luts: d=%d is not a multiple of m=%d", d, m);
    if (k > 65536) return fail(ctx, PQ_EUNSUPPORTED, "build_luts: k=%d above 65536", k);
    if (nq == 0) return PQ_OK;
    if (!queries || !codebooks || !luts) return fail(ctx, PQ_EINVAL, "build_luts: null pointer");
    return launch_build_luts(ctx, queries, codebooks, nq, d, m, k, luts);
}

int pq_quantize_luts(pq_ctx *ctx, const float *luts, int nq, int m, int k, const float *qmax, uint8_t *qluts,
                     float *qmin_out, float *scale_out) {
    if (!ctx) return PQ_EINVAL;
    if (nq < 0 || m <= 0 || k <= 0) return fail(ctx, PQ_EINVAL, "quantize_luts: sizes must be positive");
    if ((int64_t)m * k > (1 << 24)) return fail(ctx, PQ_EUNSUPPORTED, "quantize_luts: m*k too large");
    if (nq == 0) return PQ_OK;
    if (!luts || !qmax || !qluts) return fail(ctx, PQ_EINVAL, "quantize_luts: null pointer");
    return launch_quantize_luts(ctx, luts, nq, m, k, qmax, qluts, qmin_out, scale_out);
}

static int check_codes(pq_ctx *ctx, const char *who, int cf, int m, int k) {
    if (cf != PQ_CODES_U8 && cf != PQ_CODES_U4_PACKED) return fail(ctx, PQ_EINVAL, "%s: bad code format %d", who, cf);
    if (m <= 0 || k <= 0) return fail(ctx, PQ_EINVAL, "%s: m and k must be positive", who);
    if (cf == PQ_CODES_U4_PACKED && (m % 2 != 0 || k > 16))
        return fail(ctx, PQ_ESHAPE, "%s: packed 4-bit codes need even m and k <= 16 (m=%d k=%d)", who, m, k);
    if (cf == PQ_CODES_U8 && k > 256) return fail(ctx, PQ_ESHAPE, "%s: one-byte indexes need k <= 256 (k=%d)", who, k);
    return PQ_OK;
}

int pq_qmax_prescan(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const float *luts, int nq, int m,
                    int k, int init, int kq, float *qmax_out) {
    if (!ctx) return PQ_EINVAL;
    int rc = check_codes(ctx, "qmax_prescan", cf, m, k);
    if (rc) return rc;
    if (nq < 0 || n <= 0 || init <= 0 || kq <= 0) return fail(ctx, PQ_EINVAL, "qmax_prescan: n, init, kq must be positive");
    if (init > 4096) return fail(ctx, PQ_EUNSUPPORTED, "qmax_prescan: init=%d above 4096", init);
    if (nq == 0) return PQ_OK;
    if (!codes || !luts || !qmax_out) return fail(ctx, PQ_EINVAL, "qmax_prescan: null pointer");
    return launch_qmax_prescan(ctx, codes, n, cf, luts, nq, m, k, init, kq, qmax_out);
}

int pq_adc_scan_topk(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const void *luts, pq_lut_fmt lf,
                     int nq, int m, int k, int topk, void *out_val, int64_t *out_ids) {
    if (!ctx) return PQ_EINVAL;
    int rc = check_codes(ctx, "adc_scan_topk", cf, m, k);
    if (rc) return rc;
    if (lf != PQ_LUT_F32 && lf != PQ_LUT_U8) return fail(ctx, PQ_EINVAL, "adc_scan_topk: bad table format %d", lf);
    if (nq < 0 || n < 0) return fail(ctx, PQ_EINVAL, "adc_scan_topk: negative size");
    if (topk < 1) return fail(ctx, PQ_EINVAL, "adc_scan_topk: topk must be at least 1");
    if (topk > 1024) return fail(ctx, PQ_EUNSUPPORTED, "adc_scan_topk: topk=%d above 1024", topk);
    if (n >= ((int64_t)1 << 32)) return fail(ctx, PQ_EUNSUPPORTED, "adc_scan_topk: n must be below 2^32");
    if (nq == 0) return PQ_OK;
    if (!luts || !out_val || !out_ids || (n > 0 && !codes)) return fail(ctx, PQ_EINVAL, "adc_scan_topk: null pointer");
    if (!aligned16(codes)) return fail(ctx, PQ_EINVAL, "adc_scan_topk: codes must be 16-byte aligned");
    return launch_scan(ctx, codes, n, cf, luts, lf, nq, m, k, topk, out_val, out_ids);
}

int pq_adc_scan_topk_noalloc(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const void *luts,
                             pq_lut_fmt lf, int nq, int m, int k, int topk, void *out_val, int64_t *out_ids) {
    if (!ctx) return PQ_EINVAL;
    void *fixed = nullptr;
    int rc = fixed_scratch_of(ctx, &fixed);   // (looked up by pq_create; this only reads the table)
    if (rc) return rc;
    // the same validation and the same kernels as pq_adc_scan_topk, with the fixed scratch of this GPU in
    // place of the context's workspace; a request that does not fit fails in ws_reserve
    void *const own_ws = ctx->ws;
    const size_t own_bytes = ctx->ws_bytes;
    ctx->ws = fixed;
    ctx->ws_bytes = FIXED_SCRATCH_BYTES;
    ctx->ws_fixed = 1;
    rc = pq_adc_scan_topk(ctx, codes, n, cf, luts, lf, nq, m, k, topk, out_val, out_ids);
    ctx->ws = own_ws;
    ctx->ws_bytes = own_bytes;
    ctx->ws_fixed = 0;
    return rc;
}

int pq_rerank_f32(pq_ctx *ctx, const uint8_t *codes, int64_t n, pq_code_fmt cf, const float *luts, int nq, int m,
                  int k, const int64_t *cand_ids, int ncand, int topk, float *out_dist, int64_t *out_ids) {
    if (!ctx) return PQ_EINVAL;
    int rc = check_codes(ctx, "rerank_f32", cf, m, k);
    if (rc) return rc;
    if (nq < 0 || n < 0 || ncand < 1 || topk < 1) return fail(ctx, PQ_EINVAL, "rerank_f32: bad size");
    if (topk > ncand) return fail(ctx, PQ_ESHAPE, "rerank_f32: topk=%d above ncand=%d", topk, ncand);
    if (ncand > 4096) return fail(ctx, PQ_EUNSUPPORTED, "rerank_f32: ncand=%d above 4096", ncand);
    if (n >= ((int64_t)1 << 32)) return fail(ctx, PQ_EUNSUPPORTED, "rerank_f32: n must be below 2^32");
    if (nq == 0) return PQ_OK;
    if (!luts || !cand_ids || !out_dist || !out_ids || (n > 0 && !codes)) return fail(ctx, PQ_EINVAL, "rerank_f32: null pointer");
    return launch_rerank(ctx, codes, n, cf, luts, nq, m, k, cand_ids, ncand, topk, out_dist, out_ids);
}

int pq_rotate(pq_ctx *ctx, const float *vectors, const float *rot, int64_t n, int d, float *out) {
    if (!ctx) return PQ_EINVAL;
    if (n < 0 || d <= 0) return fail(ctx, PQ_EINVAL, "rotate: bad size");
    if (n == 0) return PQ_OK;
    if (!vectors || !rot || !out) return fail(ctx, PQ_EINVAL, "rotate: null pointer");
    if (vectors == out) return fail(ctx, PQ_EINVAL, "rotate: input and output must not overlap");
    return launch_rotate(ctx, vectors, rot, n, d, out);
}

int pq_encode(pq_ctx *ctx, const float *vectors, const float *codebooks, int64_t n, int d, int m, int k,
              pq_code_fmt cf, uint8_t *codes) {
    if (!ctx) return PQ_EINVAL;
    if (n < 0 || d <= 0 || m <= 0 || k <= 0) return fail(ctx, PQ_EINVAL, "encode: bad size");
    if (cf != PQ_CODES_U8 && cf != PQ_CODES_U4_PACKED) return fail(ctx, PQ_EINVAL, "encode: bad code format");
    if (d % m != 0) return fail(ctx, PQ_ESHAPE, "encode: d=%d is not a multiple of m=%d", d, m);
    if (cf == PQ_CODES_U8 && k > 256) return fail(ctx, PQ_ESHAPE, "encode: k=%d does not fit one byte per index", k);
    if (cf == PQ_CODES_U4_PACKED && (k > 16 || m % 2 != 0))
        return fail(ctx, PQ_ESHAPE, "encode: packed 4-bit codes need k <= 16 and an even m (k=%d, m=%d)", k, m);
    if (n == 0) return PQ_OK;
    if (!vectors || !codebooks || !codes) return fail(ctx, PQ_EINVAL, "encode: null pointer");
    return launch_encode(ctx, vectors, codebooks, n, d, m, k, cf, codes);
}

int pq_derived_search(pq_ctx *ctx, const uint16_t *codes, int64_t n, const float *derived_codebooks,
                      const float *codebooks, int k, const float *queries, int nq, int d, int m, int r2, int topk,
                      float *out_dist, int64_t *out_ids, uint32_t *bucket_out, int64_t *ncand_out,
                      int64_t *cand_ids_out, int64_t cand_cap) {
    if (!ctx) return PQ_EINVAL;
    if (n < 0 || nq < 0 || d <= 0 || m <= 0 || k <= 0 || r2 < 1 || topk < 1 || cand_cap < 0)
        return fail(ctx, PQ_EINVAL, "derived_search: bad size");
    if (m != 4) return fail(ctx, PQ_EUNSUPPORTED, "derived_search: m=%d (64-bit codes of four 16-bit indexes only)", m);
    if (d % m != 0) return fail(ctx, PQ_ESHAPE, "derived_search: d=%d is not a multiple of m=%d", d, m);
    if (d > 4096) return fail(ctx, PQ_EUNSUPPORTED, "derived_search: d=%d above 4096", d);
    if (k < 256 || k > 65536) return fail(ctx, PQ_ESHAPE, "derived_search: k=%d outside 256..65536", k);
    if (topk > 128) return fail(ctx, PQ_EUNSUPPORTED, "derived_search: topk=%d above 128", topk);
    if (nq > 65535) return fail(ctx, PQ_EUNSUPPORTED, "derived_search: more than 65535 queries per call");
    if (n >= ((int64_t)1 << 32)) return fail(ctx, PQ_EUNSUPPORTED, "derived_search: n must be below 2^32");
    if (nq == 0) return PQ_OK;
    if (!derived_codebooks || !codebooks || !queries || !out_dist || !out_ids || (n > 0 && !codes))
        return fail(ctx, PQ_EINVAL, "derived_search: null pointer");
    if (!aligned16(codes)) return fail(ctx, PQ_EINVAL, "derived_search: codes must be 16-byte aligned");
    return launch_derived_search(ctx, codes, n, derived_codebooks, codebooks, k, queries, nq, d, r2, topk, out_dist,
                                 out_ids, bucket_out, ncand_out, cand_ids_out, cand_cap);
}

int ivf_adc_search(pq_ctx *ctx, const ivf_lists *lists, const float *codebooks, int m, int k, pq_code_fmt cf,
                   const float *queries, int nq, int nprobe, int topk, float *out_dist, int64_t *out_ids,
                   int32_t *probe_out) {
    if (!ctx) return PQ_EINVAL;
    if (!lists) return fail(ctx, PQ_EINVAL, "ivf_adc_search: null lists");
    int rc = check_codes(ctx, "ivf_adc_search", cf, m, k);
    if (rc) return rc;
    if (lists->nlist <= 0 || lists->d <= 0 || lists->ntotal < 0 || nq < 0)
        return fail(ctx, PQ_EINVAL, "ivf_adc_search: bad size");
    if (lists->d % m != 0) return fail(ctx, PQ_ESHAPE, "ivf_adc_search: d=%d is not a multiple of m=%d", lists->d, m);
    if (nprobe < 1 || nprobe > lists->nlist)
        return fail(ctx, PQ_ESHAPE, "ivf_adc_search: nprobe=%d outside 1..nlist=%d", nprobe, lists->nlist);
    if (topk < 1) return fail(ctx, PQ_EINVAL, "ivf_adc_search: topk must be at least 1");
    if (nprobe > 1024 || topk > 128 || cf != PQ_CODES_U8 || k != 256 || (m != 8 && m != 16))
        return fail(ctx, PQ_EUNSUPPORTED, "ivf_adc_search: covered are U8 codes, k=256, m in {8,16}, nprobe<=1024, topk<=128");
    if (lists->ntotal >= ((int64_t)1 << 32)) return fail(ctx, PQ_EUNSUPPORTED, "ivf_adc_search: ntotal must be below 2^32");
    if (nq == 0) return PQ_OK;
    if (!lists->coarse_centroids || !lists->list_offsets || !codebooks || !queries || !out_dist || !out_ids ||
        (lists->ntotal > 0 && !lists->codes))
        return fail(ctx, PQ_EINVAL, "ivf_adc_search: null pointer");
    if (!aligned16(lists->codes)) return fail(ctx, PQ_EINVAL, "ivf_adc_search: codes must be 16-byte aligned");
    return launch_ivf(ctx, lists, codebooks, m, k, cf, queries, nq, nprobe, topk, out_dist, out_ids, probe_out, 0, 0);
}

int ivf_quick_adc_search(pq_ctx *ctx, const ivf_lists *lists, const float *codebooks, int m, int k, const float *queries,
                         int nq, int nprobe, int init, int kprime, int topk, float *out_dist, int64_t *out_ids,
                         int32_t *probe_out) {
    if (!ctx) return PQ_EINVAL;
    if (!lists) return fail(ctx, PQ_EINVAL, "ivf_quick_adc_search: null lists");
    if (lists->nlist <= 0 || lists->d <= 0 || lists->ntotal < 0 || nq < 0)
        return fail(ctx, PQ_EINVAL, "ivf_quick_adc_search: bad size");
    if (m != 16 || k != 16) return fail(ctx, PQ_EUNSUPPORTED, "ivf_quick_adc_search: covered is m=16, k=16 (m=%d k=%d)", m, k);
    if (lists->d % m != 0) return fail(ctx, PQ_ESHAPE, "ivf_quick_adc_search: d=%d is not a multiple of m=%d", lists->d, m);
    if (nprobe < 1 || nprobe > lists->nlist)
        return fail(ctx, PQ_ESHAPE, "ivf_quick_adc_search: nprobe=%d outside 1..nlist=%d", nprobe, lists->nlist);
    if (topk < 1 || kprime < 1 || init < 1) return fail(ctx, PQ_EINVAL, "ivf_quick_adc_search: topk, kprime and init must be at least 1");
    if (nprobe > 1024 || topk > 128 || kprime > 128 || init > 4096)
        return fail(ctx, PQ_EUNSUPPORTED, "ivf_quick_adc_search: covered are nprobe<=1024, topk<=128, kprime<=128, init<=4096");
    if (lists->ntotal >= ((int64_t)1 << 32)) return fail(ctx, PQ_EUNSUPPORTED, "ivf_quick_adc_search: ntotal must be below 2^32");
    if (nq == 0) return PQ_OK;
    if (!lists->coarse_centroids || !lists->list_offsets || !codebooks || !queries || !out_dist || !out_ids ||
        (lists->ntotal > 0 && !lists->codes))
        return fail(ctx, PQ_EINVAL, "ivf_quick_adc_search: null pointer");
    if (!aligned16(lists->codes)) return fail(ctx, PQ_EINVAL, "ivf_quick_adc_search: codes must be 16-byte aligned");
    return launch_ivf(ctx, lists, codebooks, m, k, PQ_CODES_U4_PACKED, queries, nq, nprobe, topk, out_dist, out_ids, probe_out,
                      init, kprime);
}

}  // extern "C"
