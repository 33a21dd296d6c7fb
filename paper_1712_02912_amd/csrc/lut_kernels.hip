// Tables step (Eq. (tables) of Section 2.3.3), 8-bit table quantisation (Sections 4.2.4,
// 5.2.1, 6.3 Step 1.2), the qmax pre-scan and the rerank pass of the two-pass search
// (Section 6.2.3, Alg. 5).
#include "pq_internal.h"
#include "topk_device.h"

namespace pq {


// ------------------------------------------------------------------------------------------
// Direct form  D[q][j][i] = sum_t (y[q][j*dsub+t] - C[j][i][t])^2  in f32.  All terms are
// non-negative, so the relative error is bounded by about (dsub+1) * 2^-24.
// Block = (tile of 16 queries) x (one sub-space j) x (tile of 64 centroids): the centroid
// tile and the query sub-vectors are staged in LDS in slabs of 32 dimensions.
constexpr int LUT_TQ = 16, LUT_TC = 64, LUT_TD = 32;

__global__ __launch_bounds__(256) void build_luts_kernel(const float *__restrict__ queries,
                                                         const float *__restrict__ codebooks, int nq, int d, int m,
                                                         int k, float *__restrict__ luts) {
    __shared__ float sc[LUT_TC][LUT_TD + 1];
    __shared__ float sy[LUT_TQ][LUT_TD + 1];
    const int dsub = d / m;
    const int j = blockIdx.y;
    const int c0 = blockIdx.x * LUT_TC;
    const int q0 = blockIdx.z * LUT_TQ;
    const int ci = threadIdx.x & 63;        // centroid within tile
    const int qi = threadIdx.x >> 6;        // 0..3: this thread handles queries qi, qi+4, qi+8, qi+12
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < dsub; t0 += LUT_TD) {
        const int td = dsub - t0 < LUT_TD ? dsub - t0 : LUT_TD;
        for (int e = threadIdx.x; e < LUT_TC * LUT_TD; e += 256) {
            const int c = e / LUT_TD, t = e % LUT_TD;
            sc[c][t] = (c0 + c < k && t < td) ? codebooks[((size_t)j * k + c0 + c) * dsub + t0 + t] : 0.f;
        }
        for (int e = threadIdx.x; e < LUT_TQ * LUT_TD; e += 256) {
            const int q = e / LUT_TD, t = e % LUT_TD;
            sy[q][t] = (q0 + q < nq && t < td) ? queries[(size_t)(q0 + q) * d + j * dsub + t0 + t] : 0.f;
        }
        __syncthreads();
        for (int t = 0; t < td; ++t) {
            const float c = sc[ci][t];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float diff = sy[qi + 4 * r][t] - c;
                acc[r] = fmaf(diff, diff, acc[r]);
            }
        }
        __syncthreads();
    }
    if (c0 + ci < k) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int q = q0 + qi + 4 * r;
            if (q < nq) luts[((size_t)q * m + j) * k + c0 + ci] = acc[r];
        }
    }
}

// Matrix-core form of the Tables step (Eq. (tables)) for sub-vectors of 8 dimensions and more:
//   ||y - c||^2 = ||y||^2 + ||c||^2 - 2 <y, c>,
// with the inner products of 64 queries x 64 centroids per block on the fp64 matrix cores
// (v_mfma_f64_16x16x4f64) and the norms accumulated next to them, everything in double.  Double
// is what makes the expanded form safe: in fp32 the cancellation between the three terms costs
// more than the 1e-5 this path may lose, in double it costs nothing that survives the final
// rounding to float.  Entries that cancel almost completely (query on top of a centroid) are
// recomputed from the differences, so that exact zeros stay exact.
// Block: 256 threads = 4 waves in a 2 x 2 grid, each wave 32 x 32 outputs as 2 x 2 MFMA tiles.
constexpr int MT = 64;   // queries and centroids per block
// MK: dimensions per LDS chunk (16 is used; 32 measured slower on every configured shape)
// DOT: write the inner products themselves (out[q][c] = <y_q, c>, used for R x) instead of distances.
template <bool DOT, int MK>
__global__ __launch_bounds__(256) void build_luts_mfma_kernel(const float *__restrict__ queries,
                                                              const float *__restrict__ codebooks, int nq, int d, int m,
                                                              int k, float *__restrict__ luts) {
    typedef double double4_t __attribute__((ext_vector_type(4)));
    constexpr int MDPT = MK / 4;   // dimensions of a row that one thread stages (four threads per row)
    __shared__ double ys[MK][MT + 2];
    __shared__ double cs[MK][MT + 2];
    __shared__ double ny[MT], nc[MT];
    const int ds = d / m;
    const int j = blockIdx.z, q0 = blockIdx.y * MT, c0 = blockIdx.x * MT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const float *ybase = queries + (size_t)j * ds;                 // row q: + q * d
    const float *cbase = codebooks + (size_t)j * k * ds;           // row c: + c * ds
    double4_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = (double4_t){0.0, 0.0, 0.0, 0.0};
    double norm = 0.0;   // thread t < 64: ||y_t||^2, thread 64 + t: ||c_t||^2
    const int lrow = tid >> 2, lk = (tid & 3) * MDPT;   // this thread stages MDPT consecutive dimensions of one row
    const bool yrow_ok = q0 + lrow < nq, crow_ok = c0 + lrow < k;
    const float *yrow = ybase + (size_t)(yrow_ok ? q0 + lrow : 0) * d;
    const float *crow = cbase + (size_t)(crow_ok ? c0 + lrow : 0) * ds;
    const bool vec = (ds & 3) == 0 && (d & 3) == 0;   // rows start on 16-byte boundaries
    // the two chunks after the one being multiplied are on their way or wait in registers
    float yv[2][MDPT], cv[2][MDPT];
    auto fetch = [&](int k0, float (&yr)[MDPT], float (&cr)[MDPT]) {
        const int t = k0 + lk;
        if (vec && t + MDPT <= ds) {
#pragma unroll
            for (int v = 0; v < MDPT / 4; ++v) {
                const float4 a = *reinterpret_cast<const float4 *>(yrow + t + 4 * v), b = *reinterpret_cast<const float4 *>(crow + t + 4 * v);
                yr[4 * v] = a.x; yr[4 * v + 1] = a.y; yr[4 * v + 2] = a.z; yr[4 * v + 3] = a.w;
                cr[4 * v] = b.x; cr[4 * v + 1] = b.y; cr[4 * v + 2] = b.z; cr[4 * v + 3] = b.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < MDPT; ++i) {
                yr[i] = t + i < ds ? yrow[t + i] : 0.f;
                cr[i] = t + i < ds ? crow[t + i] : 0.f;
            }
        }
    };
    // one chunk of MK dimensions: registers -> LDS (as doubles), refill the registers with the
    // chunk two steps ahead, norms, products
    auto chunk = [&](int k0, float (&yr)[MDPT], float (&cr)[MDPT]) {
#pragma unroll
        for (int i = 0; i < MDPT; ++i) {
            ys[lk + i][lrow] = yrow_ok ? (double)yr[i] : 0.0;
            cs[lk + i][lrow] = crow_ok ? (double)cr[i] : 0.0;
        }
        __syncthreads();
        if (k0 + 2 * MK < ds) fetch(k0 + 2 * MK, yr, cr);
        if (!DOT && tid < 2 * MT) {
            const double(*src)[MT + 2] = tid < MT ? ys : cs;
            const int r = tid & (MT - 1);
#pragma unroll
            for (int kk = 0; kk < MK; ++kk) norm += src[kk][r] * src[kk][r];
        }
#pragma unroll
        for (int ks = 0; ks < MK; ks += 4) {
            double a[2], b[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                a[t] = ys[ks + (lane >> 4)][wy * 32 + t * 16 + (lane & 15)];
                b[t] = cs[ks + (lane >> 4)][wx * 32 + t * 16 + (lane & 15)];
            }
#pragma unroll
            for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
        }
        __syncthreads();
    };
    fetch(0, yv[0], cv[0]);
    if (MK < ds) fetch(MK, yv[1], cv[1]);
    for (int k0 = 0; k0 < ds; k0 += 2 * MK) {
        chunk(k0, yv[0], cv[0]);
        if (k0 + MK < ds) chunk(k0 + MK, yv[1], cv[1]);
    }
    if (tid < MT) ny[tid] = norm;
    else if (tid < 2 * MT) nc[tid - MT] = norm;
    __syncthreads();
    // lane l of an MFMA tile holds rows l / 16 + 4 * v (v = 0..3) of column l % 16
#pragma unroll
    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = wy * 32 + ta * 16 + (lane >> 4) + 4 * v, c = wx * 32 + tb * 16 + (lane & 15);
                const int q = q0 + r, ci = c0 + c;
                if (q >= nq || ci >= k) continue;
                if (DOT) {
                    luts[((size_t)q * m + j) * k + ci] = (float)acc[ta][tb][v];
                    continue;
                }
                const double sum = ny[r] + nc[c];
                double dist = sum - 2.0 * acc[ta][tb][v];
                if (dist < 1e-9 * sum) {   // nearly complete cancellation: take the plain definition
                    dist = 0.0;
                    for (int t = 0; t < ds; ++t) {
                        const double df = (double)ybase[(size_t)q * d + t] - (double)cbase[(size_t)ci * ds + t];
                        dist += df * df;
                    }
                }
                luts[((size_t)q * m + j) * k + ci] = (float)dist;
            }
}

int launch_build_luts(pq_ctx *ctx, const float *queries, const float *codebooks, int nq, int d, int m, int k,
                      float *luts) {
    if (d / m >= 8 && opt_int(ctx, PQ_OPT_LUT_MFMA, 1) != 0) {
        dim3 mgrid((k + MT - 1) / MT, (nq + MT - 1) / MT, m);
        if (mgrid.y > 65535 || mgrid.z > 65535) return fail(ctx, PQ_EUNSUPPORTED, "build_luts: m or nq/64 above 65535");
        build_luts_mfma_kernel<false, 16><<<mgrid, 256, 0, ctx->stream>>>(queries, codebooks, nq, d, m, k, luts);
        PQ_HIP(ctx, hipGetLastError());
        return PQ_OK;
    }
    dim3 grid((k + LUT_TC - 1) / LUT_TC, m, (nq + LUT_TQ - 1) / LUT_TQ);
    if (grid.y > 65535 || grid.z > 65535) return fail(ctx, PQ_EUNSUPPORTED, "build_luts: m or nq/16 above 65535");
    build_luts_kernel<<<grid, 256, 0, ctx->stream>>>(queries, codebooks, nq, d, m, k, luts);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// Rotation of optimized product quantization (Section 2.3.4, OPQ: opq(x) = pq(R x)):
// out[p][r] = sum_t R[r][t] * x[p][t] -- the inner products of the vectors with the rows of R, on
// the fp64 matrix cores, rounded once to float.
int launch_rotate(pq_ctx *ctx, const float *vectors, const float *rot, int64_t n, int d, float *out) {
    const int64_t ytiles = (n + MT - 1) / MT;
    if (ytiles > 65535 * 64) return fail(ctx, PQ_EUNSUPPORTED, "rotate: more than 2^28 vectors per call");
    // the y dimension of a grid is limited to 65535 blocks: long inputs go in slices of rows
    for (int64_t t0 = 0; t0 < ytiles; t0 += 65535) {
        const int64_t rows0 = t0 * MT;
        const int64_t rows = (n - rows0) < (int64_t)65535 * MT ? (n - rows0) : (int64_t)65535 * MT;
        dim3 grid((d + MT - 1) / MT, (unsigned)((rows + MT - 1) / MT), 1);
        build_luts_mfma_kernel<true, 16><<<grid, 256, 0, ctx->stream>>>(vectors + (size_t)rows0 * d, rot, (int)rows, d, 1, d,
                                                                    out + (size_t)rows0 * d);
        PQ_HIP(ctx, hipGetLastError());
    }
    return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// One block per query.  The float operation sequence (subtract, divide, subtract, multiply,
// floor, clamp) is fixed by the definition so that the bytes are reproducible.
__global__ __launch_bounds__(256) void quantize_luts_kernel(const float *__restrict__ luts, int per,
                                                            const float *__restrict__ qmax,
                                                            uint8_t *__restrict__ qluts, float *qmin_out,
                                                            float *scale_out) {
    __shared__ float red[4];
    const int q = blockIdx.x;
    const float *D = luts + (size_t)q * per;
    float mn = __builtin_inff();
    bool has_nan = false;
    for (int e = threadIdx.x; e < per; e += 256) {
        const float v = D[e];
        mn = v < mn ? v : mn;
    }
    for (int o = 32; o > 0; o >>= 1) {
        const float other = __shfl_xor(mn, o);
        mn = other < mn ? other : mn;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mn;
    __syncthreads();
    float qmin = red[0];
    for (int w = 1; w < 4; ++w) qmin = red[w] < qmin ? red[w] : qmin;
    (void)has_nan;
    const float range = __fsub_rn(qmax[q], qmin);
    float scale = 0.f;
    if (range > 0.f && range < __builtin_inff()) scale = __fdiv_rn(255.0f, range);
    for (int e = threadIdx.x; e < per; e += 256) {
        const float t = __fmul_rn(__fsub_rn(D[e], qmin), scale);
        qluts[(size_t)q * per + e] = t >= 255.0f ? (uint8_t)255 : (uint8_t)floorf(t);
    }
    if (threadIdx.x == 0) {
        if (qmin_out) qmin_out[q] = qmin;
        if (scale_out) scale_out[q] = scale;
    }
}

int launch_quantize_luts(pq_ctx *ctx, const float *luts, int nq, int m, int k, const float *qmax, uint8_t *qluts,
                         float *qmin_out, float *scale_out) {
    if (nq == 0) return PQ_OK;
    quantize_luts_kernel<<<nq, 256, 0, ctx->stream>>>(luts, m * k, qmax, qluts, qmin_out, scale_out);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// Float ADC of one stored code with one query's tables (global memory), Eq. (adc1).
__device__ __forceinline__ float adc_one(const uint8_t *code, int cf, const float *lut, int m, int k) {
    const int cb = cf == PQ_CODES_U4_PACKED ? m / 2 : m;
    // codes of 8 or 16 bytes (every configured shape) aligned to their size come in one load
    uint32_t w[4] = {0, 0, 0, 0};
    const bool words = (cb == 8 || cb == 16) && ((uintptr_t)code & (uintptr_t)(cb - 1)) == 0;
    if (words && cb == 8) {
        const uint2 c = *reinterpret_cast<const uint2 *>(code);
        w[0] = c.x; w[1] = c.y;
    } else if (words) {
        const uint4 c = *reinterpret_cast<const uint4 *>(code);
        w[0] = c.x; w[1] = c.y; w[2] = c.z; w[3] = c.w;
    }
    float dist = 0.f;
    for (int j = 0; j < m; ++j) {
        const int pos = cf == PQ_CODES_U4_PACKED ? j >> 1 : j;
        const uint32_t byte = words ? (w[(pos >> 2) & 3] >> (8 * (pos & 3))) & 255u : code[pos];
        int idx;
        if (cf == PQ_CODES_U4_PACKED) idx = (j & 1) ? (byte >> 4) : (byte & 15u);
        else idx = byte;
        if (idx < k) dist += lut[(size_t)j * k + idx];
    }
    return dist;
}

// The query's tables copied behind the sort keys in LDS when they fit there (`staged` = their number of floats, else
// 0): every code then looks its m entries up in LDS instead of device memory.  Returns the tables to use.
__device__ __forceinline__ const float *stage_tables(const float *lut, float *lds, int staged) {
    if (staged == 0) return lut;
    for (int i = threadIdx.x; i < staged; i += blockDim.x) lds[i] = lut[i];
    __syncthreads();
    return lds;
}
// dynamic LDS of the two kernels below: n2 sort keys and, if both fit into 48 KB, the query's tables
static inline int staged_floats(int n2, int m, int k) {
    return (size_t)n2 * 8 + (size_t)m * k * 4 <= 48 * 1024 ? m * k : 0;
}

// One block per query: distances of the first `cnt` codes (cnt <= 4096) as ordered 32-bit values in LDS,
// then the kq-th smallest of them by radix selection (1 <= kq <= cnt).
__global__ __launch_bounds__(1024) void qmax_prescan_kernel(const uint8_t *__restrict__ codes, int cnt, int cb,
                                                           int cf, const float *__restrict__ luts, int m, int k,
                                                           int kq, int n2, int staged, float *qmax_out) {
    extern __shared__ uint64_t skeys[];
    __shared__ uint32_t bins[256];
    __shared__ uint32_t state[2];
    const int q = blockIdx.x, tid = threadIdx.x;
    uint32_t *ords = reinterpret_cast<uint32_t *>(skeys);
    const float *lut = stage_tables(luts + (size_t)q * m * k, reinterpret_cast<float *>(skeys + n2), staged);
    for (int i = tid; i < cnt; i += blockDim.x) ords[i] = f32_to_ord(adc_one(codes + (size_t)i * cb, cf, lut, m, k));
    __syncthreads();
    const uint32_t kth = block_kth_smallest_u32(ords, cnt, (uint32_t)kq, bins, state);
    if (tid == 0) qmax_out[q] = ord_to_f32(kth);
}

int launch_qmax_prescan(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const float *luts, int nq, int m,
                        int k, int init, int kq, float *qmax_out) {
    const int cnt = (int)(init < n ? init : n);
    if (kq > cnt) kq = cnt;
    int n2 = 64;
    while (n2 < cnt) n2 <<= 1;
    const int cb = cf == PQ_CODES_U4_PACKED ? m / 2 : m;
    const int staged = staged_floats(n2, m, k);
    qmax_prescan_kernel<<<nq, n2 >= 2048 ? 1024 : (n2 >= 1024 ? 512 : 256), (size_t)n2 * 8 + (size_t)staged * 4, ctx->stream>>>(codes, cnt, cb, cf, luts, m, k, kq, n2, staged, qmax_out);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// One block per query: float ADC of the candidates, sort by (distance, id), write topk.
__global__ __launch_bounds__(1024) void rerank_kernel(const uint8_t *__restrict__ codes, int64_t n, int cb, int cf,
                                                     const float *__restrict__ luts, int m, int k,
                                                     const int64_t *__restrict__ cand, int ncand, int n2, int topk, int staged,
                                                     float *out_dist, int64_t *out_ids) {
    extern __shared__ uint64_t skeys[];
    const int q = blockIdx.x;
    const float *lut = stage_tables(luts + (size_t)q * m * k, reinterpret_cast<float *>(skeys + n2), staged);
    for (int i = threadIdx.x; i < n2; i += blockDim.x) {
        uint64_t key = KEY_EMPTY;
        if (i < ncand) {
            const int64_t id = cand[(size_t)q * ncand + i];
            if (id >= 0 && id < n)
                key = ((uint64_t)f32_to_ord(adc_one(codes + (size_t)id * cb, cf, lut, m, k)) << 32) | (uint32_t)id;
        }
        skeys[i] = key;
    }
    block_bitonic_sort(skeys, n2);
    for (int i = threadIdx.x; i < topk; i += blockDim.x) {
        const uint64_t key = skeys[i];
        const bool empty = key == KEY_EMPTY;
        out_dist[(size_t)q * topk + i] = empty ? __builtin_inff() : ord_to_f32((uint32_t)(key >> 32));
        out_ids[(size_t)q * topk + i] = empty ? -1 : (int64_t)(uint32_t)key;
    }
}

int launch_rerank(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const float *luts, int nq, int m, int k,
                  const int64_t *cand, int ncand, int topk, float *out_dist, int64_t *out_ids) {
    int n2 = 64;
    while (n2 < ncand) n2 <<= 1;
    const int cb = cf == PQ_CODES_U4_PACKED ? m / 2 : m;
    if (nq == 0) return PQ_OK;
    const int staged = staged_floats(n2, m, k);
    rerank_kernel<<<nq, n2 >= 2048 ? 1024 : (n2 >= 1024 ? 512 : 256), (size_t)n2 * 8 + (size_t)staged * 4, ctx->stream>>>(codes, n, cb, cf, luts, m, k, cand, ncand, n2, topk,
                                                                                   staged, out_dist, out_ids);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

}  // namespace pq
