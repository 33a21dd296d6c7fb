// Encoder of the product quantizer (Section 2.3.1): a vector x is cut into m sub-vectors and
// sub-vector x^j is replaced by the index of the closest centroid of codebook j,
//   code_j(x) = argmin_i || x^j - C^j[i] ||^2          (ties: smallest i).
// The distances come from the expanded form ||x||^2 + ||c||^2 - 2<x, c> with the inner products
// on the fp64 matrix cores, as in the Tables step: everything in double, entries that cancel
// almost completely recomputed from the differences, so that the decision is the one the plain
// double-precision definition takes.
#include "pq_internal.h"

namespace pq {

constexpr int ER = 64;   // vectors per block (4 waves x 16 rows)
constexpr int EC = 64;   // centroids per tile
constexpr int EK = 16;   // dimensions per LDS chunk

// One block of 256 threads encodes 64 vectors, one sub-space after the other.  Wave w owns rows
// 16 w .. 16 w + 15 and all 64 centroids of a tile (four 16 x 16 MFMA tiles), so the arg-min of a
// row is reduced inside one wave.
__global__ __launch_bounds__(256) void pq_encode_kernel(const float *__restrict__ x, const float *__restrict__ codebooks,
                                                        int64_t n, int d, int m, int k, int packed,
                                                        uint8_t *__restrict__ codes) {
    typedef double double4_t __attribute__((ext_vector_type(4)));
    __shared__ double xs[EK][ER + 2];
    __shared__ double cs[EK][EC + 2];
    __shared__ double nx[ER], nc[EC];
    const int ds = d / m;
    const int64_t r0 = (int64_t)blockIdx.x * ER;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = tid >> 2, lk = (tid & 3) * 4;   // staging: 4 consecutive dimensions of one row
    const bool xrow_ok = r0 + lrow < n;
    const int code_bytes = packed ? m / 2 : m;
    int prev_idx[4] = {0, 0, 0, 0};   // packed codes: index of the even sub-space, kept for the odd one

    for (int j = 0; j < m; ++j) {
        const float *xrow = x + (size_t)(xrow_ok ? r0 + lrow : 0) * d + (size_t)j * ds;
        const float *cbase = codebooks + (size_t)j * k * ds;
        double best[4];
        int best_idx[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) { best[v] = __builtin_inf(); best_idx[v] = 0; }

        for (int c0 = 0; c0 < k; c0 += EC) {
            const bool crow_ok = c0 + lrow < k;
            const float *crow = cbase + (size_t)(crow_ok ? c0 + lrow : 0) * ds;
            double4_t acc[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = (double4_t){0.0, 0.0, 0.0, 0.0};
            double norm = 0.0;   // thread t < 64: ||x_t||^2, thread 64 + t: ||c_t||^2
            for (int k0 = 0; k0 < ds; k0 += EK) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = k0 + lk + i;
                    xs[lk + i][lrow] = xrow_ok && t < ds ? (double)xrow[t] : 0.0;
                    cs[lk + i][lrow] = crow_ok && t < ds ? (double)crow[t] : 0.0;
                }
                __syncthreads();
                if (tid < ER + EC) {
                    const double(*src)[ER + 2] = tid < ER ? xs : cs;
                    const int r = tid & (ER - 1);
#pragma unroll
                    for (int kk = 0; kk < EK; ++kk) norm += src[kk][r] * src[kk][r];
                }
#pragma unroll
                for (int ks = 0; ks < EK; ks += 4) {
                    const double a = xs[ks + (lane >> 4)][wave * 16 + (lane & 15)];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const double b = cs[ks + (lane >> 4)][t * 16 + (lane & 15)];
                        acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[t], 0, 0, 0);
                    }
                }
                __syncthreads();
            }
            if (tid < ER) nx[tid] = norm;
            else if (tid < ER + EC) nc[tid - ER] = norm;
            __syncthreads();
            // lane l holds rows l / 16 + 4 v of column l % 16 of each 16 x 16 tile
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = wave * 16 + (lane >> 4) + 4 * v;
                double dmin = __builtin_inf();
                int imin = 0x7fffffff;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int c = t * 16 + (lane & 15), ci = c0 + c;
                    if (ci >= k) continue;
                    const double sum = nx[r] + nc[c];
                    double dist = sum - 2.0 * acc[t][v];
                    if (dist < 1e-9 * sum && r0 + r < n) {   // nearly complete cancellation: the plain definition
                        dist = 0.0;
                        const float *xr = x + (size_t)(r0 + r) * d + (size_t)j * ds, *cr = cbase + (size_t)ci * ds;
                        for (int t2 = 0; t2 < ds; ++t2) {
                            const double df = (double)xr[t2] - (double)cr[t2];
                            dist += df * df;
                        }
                    }
                    if (dist < dmin) { dmin = dist; imin = ci; }   // columns ascend with t: the first minimum stays
                }
                // smallest (distance, index) over the 16 lanes that share the row
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) {
                    const double od = __shfl_xor(dmin, o);
                    const int oi = __shfl_xor(imin, o);
                    if (od < dmin || (od == dmin && oi < imin)) { dmin = od; imin = oi; }
                }
                if (dmin < best[v]) { best[v] = dmin; best_idx[v] = imin; }   // tiles ascend: ties keep the smaller index
            }
            __syncthreads();
        }
        if ((lane & 15) == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = r0 + wave * 16 + (lane >> 4) + 4 * v;
                if (row >= n) continue;
                if (!packed) {
                    codes[(size_t)row * code_bytes + j] = (uint8_t)best_idx[v];
                } else if (j & 1) {
                    codes[(size_t)row * code_bytes + (j >> 1)] = (uint8_t)(prev_idx[v] | (best_idx[v] << 4));
                } else {
                    prev_idx[v] = best_idx[v];
                }
            }
        }
    }
}

int launch_encode(pq_ctx *ctx, const float *vectors, const float *codebooks, int64_t n, int d, int m, int k, int cf,
                  uint8_t *codes) {
    if (n == 0) return PQ_OK;
    const int64_t nblocks = (n + ER - 1) / ER;
    if (nblocks > 0x7fffffff) return fail(ctx, PQ_EUNSUPPORTED, "encode: more than 2^37 vectors");
    pq_encode_kernel<<<(unsigned)nblocks, 256, 0, ctx->stream>>>(vectors, codebooks, n, d, m, k,
                                                                 cf == PQ_CODES_U4_PACKED ? 1 : 0, codes);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

}  // namespace pq
