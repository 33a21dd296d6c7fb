// Tables step (Eq. (tables) of Section 2.3.3), 8-bit table quantisation (Sections 4.2.4,
// 5.2.1, 6.3 Step 1.2), the qmax pre-scan and the rerank pass of the two-pass search
// (Section 6.2.3, Alg. 5).
#include "pq_internal.h"
#include "topk_device.h"

namespace pq {


// ------------------------------------------------------------------------------------------
// Direct form  D[q][j][i] = sum_t (y[q][j*dsub+t] - C[j][i][t])^2, the differences, their squares and
// the sum in double, term by term in the order of t, rounded to f32 once: the value of the plain definition.
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
    double acc[4] = {0.0, 0.0, 0.0, 0.0};   // differences, squares and their sum in double, term by term: the plain definition
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
                const double diff = (double)sy[qi + 4 * r][t] - (double)c;
                acc[r] = __dadd_rn(acc[r], __dmul_rn(diff, diff));
            }
        }
        __syncthreads();
    }
    if (c0 + ci < k) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int q = q0 + qi + 4 * r;
            if (q < nq) luts[((size_t)q * m + j) * k + c0 + ci] = (float)acc[r];
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

// The same contraction for launches with many tiles: 128 queries x 128 centroids per tile, each of
// the 4 waves 64 x 64 outputs as 4 x 4 MFMA tiles, so that one operand read from LDS feeds four
// matrix instructions instead of two and every operand byte fetched from memory feeds twice the
// arithmetic.  On this chip the fp64 matrix instructions and the ordinary vector instructions of a
// SIMD take turns (a lone wave issues one v_mfma_f64_16x16x4f64 every 64 cycles, and the rate of
// two waves drops by what their other vector instructions take), so the kernel is laid out to
// issue few of those:
//  - PRE: a pass over the operands beforehand writes them as doubles (rows padded with zeros to
//    a multiple of 16 dimensions, the centroids doubled) together with minus their squared
//    norms; staging a chunk is then loads and LDS stores only, the sums start at
//    -(||y||^2 + ||c||^2) instead of zero and end at minus the distance.  Without PRE (few dimensions per sub-vector, where that pass
//    would cost more than it saves) chunks are converted and the norms added up while staging.
//  - rows past the end of an operand are staged as whatever row 0 holds: they only reach outputs
//    that are never written.
//  - the test for nearly complete cancellation is made on the floats, four at a time, against one
//    bound per tile that no exact bound exceeds (entries it marks needlessly still get the plain
//    definition, which is never the less accurate of the two).
// Operands lie in LDS as [row][dimension] doubles with a row stride of 18: the 16 rows and 2
// dimensions that half a wave reads at once then fall into 64 different banks.  Two LDS buffers
// alternate (one barrier per chunk of 16 dimensions, placed so that the matrix cores have work
// queued while the waves of a block meet); the chunk after the one in LDS is on its way from
// memory into registers meanwhile.
// Two blocks per compute unit stay for the whole launch and take tiles in turn; the first chunk
// of a block's next tile is requested while its current tile is still being multiplied, and the
// results leave through LDS as whole rows of 64 floats per wave with stores that nothing waits for.
// Tiles are numbered so that the 8 dies of the chip (which take consecutive block ids in turn and
// have a cache each) work on separate bands of query tiles, and the tiles in flight on one die form
// a patch of 8 query tiles x 8 centroid tiles whose operands stay in that cache.
constexpr int MT2 = 128, MK2 = 16, LS2 = MK2 + 2, OS2 = 72;   // tile, chunk, operand row stride (doubles), output row stride (floats)
constexpr int GROUP_Y2 = 8;                                    // query tiles per patch

struct Tile128 {
    int j, q0, c0;
};

__device__ __forceinline__ Tile128 tile128_of(int seq, int tiles_x, int tiles_y) {
    const int per_j = tiles_x * tiles_y;
    const int j = seq / per_j, rj = seq - j * per_j;
    const int patch = rj / (GROUP_Y2 * tiles_x), rp = rj - patch * (GROUP_Y2 * tiles_x);
    const int ty0 = patch * GROUP_Y2, gy = tiles_y - ty0 < GROUP_Y2 ? tiles_y - ty0 : GROUP_Y2;
    return Tile128{j, (ty0 + rp % gy) * MT2, (rp / gy) * MT2};
}

struct Mfma128Args {
    const float *queries, *codebooks;   // [nq][d], [m][k][ds]
    const double *yd, *cd;              // PRE: [m][nq_pad][dsp], [m][k_pad][dsp]; for distances cd holds 2 c
    const double *nyg, *ncg;            // PRE: minus the squared norms, [m][nq_pad], [m][k_pad]
    const float *ymax, *cmax;           // PRE: the largest squared norm of each block of prep128_kernel, as floats (rounded up)
    int nymax, ncmax;
    float *out;                         // [nq][m][k]
    int nq, d, m, k, ds, dsp;
    int nq_pad, k_pad;                  // PRE: rows per sub-space of yd and cd (whole tiles, the padding is zeros)
    int tiles_x, tiles_y, total;
};

// Operands as doubles with their squared norms, one row of `ds` floats (at src + row * stride, for
// sub-space j at + j * jstride) per 16 lanes: dst[j * rows_pad + row][dsp] = scale * row, norms[j * rows_pad + row]
// = norm_sign * ||row||^2; rows from `rows` up to rows_pad and dimensions from `ds` up to dsp are zeros.
__global__ __launch_bounds__(256) void prep128_kernel(const float *__restrict__ src, size_t stride, size_t jstride, int rows,
                                                      int rows_pad, int m, int ds, int dsp, double *__restrict__ dst,
                                                      double *__restrict__ norms, float *__restrict__ block_max,
                                                      double scale, double norm_sign) {
    __shared__ float wmax_s[4];
    typedef double double2_t __attribute__((ext_vector_type(2)));
    const size_t g = ((size_t)blockIdx.x * 256 + threadIdx.x) >> 4;   // row over all sub-spaces
    const int l = threadIdx.x & 15;
    const bool inside = g < (size_t)rows_pad * m;
    const int j = inside ? (int)(g / rows_pad) : 0, row = inside ? (int)(g - (size_t)j * rows_pad) : 0;
    const bool ok = inside && row < rows;
    const float *r = src + (size_t)j * jstride + (size_t)(ok ? row : 0) * stride;
    double norm = 0.0;
    for (int t = l * 4; t < dsp; t += 64) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ok && t < ds) v = *reinterpret_cast<const float4 *>(r + t);   // ds is a multiple of 4
        const double a = v.x, b = v.y, c = v.z, e = v.w;
        if (inside) {
            double *o = dst + g * dsp + t;
            *reinterpret_cast<double2_t *>(o) = (double2_t){scale * a, scale * b};
            *reinterpret_cast<double2_t *>(o + 2) = (double2_t){scale * c, scale * e};
        }
        norm += a * a; norm += b * b; norm += c * c; norm += e * e;
    }
    for (int o = 8; o > 0; o >>= 1) norm += __shfl_xor(norm, o);
    if (inside && l == 0) norms[g] = norm_sign * norm;
    // the largest norm of the block's 16 rows, as a float that is not below it
    float fm = (float)norm * 1.0000002f;
    for (int o = 32; o >= 16; o >>= 1) fm = fmaxf(fm, __shfl_xor(fm, o));
    if ((threadIdx.x & 63) == 0) wmax_s[threadIdx.x >> 6] = fm;
    __syncthreads();
    if (threadIdx.x == 0) block_max[blockIdx.x] = fmaxf(fmaxf(wmax_s[0], wmax_s[1]), fmaxf(wmax_s[2], wmax_s[3]));
}

template <bool DOT, bool PRE>
__global__ __launch_bounds__(256, 2) void build_luts_mfma128_kernel(const Mfma128Args A) {
    typedef double double4_t __attribute__((ext_vector_type(4)));
    typedef double double2_t __attribute__((ext_vector_type(2)));
    __shared__ __align__(16) double lds[2 * 2 * MT2 * LS2];   // [buffer][y | c][row][LS2]
    __shared__ double ny[MT2], nc[MT2];
    __shared__ float wave_max[8];
    static_assert(4 * 64 * OS2 * sizeof(float) <= sizeof(double) * 2 * 2 * MT2 * LS2, "output staging fits the operand buffers");
    const int nq = A.nq, d = A.d, m = A.m, k = A.k, ds = A.ds;
    // die e of 8 takes the tiles [e * per_die, (e + 1) * per_die), its blocks in turn
    const int per_die = (A.total + 7) >> 3, blocks_per_die = gridDim.x >> 3;
    const int die = blockIdx.x & 7;
    int local = blockIdx.x >> 3;   // tile of this block within the die's share
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const int nchunks = PRE ? A.dsp / MK2 : (ds + MK2 - 1) / MK2;
    auto has_tile = [&](int l) { return l < per_die && die * per_die + l < A.total; };
    if (!has_tile(local)) return;

    // What a thread fetches and stages.  PRE: 8 threads per row (2 doubles each, a whole 128-byte
    // line per row and request), rows tid / 8 + 32 * pass, pass 0..3; the converted operands are
    // padded with rows of zeros to whole tiles.  Otherwise 4 threads per row (4 floats each), rows
    // tid / 4 + 64 * pass, pass 0..1, and row 0 stands in for rows past the end.
    constexpr int NPASS = PRE ? 4 : 2, ROWS_PER_PASS = MT2 / NPASS;
    const int srow = PRE ? tid >> 3 : tid >> 2, sk = PRE ? (tid & 7) * 2 : (tid & 3) * 4;
    struct Rows {
        const void *y[PRE ? 1 : 2], *c[PRE ? 1 : 2];
    };
    auto rows_of = [&](const Tile128 &t) {
        Rows r;
        if constexpr (PRE) {
            r.y[0] = A.yd + ((size_t)t.j * A.nq_pad + t.q0 + srow) * A.dsp + sk;
            r.c[0] = A.cd + ((size_t)t.j * A.k_pad + t.c0 + srow) * A.dsp + sk;
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int row = p * ROWS_PER_PASS + srow;
                const int qr = t.q0 + row < nq ? t.q0 + row : 0, cr = t.c0 + row < k ? t.c0 + row : 0;
                r.y[p] = A.queries + (size_t)t.j * ds + (size_t)qr * d + sk;
                r.c[p] = A.codebooks + ((size_t)t.j * k + cr) * ds + sk;
            }
        }
        return r;
    };
    // the chunk after the one being multiplied, [y | c][pass]: 4 floats, or 2 doubles with PRE
    float4 rf[2][PRE ? 1 : 2];
    double2_t rd[2][PRE ? 4 : 1];
    // rows start on 16-byte boundaries and hold a multiple of 4 dimensions (the launcher sees to
    // it), so a group of 4 dimensions lies inside a row or past its end as a whole
    auto fetch = [&](const Rows &r, int k0) {
        if constexpr (PRE) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                rd[0][p] = *reinterpret_cast<const double2_t *>((const double *)r.y[0] + (size_t)p * ROWS_PER_PASS * A.dsp + k0);
                rd[1][p] = *reinterpret_cast<const double2_t *>((const double *)r.c[0] + (size_t)p * ROWS_PER_PASS * A.dsp + k0);
            }
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                rf[0][p] = rf[1][p] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k0 + sk < ds) {
                    rf[0][p] = *reinterpret_cast<const float4 *>((const float *)r.y[p] + k0);
                    rf[1][p] = *reinterpret_cast<const float4 *>((const float *)r.c[p] + k0);
                }
            }
        }
    };
    double norm_y[2] = {0.0, 0.0}, norm_c[2] = {0.0, 0.0};   // without PRE: this thread's part of the squared norms of its rows
    auto stage = [&](int buf) {
        double *yd = lds + ((size_t)(buf * 2 + 0) * MT2 + srow) * LS2 + sk;
        double *cd = lds + ((size_t)(buf * 2 + 1) * MT2 + srow) * LS2 + sk;
        if constexpr (PRE) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                *reinterpret_cast<double2_t *>(yd + p * ROWS_PER_PASS * LS2) = rd[0][p];
                *reinterpret_cast<double2_t *>(cd + p * ROWS_PER_PASS * LS2) = rd[1][p];
            }
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const double y0 = rf[0][p].x, y1 = rf[0][p].y, y2 = rf[0][p].z, y3 = rf[0][p].w;
                const double c0v = rf[1][p].x, c1v = rf[1][p].y, c2v = rf[1][p].z, c3v = rf[1][p].w;
                *reinterpret_cast<double2_t *>(yd + p * ROWS_PER_PASS * LS2) = (double2_t){y0, y1};
                *reinterpret_cast<double2_t *>(yd + p * ROWS_PER_PASS * LS2 + 2) = (double2_t){y2, y3};
                *reinterpret_cast<double2_t *>(cd + p * ROWS_PER_PASS * LS2) = (double2_t){c0v, c1v};
                *reinterpret_cast<double2_t *>(cd + p * ROWS_PER_PASS * LS2 + 2) = (double2_t){c2v, c3v};
                if (!DOT) {
                    norm_y[p] += y0 * y0; norm_y[p] += y1 * y1; norm_y[p] += y2 * y2; norm_y[p] += y3 * y3;
                    norm_c[p] += c0v * c0v; norm_c[p] += c1v * c1v; norm_c[p] += c2v * c2v; norm_c[p] += c3v * c3v;
                }
            }
        }
    };
    double4_t acc[4][4];
    double a[4], b[4];   // operands of the step about to be multiplied
    // the rows of both operands that this lane feeds to the matrix cores, dimensions ks + lane / 16
    auto operands = [&](int buf, int ks, double (&ao)[4], double (&bo)[4]) {
        const double *yt = lds + ((size_t)(buf * 2 + 0) * MT2 + wy * 64 + (lane & 15)) * LS2 + (lane >> 4) + ks;
        const double *ct = lds + ((size_t)(buf * 2 + 1) * MT2 + wx * 64 + (lane & 15)) * LS2 + (lane >> 4) + ks;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            ao[t] = yt[t * 16 * LS2];
            bo[t] = ct[t * 16 * LS2];
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int ta = 0; ta < 4; ++ta)
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
    };
    // Block barrier that orders LDS accesses only (requests to memory stay in flight across it).
    auto lds_barrier = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // One chunk: the operands of each step are read while the step before it multiplies.  The
    // barrier that ends the chunk stands before its last step (whose operands are in registers by
    // then), and the first operands of the next chunk are read right behind it, so that the
    // matrix cores have those 16 instructions to work on while the waves meet and the reads return.
    auto compute = [&](int buf, bool has_next) {
        double an[4], bn[4];
#pragma unroll
        for (int ks = 0; ks < MK2; ks += 4) {
            if (ks + 4 < MK2) {
                operands(buf, ks + 4, an, bn);
            } else {
                lds_barrier();
                if (has_next) operands(buf ^ 1, 0, an, bn);
            }
            multiply();
            __builtin_amdgcn_sched_barrier(0);   // no further ahead than that: the registers hold no more
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                a[t] = an[t];
                b[t] = bn[t];
            }
        }
    };

    Tile128 cur = tile128_of(die * per_die + local, A.tiles_x, A.tiles_y);
    Rows rows = rows_of(cur);
    fetch(rows, 0);
    // Entries below `bound` are looked at again.  PRE: one bound for the launch, 1e-9 x (the largest
    // ||y||^2 + the largest ||c||^2), rounding included; otherwise one per tile, see below.
    float bound = 0.f;
    if (PRE && !DOT) {
        float my = 0.f, mc = 0.f;
        for (int i = tid; i < A.nymax; i += 256) my = fmaxf(my, A.ymax[i]);
        for (int i = tid; i < A.ncmax; i += 256) mc = fmaxf(mc, A.cmax[i]);
        for (int o = 32; o > 0; o >>= 1) {
            my = fmaxf(my, __shfl_xor(my, o));
            mc = fmaxf(mc, __shfl_xor(mc, o));
        }
        if (lane == 0) { wave_max[wave] = my; wave_max[4 + wave] = mc; }
        __syncthreads();
        bound = (fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3])) +
                 fmaxf(fmaxf(wave_max[4], wave_max[5]), fmaxf(wave_max[6], wave_max[7]))) * 1.001e-9f;
        __syncthreads();
    }
    for (;;) {
        // the registers hold chunk 0 of the tile `cur`; `next` is what this block takes after it
        const bool more = has_tile(local + blocks_per_die);
        const Tile128 next = more ? tile128_of(die * per_die + local + blocks_per_die, A.tiles_x, A.tiles_y) : cur;
        const Rows next_rows = rows_of(next);
        if (!(PRE && !DOT)) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = (double4_t){0.0, 0.0, 0.0, 0.0};
        }
        if (PRE && !DOT) {   // -||y_tid||^2 (tid < 128) or -||c_(tid - 128)||^2 of this tile, zero past the end
            const int r = tid & (MT2 - 1);
            if (tid < MT2) ny[r] = A.nyg[(size_t)cur.j * A.nq_pad + cur.q0 + r];
            else nc[r] = A.ncg[(size_t)cur.j * A.k_pad + cur.c0 + r];
        }
        norm_y[0] = norm_y[1] = norm_c[0] = norm_c[1] = 0.0;
        stage(0);
        if (1 < nchunks) fetch(rows, MK2);
        else if (more) fetch(next_rows, 0);
        lds_barrier();
        operands(0, 0, a, b);
        if (PRE && !DOT) {
            // the sums start at -(||y||^2 + ||c||^2) and the centroids come doubled: they end at minus the distance
#pragma unroll
            for (int ta = 0; ta < 4; ++ta)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        acc[ta][tb][v] = ny[wy * 64 + ta * 16 + (lane >> 4) + 4 * v] + nc[wx * 64 + tb * 16 + (lane & 15)];
        }
        for (int c = 0; c < nchunks; ++c) {
            if (c + 1 < nchunks) {
                stage((c + 1) & 1);
                if (c + 2 < nchunks) fetch(rows, (c + 2) * MK2);
                else if (more) fetch(next_rows, 0);
            }
            compute(c & 1, c + 1 < nchunks);
        }
        if (!DOT && !PRE) {
            // rows past the end hold the norms of row 0: finite, and a bound too large does no harm
            float wmax = 0.f;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                norm_y[p] += __shfl_xor(norm_y[p], 1); norm_y[p] += __shfl_xor(norm_y[p], 2);
                norm_c[p] += __shfl_xor(norm_c[p], 1); norm_c[p] += __shfl_xor(norm_c[p], 2);
                if ((tid & 3) == 0) { ny[p * ROWS_PER_PASS + srow] = norm_y[p]; nc[p * ROWS_PER_PASS + srow] = norm_c[p]; }
                wmax = fmaxf(wmax, (float)(norm_y[p] > norm_c[p] ? norm_y[p] : norm_c[p]));
            }
            for (int o = 32; o > 0; o >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, o));
            if (lane == 0) wave_max[wave] = wmax;
            __syncthreads();
            // at least 1e-9 * (||y||^2 + ||c||^2) for every entry of the tile, rounding included
            bound = 2.f * fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3])) * 1.001e-9f;
        }
        // lane l of an MFMA tile holds rows l / 16 + 4 * v (v = 0..3) of column l % 16.  Each wave turns
        // its 64 x 64 results into floats in an LDS patch of its own and writes them out as rows of 64;
        // within a wave LDS accesses take effect in program order.
        float *patch_out = reinterpret_cast<float *>(lds) + wave * 64 * OS2;
        const bool vec_out = (k & 3) == 0;
#pragma unroll
        for (int ta = 0; ta < 4; ++ta)
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int rl = ta * 16 + (lane >> 4) + 4 * v, cl = tb * 16 + (lane & 15);
                    float res;
                    if (DOT) res = (float)acc[ta][tb][v];
                    else if (PRE) res = -(float)acc[ta][tb][v];
                    else res = (float)((ny[wy * 64 + rl] + nc[wx * 64 + cl]) - 2.0 * acc[ta][tb][v]);
                    patch_out[rl * OS2 + cl] = res;
                }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll 4
        for (int i = 0; i < 16; ++i) {
            const int rl = i * 4 + (lane >> 4), cl = (lane & 15) * 4;
            const int q = cur.q0 + wy * 64 + rl, ci = cur.c0 + wx * 64 + cl;
            float4 o = *reinterpret_cast<const float4 *>(patch_out + rl * OS2 + cl);
            if (q >= nq || ci >= k) continue;
            if (!DOT && fminf(fminf(o.x, o.y), fminf(o.z, o.w)) < bound) {
                // nearly complete cancellation: the plain definition, so that exact zeros stay exact
                const float *yq = A.queries + (size_t)cur.j * ds + (size_t)q * d;
                float e4[4] = {o.x, o.y, o.z, o.w};
#pragma unroll 1
                for (int e = 0; e < 4; ++e) {
                    if (!(e4[e] < bound) || ci + e >= k) continue;
                    const float *ce = A.codebooks + ((size_t)cur.j * k + ci + e) * ds;
                    double dist = 0.0;
                    for (int t = 0; t < ds; ++t) {
                        const double df = (double)yq[t] - (double)ce[t];
                        dist += df * df;
                    }
                    e4[e] = (float)dist;
                }
                o = make_float4(e4[0], e4[1], e4[2], e4[3]);
            }
            float *dst = A.out + ((size_t)q * m + cur.j) * k + ci;
            if (vec_out && ci + 4 <= k) {
                *reinterpret_cast<float4 *>(dst) = o;
            } else {
                dst[0] = o.x;
                if (ci + 1 < k) dst[1] = o.y;
                if (ci + 2 < k) dst[2] = o.z;
                if (ci + 3 < k) dst[3] = o.w;
            }
        }
        if (!more) break;
        __syncthreads();   // every wave has left its patch: the operand buffers are free again
        local += blocks_per_die;
        cur = next;
        rows = next_rows;
    }
}

// Scratch memory of the 128 x 128 form (operands as doubles and their norms), kept by the context.
static int lut_ws_reserve(pq_ctx *ctx, size_t bytes) {
    if (bytes <= ctx->lut_ws_bytes) return PQ_OK;
    PQ_HIP(ctx, hipStreamSynchronize(ctx->stream));   // kernels already enqueued may still use the old buffer
    if (ctx->lut_ws) {
        PQ_HIP(ctx, hipFree(ctx->lut_ws));
        ctx->lut_ws = nullptr;
        ctx->lut_ws_bytes = 0;
    }
    const size_t want = (bytes + bytes / 4 + ((size_t)1 << 20) - 1) >> 20 << 20;
    void *p = nullptr;
    const hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, PQ_ENOMEM, "allocation of %zu bytes for the operands of the Tables step failed: %s", want, hipGetErrorString(e));
    }
    ctx->lut_ws = p;
    ctx->lut_ws_bytes = want;
    return PQ_OK;
}

// Launch of the 128 x 128 form: two blocks per compute unit (a multiple of 8 blocks, one share per die).
// Sub-vectors of 64 dimensions and more take the pass that converts the operands first, if every
// operand row serves 8 tiles and more (the pass costs about as much as one of them) and the copies
// stay below 2 GiB.
template <bool DOT>
static int launch_mfma128(pq_ctx *ctx, const float *queries, const float *codebooks, int nq, int d, int m, int k,
                          float *out, int tiles_x, int tiles_y) {
    Mfma128Args A{};
    A.queries = queries; A.codebooks = codebooks; A.out = out;
    A.nq = nq; A.d = d; A.m = m; A.k = k; A.ds = d / m; A.dsp = (A.ds + MK2 - 1) / MK2 * MK2;
    A.tiles_x = tiles_x; A.tiles_y = tiles_y; A.total = tiles_x * tiles_y * m;
    const int grid = (2 * ctx->num_cu + 7) / 8 * 8;
    A.nq_pad = tiles_y * MT2; A.k_pad = tiles_x * MT2;
    const size_t rows_y = (size_t)m * A.nq_pad, rows_c = (size_t)m * A.k_pad;
    const size_t bytes = (rows_y + rows_c) * (A.dsp + 1) * sizeof(double) + (rows_y + rows_c) / 16 * sizeof(float) + 64;
    if (A.ds >= 64 && tiles_x >= 8 && tiles_y >= 8 && bytes <= ((size_t)2 << 30)) {
        const int rc = lut_ws_reserve(ctx, bytes);
        if (rc) return rc;
        double *yd = (double *)ctx->lut_ws, *cd = yd + rows_y * A.dsp, *nyg = cd + rows_c * A.dsp, *ncg = nyg + rows_y;
        const unsigned by = (unsigned)((rows_y * 16 + 255) / 256), bc = (unsigned)((rows_c * 16 + 255) / 256);
        float *ymax = (float *)(ncg + rows_c), *cmax = ymax + by;
        prep128_kernel<<<by, 256, 0, ctx->stream>>>(queries, (size_t)d, (size_t)A.ds, nq, A.nq_pad, m, A.ds, A.dsp, yd, nyg, ymax, 1.0, DOT ? 1.0 : -1.0);
        prep128_kernel<<<bc, 256, 0, ctx->stream>>>(codebooks, (size_t)A.ds, (size_t)k * A.ds, k, A.k_pad, m, A.ds, A.dsp, cd, ncg, cmax, DOT ? 1.0 : 2.0, DOT ? 1.0 : -1.0);
        A.yd = yd; A.cd = cd; A.nyg = nyg; A.ncg = ncg; A.ymax = ymax; A.cmax = cmax; A.nymax = (int)by; A.ncmax = (int)bc;
        build_luts_mfma128_kernel<DOT, true><<<grid, 256, 0, ctx->stream>>>(A);
    } else {
        build_luts_mfma128_kernel<DOT, false><<<grid, 256, 0, ctx->stream>>>(A);
    }
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// Approximate squared distances ||y_q - c_i||^2 of nq vectors to k centroids (one sub-space, all d
// dimensions) on the fp32 matrix cores (v_mfma_f32_32x32x2f32: 64 cycles for 4096 flops, twice the rate of the
// fp64 ones; the 16x16x4 form measured 48 cycles for 2048 flops), for
// callers that only rank the centroids and settle the ranks that matter exactly afterwards (the
// coarse step of the inverted-index search).  Same tiling and block numbering as the fp64 form
// above: tiles of 128 x 128, each of the 4 waves 64 x 64 outputs as 2 x 2 matrix tiles of 32 x 32, persistent
// blocks, two LDS buffers (of 32 dimensions here), results written as rows through LDS.  Operands stay
// floats ([row][dimension] with a row stride of 34 words: the 32 rows x 2 dimensions that a wave
// reads at once fall into 64 different banks); norms and the final combination are fp32 as well.
// Every result is within coarse_f32_error(d) * (||y||^2 + ||c||^2) of the exact value.
constexpr int MK3 = 32;        // dimensions per chunk (one barrier per chunk: 64 matrix instructions of 32 cycles are too few to hide it)
constexpr int LS3 = MK3 + 2;   // operand row stride in floats
constexpr int OS3 = 72;        // output row stride in floats (32 rows of 64 floats per wave at a time)
constexpr int COARSE_SLOTS = 4; // places per row and tile of the filtering forms

// FILTER: instead of the matrix, the entries at or below the row's bound theta[q] leave as keys (ordered value, column),
// see coarse_filter_tile.
struct CoarseF32Args {
    const float *queries, *cents;   // [nq][d], centroid i at cents + i * cent_stride
    size_t cent_stride;
    float *out;                     // [nq][k]
    int nq, d, k;
    int tiles_x, tiles_y, total;
    const float *theta;             // FILTER: [nq]
    unsigned long long *slot_keys;  // FILTER: [nq][tiles_x][COARSE_SLOTS], every place written (~0: unused)
    unsigned long long *ov_keys;    // FILTER: [nq][ov_cap]
    unsigned int *ov_cnt;           // FILTER: [nq], zero at the start
    int ov_cap;
};

typedef float coarse_floatx16 __attribute__((ext_vector_type(16)));

// End of a 128 x 128 tile of the filtering forms: acc holds the inner products <y, c> of the wave's 64 x 64 outputs (lane l
// of a matrix tile: rows 8 * (v / 4) + 4 * (l / 32) + v % 4, v = 0..15, of column l % 32), ny / nc / th the squared norms
// and bounds of the tile's rows and columns (a bound of -inf for rows past the end, a norm of +inf for columns past the
// end).  The values ny + nc - 2 <y, c> at or below their row's bound leave as keys (ordered value, column).  They are rare,
// about one per row and tile, and nothing waits for global memory: every row has COARSE_SLOTS places per tile in LDS
// (`stash`: the operand buffers, free by now), handed out by a counter in LDS, and the rows' places, used or not, leave
// as 32 bytes per row to slot_keys[row][tile of columns][COARSE_SLOTS].  Only a row's entries beyond its places take an
// atomic operation on global memory (ov_cnt[row], zero at the start, counts them; the first ov_cap go to ov_keys[row][]).
// Every thread of the block calls this; the caller's barrier before the buffers are staged again ends it.
// The wave holds rows wy * 64 .. + 63 and columns wcol .. wcol + 32 TB - 1 of the tile, as 2 x TB matrix tiles.
template <int TB>
__device__ __forceinline__ void coarse_filter_tile(const coarse_floatx16 (&acc)[2][TB], int wy, int wcol, void *stash, const float *th,
                                                   const float *ny, const float *nc, int q0, int c0, int nq, int ctile, int tiles_x,
                                                   unsigned long long *slot_keys, unsigned long long *ov_keys, unsigned int *ov_cnt,
                                                   int ov_cap) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned long long *skeys = reinterpret_cast<unsigned long long *>(stash);          // [MT2][COARSE_SLOTS]
    unsigned int *scnt = reinterpret_cast<unsigned int *>(skeys + MT2 * COARSE_SLOTS);   // [MT2]
    // values of the wave on their way to the places: [output within a quarter of the lane's outputs][lane]
    unsigned int *held = scnt + MT2 + wave * (16 * 64) + lane;
    if (tid < 256) {
        skeys[2 * tid] = ~0ull;
        skeys[2 * tid + 1] = ~0ull;
    }
    if (tid < MT2) scnt[tid] = 0u;
    float ncc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) ncc[tb] = nc[wcol + tb * 32 + (lane & 31)];
    __syncthreads();   // (the places are cleared)
    // A quarter of the lane's outputs at a time (matrix tiles ta of both columns, 8 of their 16 registers).  Entries at or
    // below the bound are noted first and placed afterwards: placing waits for a counter in LDS, and in the unrolled
    // code every such wait would stand in the way of all 64 lanes.
#pragma unroll
    for (int quarter = 0; quarter < 4; ++quarter) {
        const int ta = quarter >> 1, g0 = (quarter & 1) * 2;   // registers 4 g0 .. 4 g0 + 7: rows 8 g + 4 (l / 32) + 0..3, g = g0, g0 + 1
        const int rbase = wy * 64 + ta * 32 + 4 * (lane >> 5);
        float4 bound4[2], nyr4[2];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            bound4[g] = *reinterpret_cast<const float4 *>(th + rbase + 8 * (g0 + g));
            nyr4[g] = *reinterpret_cast<const float4 *>(ny + rbase + 8 * (g0 + g));
        }
        unsigned int noted = 0u;   // bit TB * vv + tb: output (register 4 g0 + vv, column tile tb)
#pragma unroll
        for (int vv = 0; vv < 8; ++vv) {
            const float4 b4 = bound4[vv >> 2], n4 = nyr4[vv >> 2];
            const float bound = (vv & 3) == 0 ? b4.x : (vv & 3) == 1 ? b4.y : (vv & 3) == 2 ? b4.z : b4.w;
            const float nyr = (vv & 3) == 0 ? n4.x : (vv & 3) == 1 ? n4.y : (vv & 3) == 2 ? n4.z : n4.w;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const float val = fmaf(-2.f, acc[ta][tb][4 * g0 + vv], nyr + ncc[tb]);
                if (val <= bound) {
                    held[(TB * vv + tb) * 64] = __float_as_uint(val);
                    noted |= 1u << (TB * vv + tb);
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // within a wave LDS accesses take effect in program order
        while (noted != 0u) {
            const int o = __builtin_ctz(noted);
            noted &= noted - 1u;
            const float val = __uint_as_float(held[o * 64]);
            const int vv = o / TB, tb = o % TB;
            const int r = rbase + 8 * (g0 + (vv >> 2)) + (vv & 3);
            const unsigned int col = (unsigned int)(c0 + wcol + tb * 32 + (lane & 31));
            const unsigned long long key = ((unsigned long long)f32_to_ord(val) << 32) | col;
            const unsigned int pos = atomicAdd(&scnt[r], 1u);
            if (pos < (unsigned int)COARSE_SLOTS) {
                skeys[r * COARSE_SLOTS + pos] = key;
            } else {
                const unsigned int at = atomicAdd(&ov_cnt[q0 + r], 1u);
                if (at < (unsigned int)ov_cap) ov_keys[(size_t)(q0 + r) * ov_cap + at] = key;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (the noted values are read before the next quarter's are written)
    }
    __syncthreads();
    static_assert(COARSE_SLOTS == 4, "two threads per row, two places each");
    const int row = tid >> 1, half = tid & 1;
    if (tid < 256 && q0 + row < nq) {
        const ulonglong2 two = *reinterpret_cast<const ulonglong2 *>(skeys + row * COARSE_SLOTS + 2 * half);
        *reinterpret_cast<ulonglong2 *>(slot_keys + ((size_t)(q0 + row) * tiles_x + ctile) * COARSE_SLOTS + 2 * half) = two;
    }
}

template <bool FILTER>
__global__ __launch_bounds__(256, 2) void coarse_f32_kernel(const CoarseF32Args A) {
    typedef coarse_floatx16 floatx16;
    __shared__ __align__(16) float lds[2 * 2 * MT2 * LS3];   // [buffer][y | c][row][LS3]
    __shared__ __align__(16) float ny[MT2], nc[MT2], th[MT2];
    static_assert(4 * 32 * OS3 <= 2 * 2 * MT2 * LS3, "output staging fits the operand buffers");
    static_assert(MT2 * (COARSE_SLOTS * 8 + 4) + 256 * 16 * 4 <= (int)sizeof(float) * 2 * 2 * MT2 * LS3, "the rows' places and the noted entries fit the operand buffers");
    const int nq = A.nq, d = A.d, k = A.k;
    const int per_die = (A.total + 7) >> 3, blocks_per_die = gridDim.x >> 3;
    const int die = blockIdx.x & 7;
    int local = blockIdx.x >> 3;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const int nchunks = (d + MK3 - 1) / MK3;
    auto has_tile = [&](int l) { return l < per_die && die * per_die + l < A.total; };
    if (!has_tile(local)) return;
    // 8 threads per row (4 floats each), rows tid / 8 + 32 * pass; row 0 stands in for rows past the end
    const int srow = tid >> 3, sk = (tid & 7) * 4;
    struct Rows {
        const float *y[4], *c[4];
    };
    auto rows_of = [&](const Tile128 &t) {
        Rows r;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int row = p * 32 + srow;
            r.y[p] = A.queries + (size_t)(t.q0 + row < nq ? t.q0 + row : 0) * d + sk;
            r.c[p] = A.cents + (size_t)(t.c0 + row < k ? t.c0 + row : 0) * A.cent_stride + sk;
        }
        return r;
    };
    float4 rf[2][4];   // [y | c][pass]: the chunk after the one being multiplied
    auto fetch = [&](const Rows &r, int k0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            rf[0][p] = rf[1][p] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + sk < d) {   // d is a multiple of 4
                rf[0][p] = *reinterpret_cast<const float4 *>(r.y[p] + k0);
                rf[1][p] = *reinterpret_cast<const float4 *>(r.c[p] + k0);
            }
        }
    };
    float norm_y[4], norm_c[4];
    auto stage = [&](int buf) {
        float *yd = lds + ((size_t)(buf * 2 + 0) * MT2 + srow) * LS3 + sk;
        float *cd = lds + ((size_t)(buf * 2 + 1) * MT2 + srow) * LS3 + sk;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            // (rows of 34 words start on 8-byte boundaries)
            *reinterpret_cast<float2 *>(yd + p * 32 * LS3) = make_float2(rf[0][p].x, rf[0][p].y);
            *reinterpret_cast<float2 *>(yd + p * 32 * LS3 + 2) = make_float2(rf[0][p].z, rf[0][p].w);
            *reinterpret_cast<float2 *>(cd + p * 32 * LS3) = make_float2(rf[1][p].x, rf[1][p].y);
            *reinterpret_cast<float2 *>(cd + p * 32 * LS3 + 2) = make_float2(rf[1][p].z, rf[1][p].w);
            norm_y[p] = fmaf(rf[0][p].x, rf[0][p].x, fmaf(rf[0][p].y, rf[0][p].y, fmaf(rf[0][p].z, rf[0][p].z, fmaf(rf[0][p].w, rf[0][p].w, norm_y[p]))));
            norm_c[p] = fmaf(rf[1][p].x, rf[1][p].x, fmaf(rf[1][p].y, rf[1][p].y, fmaf(rf[1][p].z, rf[1][p].z, fmaf(rf[1][p].w, rf[1][p].w, norm_c[p]))));
        }
    };
    floatx16 acc[2][2];
    float a[2], b[2];
    // lane l feeds row l % 32 of its matrix tiles, dimension ks + l / 32
    auto operands = [&](int buf, int ks, float (&ao)[2], float (&bo)[2]) {
        const float *yt = lds + ((size_t)(buf * 2 + 0) * MT2 + wy * 64 + (lane & 31)) * LS3 + (lane >> 5) + ks;
        const float *ct = lds + ((size_t)(buf * 2 + 1) * MT2 + wx * 64 + (lane & 31)) * LS3 + (lane >> 5) + ks;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            ao[t] = yt[t * 32 * LS3];
            bo[t] = ct[t * 32 * LS3];
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
    };
    auto lds_barrier = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // (the barrier that ends a chunk stands before its last step, see the fp64 form)
    auto compute = [&](int buf, bool has_next) {
        float an[2], bn[2];
#pragma unroll
        for (int ks = 0; ks < MK3; ks += 2) {
            if (ks + 2 < MK3) {
                operands(buf, ks + 2, an, bn);
            } else {
                lds_barrier();
                if (has_next) operands(buf ^ 1, 0, an, bn);
            }
            multiply();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                a[t] = an[t];
                b[t] = bn[t];
            }
        }
    };

    Tile128 cur = tile128_of(die * per_die + local, A.tiles_x, A.tiles_y);
    Rows rows = rows_of(cur);
    fetch(rows, 0);
    for (;;) {
        const bool more = has_tile(local + blocks_per_die);
        const Tile128 next = more ? tile128_of(die * per_die + local + blocks_per_die, A.tiles_x, A.tiles_y) : cur;
        const Rows next_rows = rows_of(next);
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[ta][tb][v] = 0.f;
#pragma unroll
        for (int p = 0; p < 4; ++p) norm_y[p] = norm_c[p] = 0.f;
        if (FILTER && tid < MT2) th[tid] = cur.q0 + tid < nq ? A.theta[cur.q0 + tid] : -__builtin_inff();
        stage(0);
        if (1 < nchunks) fetch(rows, MK3);
        else if (more) fetch(next_rows, 0);
        lds_barrier();
        operands(0, 0, a, b);
        for (int c = 0; c < nchunks; ++c) {
            if (c + 1 < nchunks) {
                stage((c + 1) & 1);
                if (c + 2 < nchunks) fetch(rows, (c + 2) * MK3);
                else if (more) fetch(next_rows, 0);
            }
            compute(c & 1, c + 1 < nchunks);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
#pragma unroll
            for (int o = 1; o < 8; o <<= 1) {
                norm_y[p] += __shfl_xor(norm_y[p], o);
                norm_c[p] += __shfl_xor(norm_c[p], o);
            }
            // (columns past the end: with FILTER a norm that keeps them out)
            if ((tid & 7) == 0) { ny[p * 32 + srow] = norm_y[p]; nc[p * 32 + srow] = FILTER && cur.c0 + p * 32 + srow >= k ? __builtin_inff() : norm_c[p]; }
        }
        __syncthreads();
        // lane l of a matrix tile holds rows 8 * (v / 4) + 4 * (l / 32) + v % 4 (v = 0..15) of column l % 32
        if (FILTER) {
            coarse_filter_tile<2>(acc, wy, wx * 64, lds, th, ny, nc, cur.q0, cur.c0, nq, cur.c0 / MT2, A.tiles_x, A.slot_keys, A.ov_keys, A.ov_cnt, A.ov_cap);
            if (!more) break;
            __syncthreads();   // the rows' places have left: the operand buffers are free again
            local += blocks_per_die;
            cur = next;
            rows = next_rows;
            continue;
        }
        // 32 rows x 64 columns of a wave at a time go through an LDS patch of its own and leave as rows
        float *patch_out = lds + wave * 32 * OS3;
        const bool vec_out = (k & 3) == 0;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), cl = tb * 32 + (lane & 31);
                    patch_out[rl * OS3 + cl] = fmaf(-2.f, acc[half][tb][v], ny[wy * 64 + half * 32 + rl] + nc[wx * 64 + cl]);
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll 4
            for (int i = 0; i < 8; ++i) {
                const int rl = i * 4 + (lane >> 4), cl = (lane & 15) * 4;
                const int q = cur.q0 + wy * 64 + half * 32 + rl, ci = cur.c0 + wx * 64 + cl;
                const float4 o = *reinterpret_cast<const float4 *>(patch_out + rl * OS3 + cl);
                if (q >= nq || ci >= k) continue;
                float *dst = A.out + (size_t)q * k + ci;
                if (vec_out && ci + 4 <= k) {
                    *reinterpret_cast<float4 *>(dst) = o;
                } else {
                    dst[0] = o.x;
                    if (ci + 1 < k) dst[1] = o.y;
                    if (ci + 2 < k) dst[2] = o.z;
                    if (ci + 3 < k) dst[3] = o.w;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the patch is read before its next rows are written
        }
        if (!more) break;
        __syncthreads();   // every wave has left its patch: the operand buffers are free again
        local += blocks_per_die;
        cur = next;
        rows = next_rows;
    }
}

// Bound on |approximate - exact| / (||y||^2 + ||c||^2) for the kernel above: d products rounded once or
// twice and added in fp32 in some order (twice d units of 2^-24 on 2 |<y, c>| <= ||y||^2 + ||c||^2), the two
// norms added up the same way (d units each), the final three operations; doubled for good measure.
float coarse_f32_error(int d) { return 4.f * (float)(d + 8) * 5.9604645e-8f; }

// Whether launch_coarse_f32 serves the shape (else the caller takes the exact Tables step).
bool coarse_f32_usable(pq_ctx *ctx, const float *queries, const float *cents, int nq, int d, int k, const float *out) {
    const int64_t tiles = (int64_t)((k + MT2 - 1) / MT2) * ((nq + MT2 - 1) / MT2);
    const uintptr_t bits = (uintptr_t)queries | (uintptr_t)cents | (uintptr_t)out;
    return d >= 16 && (d & 3) == 0 && (bits & 15) == 0 && tiles >= 2 * (int64_t)ctx->num_cu && tiles < (1ll << 30);
}

int launch_coarse_f32(pq_ctx *ctx, const float *queries, const float *cents, size_t cent_stride, int nq, int d, int k, float *out) {
    if (!coarse_f32_usable(ctx, queries, cents, nq, d, k, out) || (cent_stride & 3) != 0) return fail(ctx, PQ_EINVAL, "coarse_f32: shape not served");
    CoarseF32Args A{};
    A.queries = queries; A.cents = cents; A.cent_stride = cent_stride; A.out = out; A.nq = nq; A.d = d; A.k = k;
    A.tiles_x = (k + MT2 - 1) / MT2; A.tiles_y = (nq + MT2 - 1) / MT2; A.total = A.tiles_x * A.tiles_y;
    const int grid = (2 * ctx->num_cu + 7) / 8 * 8;
    coarse_f32_kernel<false><<<grid, 256, 0, ctx->stream>>>(A);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// The same distances, but only those at or below theta[q] leave, as keys (ordered value << 32 | centroid): COARSE_SLOTS
// places per query and 128 centroids in slot_keys[q][coarse_filter_slots(k)] (~0: unused), the entries beyond them in
// ov_keys[q][ov_cap]; ov_cnt[q] (zero at the start) counts those.
int coarse_filter_slots(int k) { return (k + MT2 - 1) / MT2 * COARSE_SLOTS; }

int launch_coarse_f32_filter(pq_ctx *ctx, const float *queries, const float *cents, int nq, int d, int k, const float *theta,
                             unsigned long long *slot_keys, unsigned long long *ov_keys, unsigned int *ov_cnt, int ov_cap) {
    if (!coarse_f32_usable(ctx, queries, cents, nq, d, k, queries)) return fail(ctx, PQ_EINVAL, "coarse_f32: shape not served");
    CoarseF32Args A{};
    A.queries = queries; A.cents = cents; A.cent_stride = (size_t)d; A.out = nullptr; A.nq = nq; A.d = d; A.k = k;
    A.tiles_x = (k + MT2 - 1) / MT2; A.tiles_y = (nq + MT2 - 1) / MT2; A.total = A.tiles_x * A.tiles_y;
    A.theta = theta; A.slot_keys = slot_keys; A.ov_keys = ov_keys; A.ov_cnt = ov_cnt; A.ov_cap = ov_cap;
    const int grid = (2 * ctx->num_cu + 7) / 8 * 8;
    coarse_f32_kernel<true><<<grid, 256, 0, ctx->stream>>>(A);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// The filtering pass on the fp16 matrix cores (v_mfma_f32_32x32x16_f16: 16 times the rate of the fp32 form) without
// giving up fp32 accuracy: every operand value x, scaled by a power of two s that brings the greatest magnitude of its
// matrix to [2^13, 2^14), is kept as two halves hi = fp16(x s), lo = fp16(x s - hi) (x s = hi + lo up to 2^-22 of
// its size), and <y, c> is accumulated in fp32 as hi hi + hi lo + lo hi (products of halves are exact in fp32; the
// omitted lo lo is below 2^-22 of |y| |c|).  The operands are split once per call by split16_prep_kernel, [row][chunk
// of 32 dimensions][32 hi | 32 lo] with the rows' squared norms beside them, so the kernel stages 16-byte pieces
// as they are.  Tiles of 128 x 128, block numbering and end of tile as in the fp32 form.
// Magnitudes outside 2^-40 .. 2^40 (or not finite) are not served: the kernel keeps nothing then, and the caller's
// queries, left without candidates, take their exact rows.
constexpr int HK = 32;     // dimensions per chunk
constexpr int HROW = 9;    // 16-byte pieces per staged row of a chunk: 4 of hi, 4 of lo, 1 unused (rows 36 words apart:
                           // the 16 rows that a 16-byte read serves at a time fall into different banks)

typedef uint32_t lut_u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 lut_half8 __attribute__((ext_vector_type(8)));

__global__ void split16_clear_kernel(unsigned int *maxbits) {
    if (threadIdx.x < 2) maxbits[threadIdx.x] = 0u;
}

// maxbits[0] = greatest |a[i]|, maxbits[1] = greatest |b[i]| as float bits (they start at 0; NaNs order above infinity)
__global__ __launch_bounds__(256) void split16_absmax_kernel(const float *__restrict__ a, size_t na, const float *__restrict__ b,
                                                             size_t nb, unsigned int *maxbits) {
    __shared__ unsigned int red[2][4];
    unsigned int m[2] = {0u, 0u};
    const size_t step = (size_t)gridDim.x * 256;
    for (int w = 0; w < 2; ++w) {
        const float *v = w ? b : a;
        const size_t n = w ? nb : na;
        for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += step) {
            const unsigned int bits = __float_as_uint(v[i]) & 0x7fffffffu;   // (|x|: orders like the value, NaNs above infinity)
            m[w] = bits > m[w] ? bits : m[w];
        }
        for (int o = 32; o > 0; o >>= 1) { const unsigned int t = (unsigned int)__shfl_xor((int)m[w], o); m[w] = t > m[w] ? t : m[w]; }
        if ((threadIdx.x & 63) == 0) red[w][threadIdx.x >> 6] = m[w];
    }
    __syncthreads();
    if (threadIdx.x < 2) {
        const unsigned int *r = red[threadIdx.x];
        unsigned int t = r[0] > r[1] ? r[0] : r[1];
        t = r[2] > t ? r[2] : t;
        t = r[3] > t ? r[3] : t;
        atomicMax(&maxbits[threadIdx.x], t);
    }
}

// Power of two that brings a matrix whose greatest magnitude has the bits `maxbits` to [2^13, 2^14), as the exponent
// field of a float; 0 if the magnitude is outside 2^-40 .. 2^40 (an all-zero matrix counts as 1).
__device__ __forceinline__ unsigned int split16_scale_field(unsigned int maxbits) {
    if (maxbits == 0u) return 127u + 13u;
    const unsigned int e = maxbits >> 23;
    if (e < 127u - 40u || e > 127u + 40u) return 0u;
    return 267u - e;   // 2^(13 - (e - 127))
}

// 8 threads per row, 4 dimensions of every chunk each.  Rows from `rows` up to rows_pad and dimensions from d up to
// nch * 32 are zeros.  norms[row] = ||row||^2 in fp32 (each thread a chain of fused multiply-adds, then three additions).
__global__ __launch_bounds__(256) void split16_prep_kernel(const float *__restrict__ src, int rows, int rows_pad, int d, int nch,
                                                           const unsigned int *__restrict__ maxbits, lut_u32x4 *__restrict__ dst,
                                                           float *__restrict__ norms) {
    const int row = blockIdx.x * 32 + (threadIdx.x >> 3), seg = threadIdx.x & 7;
    if (row >= rows_pad) return;
    const unsigned int field = split16_scale_field(*maxbits);
    const float s = __uint_as_float(field << 23);   // (0 for matrices not served: the halves are zeros then, and unused)
    uint2 *out = reinterpret_cast<uint2 *>(dst + (size_t)row * nch * 8);
    float norm = 0.f;
    for (int c = 0; c < nch; ++c) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        const int t = c * HK + seg * 4;
        if (row < rows && t < d) x = *reinterpret_cast<const float4 *>(src + (size_t)row * d + t);   // (d is a multiple of 4)
        norm = fmaf(x.x, x.x, fmaf(x.y, x.y, fmaf(x.z, x.z, fmaf(x.w, x.w, norm))));
        const float v[4] = {x.x * s, x.y * s, x.z * s, x.w * s};
        _Float16 hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hi[i] = (_Float16)v[i];
            lo[i] = (_Float16)(v[i] - (float)hi[i]);
        }
        auto pack = [](_Float16 a, _Float16 b) {
            return (uint32_t)__builtin_bit_cast(unsigned short, a) | ((uint32_t)__builtin_bit_cast(unsigned short, b) << 16);
        };
        out[c * 16 + seg] = make_uint2(pack(hi[0], hi[1]), pack(hi[2], hi[3]));       // hi: the first 64 bytes of the chunk
        out[c * 16 + 8 + seg] = make_uint2(pack(lo[0], lo[1]), pack(lo[2], lo[3]));   // lo: the second
    }
    norm += __shfl_xor(norm, 1);
    norm += __shfl_xor(norm, 2);
    norm += __shfl_xor(norm, 4);
    if (seg == 0) norms[row] = norm;
}

struct CoarseSplit16Args {
    const lut_u32x4 *yh, *ch;       // [rows_pad][nch][8]: the split operands
    const float *nyg, *ncg;         // squared norms
    const unsigned int *maxbits;    // [2]: greatest magnitudes of the two matrices
    int nq, k, nch;
    int tiles_x, tiles_y, total;
    const float *theta;             // [nq]
    unsigned long long *slot_keys;  // [nq][tiles_x][COARSE_SLOTS], every place written (~0: unused)
    unsigned long long *ov_keys;    // [nq][ov_cap]
    unsigned int *ov_cnt;           // [nq], zero at the start
    int ov_cap;
};

#ifdef PQ_SCAN_TIMING
__device__ unsigned long long g_split16_ticks[8];
#define H16_TICK(phase) do { const unsigned long long now__ = __builtin_amdgcn_s_memtime(); tick_acc[phase] += now__ - tick_last; tick_last = now__; } while (0)
#else
#define H16_TICK(phase) do { } while (0)
#endif

// Blocks of 8 waves, two per compute unit (4 waves per SIMD: the end of a tile and the staging are waits, mostly); wave
// (wy, wx) holds rows 64 wy .. and columns 32 wx .. of the tile.
__global__ __launch_bounds__(512, 4) void coarse_split16_filter_kernel(const CoarseSplit16Args A) {
    __shared__ lut_u32x4 lds[2 * 2 * MT2 * HROW];   // [buffer][y | c][row][HROW]
    __shared__ __align__(16) float ny[MT2], nc[MT2], th[MT2];
    static_assert(MT2 * (COARSE_SLOTS * 8 + 4) + 512 * 16 * 4 <= (int)sizeof(lut_u32x4) * 2 * 2 * MT2 * HROW, "the rows' places and the noted entries fit the operand buffers");
    const unsigned int fy = split16_scale_field(A.maxbits[0]), fc = split16_scale_field(A.maxbits[1]);
    if (fy == 0u || fc == 0u) return;   // (uniform: magnitudes that the halves do not serve)
    const float unscale = __uint_as_float((381u - fy - fc) << 23);   // 1 / (s_y s_c) = 2^(254 - fy - fc): between 2^-106 and 2^54
    const int nq = A.nq, k = A.k, nch = A.nch;
    const int per_die = (A.total + 7) >> 3, blocks_per_die = gridDim.x >> 3;
    const int die = blockIdx.x & 7;
    int local = blockIdx.x >> 3;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 2, wx = wave & 3;
    auto has_tile = [&](int l) { return l < per_die && die * per_die + l < A.total; };
    if (!has_tile(local)) return;
    // piece tid % 8 of rows tid / 8 + 64 * pass (the operands are padded to whole tiles)
    const int srow = tid >> 3, seg = tid & 7;
    lut_u32x4 rf[2][2];   // [y | c][pass]: the chunk after the one being multiplied
    auto fetch = [&](const Tile128 &t, int c) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            rf[0][p] = A.yh[((size_t)(t.q0 + p * 64 + srow) * nch + c) * 8 + seg];
            rf[1][p] = A.ch[((size_t)(t.c0 + p * 64 + srow) * nch + c) * 8 + seg];
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            lds[((buf * 2 + 0) * MT2 + p * 64 + srow) * HROW + seg] = rf[0][p];
            lds[((buf * 2 + 1) * MT2 + p * 64 + srow) * HROW + seg] = rf[1][p];
        }
    };
    coarse_floatx16 acc[2][1];
    // lane l feeds row l % 32 of its matrix tiles, dimensions 16 * step + 8 * (l / 32) .. + 7 of the chunk
    auto compute = [&](int buf) {
        const lut_u32x4 *yt = lds + ((buf * 2 + 0) * MT2 + wy * 64 + (lane & 31)) * HROW + (lane >> 5);
        const lut_u32x4 *ct = lds + ((buf * 2 + 1) * MT2 + wx * 32 + (lane & 31)) * HROW + (lane >> 5);
#pragma unroll
        for (int step = 0; step < HK / 16; ++step) {
            lut_half8 ah[2], al[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                ah[t] = __builtin_bit_cast(lut_half8, yt[t * 32 * HROW + 2 * step]);
                al[t] = __builtin_bit_cast(lut_half8, yt[t * 32 * HROW + 4 + 2 * step]);
            }
            const lut_half8 bh = __builtin_bit_cast(lut_half8, ct[2 * step]);
            const lut_half8 bl = __builtin_bit_cast(lut_half8, ct[4 + 2 * step]);
#pragma unroll
            for (int ta = 0; ta < 2; ++ta) {
                acc[ta][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[ta], bh, acc[ta][0], 0, 0, 0);
                acc[ta][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[ta], bl, acc[ta][0], 0, 0, 0);
                acc[ta][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[ta], bh, acc[ta][0], 0, 0, 0);
            }
        }
    };

    Tile128 cur = tile128_of(die * per_die + local, A.tiles_x, A.tiles_y);
    fetch(cur, 0);
#ifdef PQ_SCAN_TIMING
    unsigned long long tick_acc[5] = {0, 0, 0, 0, 0}, tick_last = __builtin_amdgcn_s_memtime();
#endif
    for (;;) {
        const bool more = has_tile(local + blocks_per_die);
        const Tile128 next = more ? tile128_of(die * per_die + local + blocks_per_die, A.tiles_x, A.tiles_y) : cur;
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ta][0][v] = 0.f;
        if (tid < MT2) {
            th[tid] = cur.q0 + tid < nq ? A.theta[cur.q0 + tid] : -__builtin_inff();
            ny[tid] = A.nyg[cur.q0 + tid];
            nc[tid] = cur.c0 + tid < k ? A.ncg[cur.c0 + tid] : __builtin_inff();   // (columns past the end stay out)
        }
        stage(0);
        if (1 < nch) fetch(cur, 1);
        else if (more) fetch(next, 0);
        __syncthreads();
        H16_TICK(0);
        // chunk c is multiplied from buffer c % 2 while chunk c + 1 goes into the other one (which every wave has left:
        // the barrier stands after the multiplications) and chunk c + 2 is on its way from memory
        for (int c = 0; c < nch; ++c) {
            if (c + 1 < nch) {
                stage((c + 1) & 1);
                if (c + 2 < nch) fetch(cur, c + 2);
                else if (more) fetch(next, 0);
            }
            H16_TICK(1);
            compute(c & 1);
            H16_TICK(2);
            __syncthreads();
            H16_TICK(3);
        }
#pragma unroll
        for (int ta = 0; ta < 2; ++ta)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ta][0][v] *= unscale;   // (a power of two: exact)
        coarse_filter_tile<1>(acc, wy, wx * 32, lds, th, ny, nc, cur.q0, cur.c0, nq, cur.c0 / MT2, A.tiles_x, A.slot_keys, A.ov_keys, A.ov_cnt, A.ov_cap);
        if (!more) break;
        __syncthreads();   // the rows' places have left: the operand buffers are free again
        H16_TICK(4);
        local += blocks_per_die;
        cur = next;
    }
#ifdef PQ_SCAN_TIMING
    if (lane == 0) for (int i = 0; i < 5; ++i) atomicAdd(&g_split16_ticks[i], tick_acc[i]);
#endif
}

// Bound on |approximate - exact| / (||y||^2 + ||c||^2) for the kernel above.  The inner product is a sum of 3 dpad exact
// products whose magnitudes add up to at most (1 + 2^-9) |y| |c|; each of the 3 dpad additions may lose one unit of
// 2^-23 of that (whatever the order and the rounding of the matrix unit's adder), the representation 2^-19 in all (halves,
// omitted products, fp16 values below the normal range); with 2 |y| |c| <= ||y||^2 + ||c||^2 the term 2 <y, c> is off by at
// most (3 dpad 2^-23 + 2^-19) (||y||^2 + ||c||^2).  The two norms add d / 8 + 6 units of 2^-24 of themselves each, the final
// combination three.  Doubled for good measure, like the bound of the fp32 form.
float coarse_split16_error(int d) {
    const int dpad = (d + HK - 1) / HK * HK;
    return 2.f * ((float)(3 * dpad) * 1.1920929e-7f + 1.9073486e-6f + (float)(d / 8 + 12) * 5.9604645e-8f);
}

// The filtering pass of launch_coarse_f32_filter through split fp16 operands (shapes as coarse_f32_usable accepts them).
int launch_coarse_split16_filter(pq_ctx *ctx, const float *queries, const float *cents, int nq, int d, int k, const float *theta,
                                 unsigned long long *slot_keys, unsigned long long *ov_keys, unsigned int *ov_cnt, int ov_cap) {
    if (!coarse_f32_usable(ctx, queries, cents, nq, d, k, queries)) return fail(ctx, PQ_EINVAL, "coarse_split16: shape not served");
    CoarseSplit16Args A{};
    A.nq = nq; A.k = k; A.nch = (d + HK - 1) / HK;
    A.tiles_x = (k + MT2 - 1) / MT2; A.tiles_y = (nq + MT2 - 1) / MT2; A.total = A.tiles_x * A.tiles_y;
    const size_t rows_y = (size_t)A.tiles_y * MT2, rows_c = (size_t)A.tiles_x * MT2;
    const size_t row_bytes = (size_t)A.nch * 8 * sizeof(lut_u32x4);
    const size_t bytes = (rows_y + rows_c) * (row_bytes + sizeof(float)) + 256;
    const int rc = lut_ws_reserve(ctx, bytes);
    if (rc) return rc;
    lut_u32x4 *yh = (lut_u32x4 *)ctx->lut_ws, *ch = yh + rows_y * A.nch * 8;
    float *nyg = (float *)(ch + rows_c * A.nch * 8), *ncg = nyg + rows_y;
    unsigned int *maxbits = (unsigned int *)(ncg + rows_c);
    split16_clear_kernel<<<1, 64, 0, ctx->stream>>>(maxbits);
    split16_absmax_kernel<<<ctx->num_cu * 4, 256, 0, ctx->stream>>>(queries, (size_t)nq * d, cents, (size_t)k * d, maxbits);
    split16_prep_kernel<<<(unsigned)((rows_y + 31) / 32), 256, 0, ctx->stream>>>(queries, nq, (int)rows_y, d, A.nch, maxbits, yh, nyg);
    split16_prep_kernel<<<(unsigned)((rows_c + 31) / 32), 256, 0, ctx->stream>>>(cents, k, (int)rows_c, d, A.nch, maxbits + 1, ch, ncg);
    A.yh = yh; A.ch = ch; A.nyg = nyg; A.ncg = ncg; A.maxbits = maxbits;
    A.theta = theta; A.slot_keys = slot_keys; A.ov_keys = ov_keys; A.ov_cnt = ov_cnt; A.ov_cap = ov_cap;
    const int grid = (2 * ctx->num_cu + 7) / 8 * 8;
    coarse_split16_filter_kernel<<<grid, 512, 0, ctx->stream>>>(A);
    PQ_HIP(ctx, hipGetLastError());
#ifdef PQ_SCAN_TIMING
    {
        unsigned long long t[8] = {0};
        PQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
        PQ_HIP(ctx, hipMemcpyFromSymbol(t, HIP_SYMBOL(g_split16_ticks), sizeof(t)));
        fprintf(stderr, "split16 filter (wave ticks x 1e6): tile start %.1f stage %.1f multiply %.1f barrier %.1f end of tile %.1f\n", t[0] / 1e6,
                t[1] / 1e6, t[2] / 1e6, t[3] / 1e6, t[4] / 1e6);
        unsigned long long z[8] = {0};
        PQ_HIP(ctx, hipMemcpyToSymbol(HIP_SYMBOL(g_split16_ticks), z, sizeof(z)));
    }
#endif
    return PQ_OK;
}

// Number of 128 x 128 tiles from which the large form is used: two blocks for every compute unit.
// Rows of both operands and of the output must start on 16-byte boundaries (the output rows only
// where their length allows 16-byte stores at all) and hold a multiple of 4 dimensions.
static bool use_mfma128(pq_ctx *ctx, int64_t tiles, int d, int ds, const void *a, const void *b, const void *out) {
    const uintptr_t bits = (uintptr_t)a | (uintptr_t)b | (uintptr_t)out;
    return tiles >= 2 * (int64_t)ctx->num_cu && tiles < (1ll << 30) && (d & 3) == 0 && (ds & 3) == 0 && (bits & 15) == 0;
}

int launch_build_luts(pq_ctx *ctx, const float *queries, const float *codebooks, int nq, int d, int m, int k,
                      float *luts) {
    if (d / m >= 8 && opt_int(ctx, PQ_OPT_LUT_MFMA, 1) != 0) {
        const int64_t tx = (k + MT2 - 1) / MT2, ty = (nq + MT2 - 1) / MT2;
        if (use_mfma128(ctx, tx * ty * m, d, d / m, queries, codebooks, luts)) {
            return launch_mfma128<false>(ctx, queries, codebooks, nq, d, m, k, luts, (int)tx, (int)ty);
        }
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
    const int64_t tx2 = (d + MT2 - 1) / MT2, ty2 = (n + MT2 - 1) / MT2;
    if (d >= 8 && use_mfma128(ctx, tx2 * ty2, d, d, vectors, rot, out)) {
        return launch_mfma128<true>(ctx, vectors, rot, (int)n, d, 1, d, out, (int)tx2, (int)ty2);
    }
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
