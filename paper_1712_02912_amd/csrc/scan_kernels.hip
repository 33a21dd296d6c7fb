// Scan step: ADC over a contiguous code array with top-k selection (Alg. 1 `scan`/`adc`,
// Eq. (adc1); Alg. 3 `quick_adc_scan` for packed 4-bit codes with 8-bit tables).
//
// Work decomposition.  The code array is cut into chunks; the queries into groups of QB.
// One block (8 waves) scans one chunk for one group: the group's tables sit in LDS with the
// QB queries interleaved per entry, so that one LDS read of 16 bytes serves QB queries for
// the same code byte, and every code byte fetched from HBM is used QB times.  Each lane owns
// whole codes (one 16-byte load per iteration): row-major codes are already coalesced, no
// transposed block layout is needed.
//
// Top-k.  Each wave keeps, per query, a candidate buffer in device scratch and a threshold.
// A code is a candidate if its value is below the threshold; when a buffer is nearly full
// the wave selects its k smallest keys, keeps them and lowers its threshold to the k-th.
// Thresholds are shared (block LDS and a per-query device word, atomic min) so that waves
// and later blocks prune with the best bound known.  A bound learnt from another wave is
// the k-th smallest of a different subset: codes equal to it may still belong to the
// result, so foreign bounds prune with "<=" and the wave's own with "<" (the wave meets
// ids in increasing order, so a later code equal to its own k-th key can never replace it).
// At the end of the block the 8 wave lists of each query are merged to one list of k keys;
// a second kernel sorts the lists of all chunks of a query and writes the result.
#include "pq_internal.h"
#include "topk_device.h"

namespace pq {

constexpr int SCAN_WAVES = 8;
constexpr int SCAN_THREADS = SCAN_WAVES * 64;

struct ScanArgs {
    const uint8_t *codes;
    int64_t n;
    int64_t chunk_codes;   // multiple of the block tile
    int nchunks;
    int ngroups;
    const void *luts;      // [nq][m][k] f32 or u8
    int nq;
    int topk;
    uint32_t *tau_global;  // [ngroups*QB], ordered-value domain
    uint64_t *scratch;     // [nblocks][SCAN_WAVES][QB][CAP]
    uint64_t *partial;     // [nchunks*ngroups][QB][KPAD]
};

// ------------------------------------------------------------------------------------------
// Value traits: how the accumulated value of one (code, query) pair maps to the ordered
// 32-bit domain used in keys and shared thresholds.
struct F32Val {
    typedef float type;
    static __device__ __forceinline__ uint32_t to_ord(float v) { return f32_to_ord(v); }
    static __device__ __forceinline__ float from_ord(uint32_t o) { return ord_to_f32(o); }
    static __device__ __forceinline__ uint32_t ord_inf() { return f32_to_ord(__builtin_inff()); }
};
struct U32Val {
    typedef uint32_t type;
    static __device__ __forceinline__ uint32_t to_ord(uint32_t v) { return v; }
    static __device__ __forceinline__ uint32_t from_ord(uint32_t o) { return o; }
    static __device__ __forceinline__ uint32_t ord_inf() { return 0x7fffu; }  // above any sum of 16 bytes
};

// Per-wave selection state for QB queries.  Everything here is wave-uniform.
template <class V, int QB, int E>
struct WaveTopK {
    static constexpr int CAP = 64 * E;
    uint64_t *buf[QB];
    int cnt[QB];
    uint32_t own_ord[QB];            // k-th smallest value of the wave's own list (ord_inf if not full)
    typename V::type tau[QB];        // candidates satisfy value < tau
    int k;

    __device__ __forceinline__ void set_tau(int q, uint32_t shared_ord) {
        // foreign bound prunes with "<=": value < shared+1 in the ordered domain
        const uint32_t loose = shared_ord == 0xffffffffu ? shared_ord : shared_ord + 1u;
        const uint32_t eff = own_ord[q] < loose ? own_ord[q] : loose;
        tau[q] = V::from_ord(eff);
    }

    // insert the lanes with pass set; returns true if the wave's own bound changed
    __device__ __forceinline__ bool insert(int q, bool pass, typename V::type val, uint32_t id) {
        const uint64_t key = ((uint64_t)V::to_ord(val) << 32) | id;
        cnt[q] = wave_append(buf[q], cnt[q], pass, key);
        if (cnt[q] > CAP - 64) {
            const uint64_t kth = wave_compact<E>(buf[q], cnt[q], k);
            if (kth != KEY_EMPTY) {
                own_ord[q] = (uint32_t)(kth >> 32);
                return true;
            }
        }
        return false;
    }
};

// ------------------------------------------------------------------------------------------
// End of block: every wave has left at most k keys per query in its scratch list and its
// count in wave_cnt.  Wave q (q < QB) folds the 8 lists of query q into the list of wave 0
// and writes KPAD keys (padded with KEY_EMPTY) to `out`.
template <int QB, int E, int KPAD>
__device__ __forceinline__ void block_merge_lists(uint64_t *block_scratch, int (*wave_cnt)[QB], int k,
                                                   uint64_t *out_item) {
    constexpr int CAP = 64 * E;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    if (wave < QB) {
        const int q = wave;
        uint64_t *acc = block_scratch + (size_t)(0 * QB + q) * CAP;
        int cnt = wave_cnt[0][q];
        for (int w = 1; w < SCAN_WAVES; ++w) {
            const uint64_t *src = block_scratch + (size_t)(w * QB + q) * CAP;
            const int cw = wave_cnt[w][q];
            for (int i = lane; i < cw; i += 64) key_store(acc + cnt + i, key_load(src + i));
            cnt += cw;
            if (cnt > k) wave_compact<E>(acc, cnt, k);
        }
        __threadfence();
        uint64_t *out = out_item + (size_t)q * KPAD;
        for (int i = lane; i < KPAD; i += 64) out[i] = i < cnt ? key_load(acc + i) : KEY_EMPTY;
    }
}

// ------------------------------------------------------------------------------------------
// Float tables, one index per byte, 256 entries per table, MB = m = code bytes (8 or 16).
// LDS: lut4[j*256 + i] = the entries (j, i) of the block's 4 queries.
template <int MB, int E, int KPAD>
__global__ __launch_bounds__(SCAN_THREADS) void scan_f32_kernel(ScanArgs a) {
    constexpr int QB = 4;
    constexpr int CPL = 16 / MB;          // codes per lane per tile
    constexpr int TILE = 64 * CPL;        // codes per wave tile
    constexpr int CAP = 64 * E;
    extern __shared__ float4 lut4[];
    __shared__ uint32_t tau_blk[QB];
    __shared__ int wave_cnt[SCAN_WAVES][QB];

    const int group = blockIdx.x % a.ngroups;
    const int chunk = blockIdx.x / a.ngroups;
    const int wave = threadIdx.x >> 6, lane = lane_id();

    // stage the tables: global [q][j*256+i] -> LDS [(j*256+i)][q]; queries past nq get +inf
    {
        const float *luts = (const float *)a.luts;
        float *lds = (float *)lut4;
        for (int q = 0; q < QB; ++q) {
            const int gq = group * QB + q;
            for (int e = threadIdx.x; e < MB * 256; e += SCAN_THREADS)
                lds[e * QB + q] = gq < a.nq ? luts[(size_t)gq * (MB * 256) + e] : __builtin_inff();
        }
        if (threadIdx.x < QB) tau_blk[threadIdx.x] = a.tau_global[group * QB + threadIdx.x];
    }
    __syncthreads();

    WaveTopK<F32Val, QB, E> st;
    uint64_t *block_scratch = a.scratch + (size_t)blockIdx.x * SCAN_WAVES * QB * CAP;
    st.k = a.topk;
#pragma unroll
    for (int q = 0; q < QB; ++q) {
        st.buf[q] = block_scratch + (size_t)(wave * QB + q) * CAP;
        st.cnt[q] = 0;
        st.own_ord[q] = F32Val::ord_inf();
        st.set_tau(q, tau_blk[q]);
    }

    const int64_t cbeg = (int64_t)chunk * a.chunk_codes;
    const int64_t cend = cbeg + a.chunk_codes < a.n ? cbeg + a.chunk_codes : a.n;
    const int64_t ntiles = cend > cbeg ? (cend - cbeg + TILE - 1) / TILE : 0;

    auto load_tile = [&](int64_t t) -> uint4 {
        const int64_t first = cbeg + t * TILE + (int64_t)lane * CPL;   // first code of this lane
        uint4 c = make_uint4(0, 0, 0, 0);
        if (first + CPL <= cend) {
            c = *reinterpret_cast<const uint4 *>(a.codes + first * MB);
        } else if (CPL == 2 && first < cend) {
            const uint2 h = *reinterpret_cast<const uint2 *>(a.codes + first * MB);
            c.x = h.x; c.y = h.y;
        }
        return c;
    };

    uint4 cur = make_uint4(0, 0, 0, 0);
    if (wave < ntiles) cur = load_tile(wave);
    int iter = 0;
    for (int64_t t = wave; t < ntiles; t += SCAN_WAVES, ++iter) {
        uint4 nxt = make_uint4(0, 0, 0, 0);
        if (t + SCAN_WAVES < ntiles) nxt = load_tile(t + SCAN_WAVES);

        const uint32_t w[4] = {cur.x, cur.y, cur.z, cur.w};
        float d[CPL][QB];
#pragma unroll
        for (int h = 0; h < CPL; ++h) {
#pragma unroll
            for (int q = 0; q < QB; ++q) d[h][q] = 0.f;
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                const uint32_t word = w[h * (MB / 4) + j / 4];
                const uint32_t b = (word >> (8 * (j & 3))) & 255u;
                const float4 v = lut4[j * 256 + b];
                d[h][0] += v.x; d[h][1] += v.y; d[h][2] += v.z; d[h][3] += v.w;
            }
        }
        const int64_t first = cbeg + t * TILE + (int64_t)lane * CPL;
        bool any = false;
#pragma unroll
        for (int h = 0; h < CPL; ++h) {
            const bool valid = first + h < cend;
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                if (!valid) d[h][q] = __builtin_inff();
                any |= d[h][q] < st.tau[q];
            }
        }
        if (__ballot(any) != 0ull) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
#pragma unroll
                for (int h = 0; h < CPL; ++h) {
                    const bool pass = d[h][q] < st.tau[q];
                    if (__ballot(pass) != 0ull) {
                        if (st.insert(q, pass, d[h][q], (uint32_t)(first + h))) {
                            atomicMin(&tau_blk[q], st.own_ord[q]);
                            atomicMin(&a.tau_global[group * QB + q], st.own_ord[q]);
                            st.set_tau(q, tau_blk[q]);
                        }
                    }
                }
            }
        }
        if ((iter & 15) == 15) {   // pick up bounds found by other waves and blocks
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                uint32_t s = tau_blk[q];
                if ((iter & 63) == 63) {
                    const uint32_t g = __hip_atomic_load(&a.tau_global[group * QB + q], __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
                    if (g < s) { atomicMin(&tau_blk[q], g); s = g; }
                }
                st.set_tau(q, s);
            }
        }
        cur = nxt;
    }

#pragma unroll
    for (int q = 0; q < QB; ++q) {
        if (st.cnt[q] > st.k) wave_compact<E>(st.buf[q], st.cnt[q], st.k);
        if (lane == 0) wave_cnt[wave][q] = st.cnt[q];
    }
    __threadfence();
    __syncthreads();
    block_merge_lists<QB, E, KPAD>(block_scratch, wave_cnt, a.topk,
                                   a.partial + (size_t)blockIdx.x * QB * KPAD);
}

// ------------------------------------------------------------------------------------------
// 8-bit tables, packed 4-bit indexes, m = 16 (8 bytes per code), 8 queries per block.
// The 16 tables of 16 entries are merged in pairs when staged:
//   T[r][byte] = Q[2r][byte & 15] + Q[2r+1][byte >> 4]          (r < 8, byte < 256)
// so that one lookup per code byte gives the contribution of both nibbles; the integer
// sums are unchanged.  Entries are 16 bits; LDS holds tab[r*256 + byte] = 8 queries x u16
// (16 bytes), and the per-query sums (at most 16*255 = 4080) are accumulated as packed
// pairs of 16-bit fields in 32-bit adds, which cannot carry across fields.
template <int E, int KPAD>
__global__ __launch_bounds__(SCAN_THREADS) void scan_u4_kernel(ScanArgs a) {
    constexpr int QB = 8;
    constexpr int CPL = 2, TILE = 128;
    constexpr int CAP = 64 * E;
    __shared__ uint4 tab[8 * 256];
    __shared__ uint8_t qstage[QB][256];
    __shared__ uint32_t tau_blk[QB];
    __shared__ int wave_cnt[SCAN_WAVES][QB];

    const int group = blockIdx.x % a.ngroups;
    const int chunk = blockIdx.x / a.ngroups;
    const int wave = threadIdx.x >> 6, lane = lane_id();

    {
        const uint8_t *ql = (const uint8_t *)a.luts;
        for (int e = threadIdx.x; e < QB * 256; e += SCAN_THREADS) {
            const int q = e >> 8, gq = group * QB + q;
            qstage[q][e & 255] = gq < a.nq ? ql[(size_t)gq * 256 + (e & 255)] : 0;
        }
        if (threadIdx.x < QB) tau_blk[threadIdx.x] = a.tau_global[group * QB + threadIdx.x];
    }
    __syncthreads();
    {
        uint16_t *t16 = (uint16_t *)tab;
        for (int e = threadIdx.x; e < 8 * 256 * QB; e += SCAN_THREADS) {
            const int q = e & 7, byte = (e >> 3) & 255, r = e >> 11;
            const int gq = group * QB + q;
            const uint32_t s = (uint32_t)qstage[q][(2 * r) * 16 + (byte & 15)] +
                               (uint32_t)qstage[q][(2 * r + 1) * 16 + (byte >> 4)];
            t16[e] = gq < a.nq ? (uint16_t)s : (uint16_t)0x0fff;   // padded queries never qualify
        }
    }
    __syncthreads();

    WaveTopK<U32Val, QB, E> st;
    uint64_t *block_scratch = a.scratch + (size_t)blockIdx.x * SCAN_WAVES * QB * CAP;
    st.k = a.topk;
#pragma unroll
    for (int q = 0; q < QB; ++q) {
        st.buf[q] = block_scratch + (size_t)(wave * QB + q) * CAP;
        st.cnt[q] = 0;
        st.own_ord[q] = U32Val::ord_inf();
        st.set_tau(q, tau_blk[q]);
        if (group * QB + q >= a.nq) st.tau[q] = 0;
    }

    const int64_t cbeg = (int64_t)chunk * a.chunk_codes;
    const int64_t cend = cbeg + a.chunk_codes < a.n ? cbeg + a.chunk_codes : a.n;
    const int64_t ntiles = cend > cbeg ? (cend - cbeg + TILE - 1) / TILE : 0;

    auto load_tile = [&](int64_t t) -> uint4 {
        const int64_t first = cbeg + t * TILE + (int64_t)lane * CPL;
        uint4 c = make_uint4(0, 0, 0, 0);
        if (first + CPL <= cend) {
            c = *reinterpret_cast<const uint4 *>(a.codes + first * 8);
        } else if (first < cend) {
            const uint2 h = *reinterpret_cast<const uint2 *>(a.codes + first * 8);
            c.x = h.x; c.y = h.y;
        }
        return c;
    };

    uint4 cur = make_uint4(0, 0, 0, 0);
    if (wave < ntiles) cur = load_tile(wave);
    int iter = 0;
    for (int64_t t = wave; t < ntiles; t += SCAN_WAVES, ++iter) {
        uint4 nxt = make_uint4(0, 0, 0, 0);
        if (t + SCAN_WAVES < ntiles) nxt = load_tile(t + SCAN_WAVES);

        const uint32_t w[4] = {cur.x, cur.y, cur.z, cur.w};
        uint32_t acc[CPL][4];   // acc[h][p] = sums of queries 2p (low half) and 2p+1 (high half)
#pragma unroll
        for (int h = 0; h < CPL; ++h) {
#pragma unroll
            for (int p = 0; p < 4; ++p) acc[h][p] = 0;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint32_t word = w[h * 2 + r / 4];
                const uint32_t b = (word >> (8 * (r & 3))) & 255u;
                const uint4 v = tab[r * 256 + b];
                acc[h][0] += v.x; acc[h][1] += v.y; acc[h][2] += v.z; acc[h][3] += v.w;
            }
        }
        const int64_t first = cbeg + t * TILE + (int64_t)lane * CPL;
        // fast test on packed fields: (x | 0x8000) - tau keeps bit 15 iff x >= tau
        uint32_t allge = 0x80008000u;
#pragma unroll
        for (int h = 0; h < CPL; ++h) {
            const bool valid = first + h < cend;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (!valid) acc[h][p] = 0x7fff7fffu;
                const uint32_t taupk = st.tau[2 * p] | (st.tau[2 * p + 1] << 16);
                allge &= (acc[h][p] | 0x80008000u) - taupk;
            }
        }
        const bool any = (allge & 0x80008000u) != 0x80008000u;
        if (__ballot(any) != 0ull) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
#pragma unroll
                for (int h = 0; h < CPL; ++h) {
                    const uint32_t x = (acc[h][q >> 1] >> (16 * (q & 1))) & 0xffffu;
                    const bool pass = x < st.tau[q];
                    if (__ballot(pass) != 0ull) {
                        if (st.insert(q, pass, x, (uint32_t)(first + h))) {
                            atomicMin(&tau_blk[q], st.own_ord[q]);
                            atomicMin(&a.tau_global[group * QB + q], st.own_ord[q]);
                            st.set_tau(q, tau_blk[q]);
                        }
                    }
                }
            }
        }
        if ((iter & 15) == 15) {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                uint32_t s = tau_blk[q];
                if ((iter & 63) == 63) {
                    const uint32_t g = __hip_atomic_load(&a.tau_global[group * QB + q], __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
                    if (g < s) { atomicMin(&tau_blk[q], g); s = g; }
                }
                if (group * QB + q < a.nq) st.set_tau(q, s);
            }
        }
        cur = nxt;
    }

#pragma unroll
    for (int q = 0; q < QB; ++q) {
        if (st.cnt[q] > st.k) wave_compact<E>(st.buf[q], st.cnt[q], st.k);
        if (lane == 0) wave_cnt[wave][q] = st.cnt[q];
    }
    __threadfence();
    __syncthreads();
    block_merge_lists<QB, E, KPAD>(block_scratch, wave_cnt, a.topk,
                                   a.partial + (size_t)blockIdx.x * QB * KPAD);
}

// ------------------------------------------------------------------------------------------
// General kernel: any m, k with m*k <= 8192 entries, float or 8-bit tables, either code
// format, one query per block.  Used for shapes outside the two tuned kernels.
template <bool LUT_U8, int E, int KPAD>
__global__ __launch_bounds__(SCAN_THREADS) void scan_generic_kernel(ScanArgs a, int m, int k, int cf) {
    constexpr int QB = 1;
    constexpr int CAP = 64 * E;
    typedef typename std::conditional<LUT_U8, U32Val, F32Val>::type V;
    __shared__ float lutf[8192];
    __shared__ uint32_t tau_blk[QB];
    __shared__ int wave_cnt[SCAN_WAVES][QB];

    const int group = blockIdx.x % a.ngroups;   // = query
    const int chunk = blockIdx.x / a.ngroups;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int cb = cf == PQ_CODES_U4_PACKED ? m / 2 : m;
    uint32_t *lutu = (uint32_t *)lutf;

    for (int e = threadIdx.x; e < m * k; e += SCAN_THREADS) {
        if (LUT_U8) lutu[e] = ((const uint8_t *)a.luts)[(size_t)group * m * k + e];
        else lutf[e] = ((const float *)a.luts)[(size_t)group * m * k + e];
    }
    if (threadIdx.x < QB) tau_blk[threadIdx.x] = a.tau_global[group];
    __syncthreads();

    WaveTopK<V, QB, E> st;
    uint64_t *block_scratch = a.scratch + (size_t)blockIdx.x * SCAN_WAVES * QB * CAP;
    st.k = a.topk;
    st.buf[0] = block_scratch + (size_t)wave * CAP;
    st.cnt[0] = 0;
    st.own_ord[0] = V::ord_inf();
    if (LUT_U8) st.own_ord[0] = 0xfffffffeu;   // sums of up to 8192 bytes exceed the 16-bit bound of the packed kernel
    st.set_tau(0, tau_blk[0]);

    const int64_t cbeg = (int64_t)chunk * a.chunk_codes;
    const int64_t cend = cbeg + a.chunk_codes < a.n ? cbeg + a.chunk_codes : a.n;
    int iter = 0;
    for (int64_t base = cbeg + (int64_t)wave * 64; base < cend; base += SCAN_WAVES * 64, ++iter) {
        const int64_t i = base + lane;
        const bool valid = i < cend;
        typename V::type val = 0;
        if (valid) {
            const uint8_t *c = a.codes + i * cb;
            for (int j = 0; j < m; ++j) {
                int idx;
                if (cf == PQ_CODES_U4_PACKED) {
                    const uint32_t byte = c[j >> 1];
                    idx = (j & 1) ? (byte >> 4) : (byte & 15u);
                } else {
                    idx = c[j];
                }
                if (idx < k) {
                    if (LUT_U8) val += lutu[j * k + idx]; else val += lutf[j * k + idx];
                }
            }
        }
        const bool pass = valid && val < st.tau[0];
        if (__ballot(pass) != 0ull) {
            if (st.insert(0, pass, val, (uint32_t)i)) {
                atomicMin(&tau_blk[0], st.own_ord[0]);
                atomicMin(&a.tau_global[group], st.own_ord[0]);
                st.set_tau(0, tau_blk[0]);
            }
        }
        if ((iter & 15) == 15) {
            uint32_t s = tau_blk[0];
            if ((iter & 63) == 63) {
                const uint32_t g = __hip_atomic_load(&a.tau_global[group], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (g < s) { atomicMin(&tau_blk[0], g); s = g; }
            }
            st.set_tau(0, s);
        }
    }
    if (st.cnt[0] > st.k) wave_compact<E>(st.buf[0], st.cnt[0], st.k);
    if (lane == 0) wave_cnt[wave][0] = st.cnt[0];
    __threadfence();
    __syncthreads();
    block_merge_lists<QB, E, KPAD>(block_scratch, wave_cnt, a.topk, a.partial + (size_t)blockIdx.x * QB * KPAD);
}

// ------------------------------------------------------------------------------------------
__global__ void init_tau_kernel(uint32_t *tau, int count, uint32_t value) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) tau[i] = value;
}

// One block per query: gather the KPAD-key lists of all chunks, sort, write the first topk.
template <bool VAL_U32>
__global__ __launch_bounds__(1024) void merge_topk_kernel(const uint64_t *partial, int nchunks, int ngroups, int qb,
                                                           int kpad, int n2, int topk, void *out_val,
                                                           int64_t *out_ids) {
    extern __shared__ uint64_t skeys[];
    const int gq = blockIdx.x, group = gq / qb, q = gq % qb;
    const int total = nchunks * kpad;
    for (int i = threadIdx.x; i < n2; i += blockDim.x) {
        uint64_t key = KEY_EMPTY;
        if (i < total) {
            const int c = i / kpad, e = i % kpad;
            key = partial[((size_t)(c * ngroups + group) * qb + q) * kpad + e];
        }
        skeys[i] = key;
    }
    block_bitonic_sort(skeys, n2);
    for (int i = threadIdx.x; i < topk; i += blockDim.x) {
        const uint64_t key = skeys[i];
        const bool empty = key == KEY_EMPTY;
        if (VAL_U32) ((uint32_t *)out_val)[(size_t)gq * topk + i] = empty ? 0xffffffffu : (uint32_t)(key >> 32);
        else ((float *)out_val)[(size_t)gq * topk + i] = empty ? __builtin_inff() : ord_to_f32((uint32_t)(key >> 32));
        out_ids[(size_t)gq * topk + i] = empty ? -1 : (int64_t)(uint32_t)key;
    }
}

// ------------------------------------------------------------------------------------------
static int next_pow2(int x) { int p = 1; while (p < x) p <<= 1; return p; }

static int env_int(const char *name, int dflt) {
    const char *s = getenv(name);
    return s && *s ? atoi(s) : dflt;
}

template <class Launch>
static int run_scan(pq_ctx *ctx, const uint8_t *codes, int64_t n, const void *luts, int nq, int topk, int qb,
                    int tile_codes, int kpad, int cap, bool val_u32, uint32_t tau_init, void *out_val,
                    int64_t *out_ids, Launch launch) {
    const int ngroups = (nq + qb - 1) / qb;
    const int64_t block_tile = (int64_t)tile_codes * SCAN_WAVES;
    // enough blocks to keep every CU busy for several rounds, but chunks of at least 8 block tiles
    const int target_blocks = env_int("PQ_SCAN_TARGET_BLOCKS", 16 * ctx->num_cu);
    int64_t nchunks = (target_blocks + ngroups - 1) / ngroups;
    const int64_t max_by_n = (n + 8 * block_tile - 1) / (8 * block_tile);
    const int64_t max_by_merge = 16384 / kpad;
    if (nchunks > max_by_n) nchunks = max_by_n;
    if (nchunks > max_by_merge) nchunks = max_by_merge;
    if (env_int("PQ_SCAN_CHUNKS", 0) > 0) nchunks = env_int("PQ_SCAN_CHUNKS", 0);
    if (nchunks > max_by_merge) nchunks = max_by_merge;
    if (nchunks < 1) nchunks = 1;
    int64_t chunk_codes = (n + nchunks - 1) / nchunks;
    chunk_codes = (chunk_codes + block_tile - 1) / block_tile * block_tile;
    if (chunk_codes < block_tile) chunk_codes = block_tile;
    nchunks = n > 0 ? (n + chunk_codes - 1) / chunk_codes : 1;
    const int64_t nblocks = nchunks * ngroups;
    if (nblocks > 0x7fffffff) return fail(ctx, PQ_EUNSUPPORTED, "scan grid too large (%lld blocks)", (long long)nblocks);

    const size_t tau_bytes = align_up((size_t)ngroups * qb * sizeof(uint32_t), 256);
    const size_t scratch_bytes = (size_t)nblocks * SCAN_WAVES * qb * cap * sizeof(uint64_t);
    const size_t partial_bytes = (size_t)nblocks * qb * kpad * sizeof(uint64_t);
    int rc = ws_reserve(ctx, tau_bytes + scratch_bytes + partial_bytes);
    if (rc) return rc;
    uint8_t *ws = (uint8_t *)ctx->ws;

    ScanArgs a;
    a.codes = codes; a.n = n; a.chunk_codes = chunk_codes; a.nchunks = (int)nchunks; a.ngroups = ngroups;
    a.luts = luts; a.nq = nq; a.topk = topk;
    a.tau_global = (uint32_t *)ws;
    a.scratch = (uint64_t *)(ws + tau_bytes);
    a.partial = (uint64_t *)(ws + tau_bytes + scratch_bytes);

    const int ntau = ngroups * qb;
    init_tau_kernel<<<(ntau + 255) / 256, 256, 0, ctx->stream>>>(a.tau_global, ntau, tau_init);
    PQ_HIP(ctx, hipGetLastError());
    if (ctx->profiling) PQ_HIP(ctx, hipEventRecord(ctx->ev_begin, ctx->stream));
    rc = launch(a, (int)nblocks);
    if (rc) return rc;
    if (ctx->profiling) {
        PQ_HIP(ctx, hipEventRecord(ctx->ev_end, ctx->stream));
        ctx->ev_valid = 1;
    }
    const int n2 = next_pow2((int)nchunks * kpad);
    const int mthreads = n2 / 2 < 1024 ? (n2 / 2 < 64 ? 64 : n2 / 2) : 1024;
    if (val_u32)
        merge_topk_kernel<true><<<nq, mthreads, (size_t)n2 * 8, ctx->stream>>>(a.partial, (int)nchunks, ngroups, qb, kpad, n2, topk, out_val, out_ids);
    else
        merge_topk_kernel<false><<<nq, mthreads, (size_t)n2 * 8, ctx->stream>>>(a.partial, (int)nchunks, ngroups, qb, kpad, n2, topk, out_val, out_ids);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

template <class K>
static int set_lds(pq_ctx *ctx, K kernel, size_t bytes) {
    PQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return PQ_OK;
}

int launch_scan(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const void *luts, int lf, int nq, int m, int k,
                int topk, void *out_val, int64_t *out_ids) {
    const bool small = topk <= 128;
    const int kpad = small ? 128 : 1024;
    const int cap = 2 * kpad;
    hipStream_t s = ctx->stream;
    {
        int rc = set_lds(ctx, merge_topk_kernel<true>, 131072);
        if (!rc) rc = set_lds(ctx, merge_topk_kernel<false>, 131072);
        if (rc) return rc;
    }
    if (cf == PQ_CODES_U8 && lf == PQ_LUT_F32 && k == 256 && (m == 8 || m == 16)) {
        const size_t lds = (size_t)m * 256 * 16;
        auto launch = [&](const ScanArgs &a, int nblocks) -> int {
#define PQ_LAUNCH_F32(MB, E, KP)                                                                  \
    do {                                                                                          \
        int rc_ = set_lds(ctx, scan_f32_kernel<MB, E, KP>, lds);                                  \
        if (rc_) return rc_;                                                                      \
        scan_f32_kernel<MB, E, KP><<<nblocks, SCAN_THREADS, lds, s>>>(a);                         \
    } while (0)
            if (m == 8) { if (small) PQ_LAUNCH_F32(8, 4, 128); else PQ_LAUNCH_F32(8, 32, 1024); }
            else { if (small) PQ_LAUNCH_F32(16, 4, 128); else PQ_LAUNCH_F32(16, 32, 1024); }
#undef PQ_LAUNCH_F32
            PQ_HIP(ctx, hipGetLastError());
            return PQ_OK;
        };
        return run_scan(ctx, codes, n, luts, nq, topk, 4, m == 8 ? 128 : 64, kpad, cap, false,
                        0xff800000u /* ordered +inf */, out_val, out_ids, launch);
    }
    if (cf == PQ_CODES_U4_PACKED && lf == PQ_LUT_U8 && k == 16 && m == 16) {
        auto launch = [&](const ScanArgs &a, int nblocks) -> int {
            if (small) scan_u4_kernel<4, 128><<<nblocks, SCAN_THREADS, 0, s>>>(a);
            else scan_u4_kernel<32, 1024><<<nblocks, SCAN_THREADS, 0, s>>>(a);
            PQ_HIP(ctx, hipGetLastError());
            return PQ_OK;
        };
        return run_scan(ctx, codes, n, luts, nq, topk, 8, 128, kpad, cap, true, 0x7fffu, out_val, out_ids, launch);
    }
    if ((int64_t)m * k <= 8192) {
        const bool u8 = lf == PQ_LUT_U8;
        auto launch = [&](const ScanArgs &a, int nblocks) -> int {
            if (u8) {
                if (small) scan_generic_kernel<true, 4, 128><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
                else scan_generic_kernel<true, 32, 1024><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
            } else {
                if (small) scan_generic_kernel<false, 4, 128><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
                else scan_generic_kernel<false, 32, 1024><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
            }
            PQ_HIP(ctx, hipGetLastError());
            return PQ_OK;
        };
        return run_scan(ctx, codes, n, luts, nq, topk, 1, 64, kpad, cap, u8, u8 ? 0xfffffffeu : 0xff800000u, out_val,
                        out_ids, launch);
    }
    return fail(ctx, PQ_EUNSUPPORTED, "scan: no kernel for m=%d k=%d code_fmt=%d lut_fmt=%d", m, k, cf, lf);
}

}  // namespace pq
