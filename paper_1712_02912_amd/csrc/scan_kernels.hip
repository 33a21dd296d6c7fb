// Scan step (Alg. 1 `scan`/`adc`, Eq. (adc1)): the general kernel for shapes outside the tuned
// ones, the kernel that merges the per-block candidate lists into the final top-k, and the
// dispatcher behind pq_adc_scan_topk.
//
// Top-k in the general kernel.  Each wave keeps a candidate buffer in device scratch and a
// threshold.  A code is a candidate if its value is below the threshold; when the buffer is
// nearly full the wave selects its k smallest keys, keeps them and lowers its threshold to the
// k-th.  Thresholds are shared (block LDS and a per-query device word, atomic min).  A bound
// learnt from another wave is the k-th smallest of a different subset: codes equal to it may
// still belong to the result, so foreign bounds prune with "<=" and the wave's own with "<"
// (the wave meets ids in increasing order, so a later code equal to its own k-th key can never
// replace it).  At the end of the block the 8 wave lists are merged to one list of k keys; the
// merge kernel sorts the lists of all chunks of a query and writes the result.
#include <type_traits>

#include "pq_internal.h"
#include "scan_common.h"
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
        list_fence();
        uint64_t *out = out_item + (size_t)q * KPAD;
        for (int i = lane; i < KPAD; i += 64) out[i] = i < cnt ? key_load(acc + i) : KEY_EMPTY;
    }
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
    list_fence();
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

// One block per query: the k smallest keys over all result lists of the query, for scans that
// leave a final bound per query (at least k keys are at or below it): keys above the bound cannot
// be in the result and are dropped before the sort, so the number of lists is not limited by the
// sort.  The lists of query gq are either lists qlist_off[gq] .. qlist_off[gq + 1] of `partial`
// (inverted-list search) or, with qlist_off == nullptr, list (c * ngroups + gq / qb) * qb + gq % qb
// for every chunk c (flat scan).  ids (optional) maps rows to the ids to return.
// MERGE_CAP keys are kept in LDS (more than that at or below the bound: the bisection below).  Calls of few queries
// give every query a block of 1024 threads and room for 8192 keys; calls of many queries take blocks of 256 threads
// and 2048 keys (512 threads and 4096 keys for topk above 512), of which a compute unit holds several.
constexpr int merge_lds_bytes(int cap) { return cap * 8 + cap * 4 + 1024 * 8; }   // kept keys, 32-bit values for the selection, the result's keys
template <bool VAL_U32, int MERGE_CAP>
__global__ __launch_bounds__(1024) void merge_filtered_kernel(const uint64_t *__restrict__ partial,
                                                              const uint32_t *__restrict__ qlist_off, int nchunks,
                                                              int ngroups, int qb,
                                                              const unsigned long long *__restrict__ tau_key, int kpad, int topk,
                                                              const int64_t *__restrict__ ids, void *out_val,
                                                              int64_t *out_ids) {
    extern __shared__ uint64_t skeys[];
    __shared__ int s_count;
    const int gq = blockIdx.x, tid = threadIdx.x;
    const size_t nlists = qlist_off ? (size_t)(qlist_off[gq + 1] - qlist_off[gq]) : (size_t)nchunks;
    // Every list is packed (its keys first, KEY_EMPTY behind them; kpad is a multiple of 64): a wave
    // takes whole lists, 64 keys at a time, and leaves a list at the first empty slot it sees.
    const int wave = tid >> 6, lane = tid & 63, nwaves = (int)(blockDim.x >> 6);
    // (the first 64 keys of four lists are requested together: a walk over a thousand short lists is otherwise a
    // chain of memory round trips)
    auto list_ptr = [&](size_t l) {
        const size_t list = qlist_off ? (size_t)qlist_off[gq] + l : (l * ngroups + gq / qb) * qb + gq % qb;
        return partial + list * kpad;
    };
    auto for_each_key = [&](auto &&f) {
        constexpr int MLP = 4;
        for (size_t l0 = wave; l0 < nlists; l0 += (size_t)MLP * nwaves) {
            const uint64_t *lp[MLP];
            uint64_t first[MLP];
#pragma unroll
            for (int u = 0; u < MLP; ++u) {
                const size_t l = l0 + (size_t)u * nwaves;
                lp[u] = l < nlists ? list_ptr(l) : nullptr;
                first[u] = lp[u] ? lp[u][lane] : KEY_EMPTY;
            }
#pragma unroll
            for (int u = 0; u < MLP; ++u) {
                if (lp[u] == nullptr) continue;
                uint64_t key = first[u];
                for (int e0 = 0;;) {
                    f(key);
                    e0 += 64;
                    if (__ballot(key == KEY_EMPTY) != 0ull || e0 >= kpad) break;
                    key = lp[u][e0 + lane];
                }
            }
        }
    };
    const uint64_t tau_k = tau_key[gq];   // a whole key at or below which k keys exist (rows separate ties of the value)
    if (tid == 0) s_count = 0;
    __syncthreads();
    for_each_key([&](uint64_t key) {
        if (key != KEY_EMPTY && key <= tau_k) {
            const int pos = atomicAdd(&s_count, 1);
            if (pos < MERGE_CAP) skeys[pos] = key;
        }
    });
    __syncthreads();
    int kept = s_count;
    if (kept > MERGE_CAP) {
        // too many keys at or below the bound (massive ties): the topk-th key by radix selection, one byte of the key per
        // pass over the lists, most significant first
        __shared__ uint32_t key_bins[256];
        __shared__ unsigned long long sel_prefix;
        __shared__ uint32_t sel_want;
        if (tid == 0) { sel_prefix = 0ull; sel_want = (uint32_t)topk; }
        for (int pass = 7; pass >= 0; --pass) {
            if (tid < 256) key_bins[tid] = 0u;
            __syncthreads();
            const int shift = 8 * pass;
            const uint64_t fixed = pass == 7 ? 0ull : ~0ull << (shift + 8);   // bytes decided in earlier passes
            const uint64_t prefix = sel_prefix;
            const uint32_t want = sel_want;
            for_each_key([&](uint64_t key) {
                if (key != KEY_EMPTY && (key & fixed) == prefix) atomicAdd(&key_bins[(uint32_t)(key >> shift) & 255u], 1u);
            });
            __syncthreads();
            if (tid < 64) {   // one wave: the byte value whose bin holds the `want`-th key
                const uint32_t h[4] = {key_bins[4 * tid], key_bins[4 * tid + 1], key_bins[4 * tid + 2], key_bins[4 * tid + 3]};
                const uint32_t tot = h[0] + h[1] + h[2] + h[3];
                uint32_t incl = tot;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t up = __shfl_up(incl, o);
                    if (tid >= o) incl += up;
                }
                const uint64_t reach = __ballot(incl >= want);   // never empty: more than topk keys lie at or below the bound
                if (reach != 0ull && tid == __builtin_ctzll(reach)) {
                    uint32_t cum = incl - tot;
                    int bsel = 4 * tid;
                    for (int t = 0; t < 3 && cum + h[t] < want; ++t) { cum += h[t]; ++bsel; }
                    sel_prefix = prefix | ((uint64_t)bsel << shift);
                    sel_want = want - cum;
                }
            }
            __syncthreads();
        }
        if (tid == 0) s_count = 0;
        __syncthreads();
        const uint64_t kth = sel_prefix;
        for_each_key([&](uint64_t key) {
            if (key != KEY_EMPTY && key <= kth) { const int pos = atomicAdd(&s_count, 1); if (pos < MERGE_CAP) skeys[pos] = key; }
        });
        __syncthreads();
        kept = s_count < MERGE_CAP ? s_count : MERGE_CAP;
    }
    auto emit = [&](int i, uint64_t key) {
        const bool empty = key == KEY_EMPTY;
        const uint32_t row = (uint32_t)key;
        if (VAL_U32) ((uint32_t *)out_val)[(size_t)gq * topk + i] = empty ? 0xffffffffu : (uint32_t)(key >> 32);
        else ((float *)out_val)[(size_t)gq * topk + i] = empty ? __builtin_inff() : ord_to_f32((uint32_t)(key >> 32));
        out_ids[(size_t)gq * topk + i] = empty ? -1 : (ids ? ids[row] : (int64_t)row);
    };
    // The topk smallest of the kept keys without sorting them all (a bitonic sort of a few thousand keys is dozens of
    // barrier stages): radix selection of the topk-th value, then of the row among the keys that tie with it, gives the
    // topk-th key; the keys up to it are moved to a short list, where every thread finds the rank of its keys by
    // counting the smaller ones and writes them straight to their places.
    uint32_t *vals = reinterpret_cast<uint32_t *>(skeys + MERGE_CAP);          // [MERGE_CAP]
    uint64_t *shortlist = skeys + MERGE_CAP + MERGE_CAP / 2;                   // [1024]
    __shared__ uint32_t sel_bins[256], sel_state[2];
    __shared__ int s_below, s_ties;
    int nshort = kept;
    const uint64_t *src = skeys;
    if (kept > topk) {
        for (int i = tid; i < kept; i += blockDim.x) vals[i] = (uint32_t)(skeys[i] >> 32);
        if (tid == 0) { s_below = 0; s_ties = 0; s_count = 0; }
        __syncthreads();
        const uint32_t vk = block_kth_smallest_u32(vals, kept, (uint32_t)topk, sel_bins, sel_state);
        // rows of the keys that tie with the topk-th value (into vals, which has served its purpose), keys below it counted
        __syncthreads();
        int below = 0;
        for (int i = tid; i < kept; i += blockDim.x) {
            const uint32_t v = (uint32_t)(skeys[i] >> 32);
            below += v < vk ? 1 : 0;
        }
        atomicAdd(&s_below, below);
        __syncthreads();
        for (int i = tid; i < kept; i += blockDim.x)
            if ((uint32_t)(skeys[i] >> 32) == vk) vals[atomicAdd(&s_ties, 1)] = (uint32_t)skeys[i];
        __syncthreads();
        const uint32_t rk = block_kth_smallest_u32(vals, s_ties, (uint32_t)(topk - s_below), sel_bins, sel_state);
        const uint64_t kth = ((uint64_t)vk << 32) | rk;
        __syncthreads();
        for (int i = tid; i < kept; i += blockDim.x)
            if (skeys[i] <= kth) shortlist[atomicAdd(&s_count, 1)] = skeys[i];   // exactly topk keys (keys are distinct)
        __syncthreads();
        nshort = s_count;
        src = shortlist;
    }
    if (nshort > 256) {
        // long results: counting the smaller keys is nshort^2 broadcast reads (a thousand keys: 40 us of LDS time on a
        // compute unit that holds four such blocks); the short list is sorted instead (at most 1024 keys: 55 stages)
        uint64_t *buf = kept > topk ? shortlist : skeys;   // (nshort <= topk <= 1024 either way)
        int n2 = 512;
        while (n2 < nshort) n2 <<= 1;
        for (int i = nshort + tid; i < n2; i += blockDim.x) buf[i] = KEY_EMPTY;
        block_bitonic_sort(buf, n2);
        for (int i = tid; i < topk; i += blockDim.x) emit(i, i < nshort ? buf[i] : KEY_EMPTY);
        return;
    }
    for (int i = tid; i < nshort; i += blockDim.x) {
        const uint64_t mine = src[i];
        int rank = 0;
        for (int j = 0; j < nshort; ++j) rank += src[j] < mine ? 1 : 0;
        if (rank < topk) emit(rank, mine);
    }
    for (int i = nshort + tid; i < topk; i += blockDim.x) emit(i, KEY_EMPTY);
}

int launch_merge_filtered(pq_ctx *ctx, const uint64_t *partial, const uint32_t *qlist_off, int nchunks, int ngroups, int qb,
                          const unsigned long long *tau_key, int kpad, int nq, int topk, const int64_t *ids, bool val_u32,
                          void *out_val, int64_t *out_ids) {
    if (nq == 0) return PQ_OK;
    auto launch = [&](auto kernel, int cap, int threads) -> int {
        PQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, merge_lds_bytes(cap)));
        kernel<<<nq, threads, merge_lds_bytes(cap), ctx->stream>>>(partial, qlist_off, nchunks, ngroups, qb, tau_key, kpad, topk, ids, out_val, out_ids);
        PQ_HIP(ctx, hipGetLastError());
        return PQ_OK;
    };
    // calls of many queries: several smaller blocks per compute unit (room for at least four times topk keys)
    const bool many = nq >= 2 * ctx->num_cu;
    if (many && topk <= 512) {
        if (val_u32) return launch(merge_filtered_kernel<true, 2048>, 2048, 256);
        return launch(merge_filtered_kernel<false, 2048>, 2048, 256);
    }
    if (many) {
        if (val_u32) return launch(merge_filtered_kernel<true, 4096>, 4096, 512);
        return launch(merge_filtered_kernel<false, 4096>, 4096, 512);
    }
    if (val_u32) return launch(merge_filtered_kernel<true, 8192>, 8192, 1024);
    return launch(merge_filtered_kernel<false, 8192>, 8192, 1024);
}

// ------------------------------------------------------------------------------------------
static int next_pow2(int x) { int p = 1; while (p < x) p <<= 1; return p; }

int launch_merge_topk(pq_ctx *ctx, const uint64_t *partial, int nchunks, int ngroups, int qb, int kpad, int nq,
                      int topk, bool val_u32, void *out_val, int64_t *out_ids) {
    const int n2 = next_pow2(nchunks * kpad);
    if (n2 > 16384) return fail(ctx, PQ_EUNSUPPORTED, "merge: %d keys per query exceed the LDS sort", n2);
    const int mthreads = n2 / 2 < 1024 ? (n2 / 2 < 64 ? 64 : n2 / 2) : 1024;
    if (val_u32) {
        PQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(merge_topk_kernel<true>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
        merge_topk_kernel<true><<<nq, mthreads, (size_t)n2 * 8, ctx->stream>>>(partial, nchunks, ngroups, qb, kpad, n2,
                                                                               topk, out_val, out_ids);
    } else {
        PQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(merge_topk_kernel<false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
        merge_topk_kernel<false><<<nq, mthreads, (size_t)n2 * 8, ctx->stream>>>(partial, nchunks, ngroups, qb, kpad, n2,
                                                                                topk, out_val, out_ids);
    }
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

// General kernel: one block per (chunk, query).
static int run_generic(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const void *luts, bool lut_u8, int nq,
                       int m, int k, int topk, void *out_val, int64_t *out_ids) {
    const bool small = topk <= 128;
    const int kpad = small ? 128 : 1024, cap = 2 * kpad, qb = 1;
    const int ngroups = nq;
    const int64_t block_tile = 64 * SCAN_WAVES;
    // enough blocks to keep every CU busy for several rounds, but chunks of at least 8 block tiles
    int64_t nchunks = (16 * ctx->num_cu + ngroups - 1) / ngroups;
    const int64_t max_by_n = (n + 8 * block_tile - 1) / (8 * block_tile);
    const int64_t max_by_merge = 16384 / kpad;
    if (nchunks > max_by_n) nchunks = max_by_n;
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
    init_tau_kernel<<<(ntau + 255) / 256, 256, 0, ctx->stream>>>(a.tau_global, ntau,
                                                                 lut_u8 ? 0xfffffffeu : 0xff800000u /* ordered +inf */);
    PQ_HIP(ctx, hipGetLastError());
    if (ctx->profiling) {
        note_plain_scan(ctx, "scan_generic_kernel (one query per block)", 1, nq);
        PQ_HIP(ctx, hipEventRecord(ctx->ev_begin, ctx->stream));
    }
    hipStream_t s = ctx->stream;
    if (lut_u8) {
        if (small) scan_generic_kernel<true, 4, 128><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
        else scan_generic_kernel<true, 32, 1024><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
    } else {
        if (small) scan_generic_kernel<false, 4, 128><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
        else scan_generic_kernel<false, 32, 1024><<<nblocks, SCAN_THREADS, 0, s>>>(a, m, k, cf);
    }
    PQ_HIP(ctx, hipGetLastError());
    if (ctx->profiling) {
        PQ_HIP(ctx, hipEventRecord(ctx->ev_end, ctx->stream));
        ctx->ev_valid = 1;
    }
    return launch_merge_topk(ctx, a.partial, (int)nchunks, ngroups, qb, kpad, nq, topk, lut_u8, out_val, out_ids);
}

int launch_scan(pq_ctx *ctx, const uint8_t *codes, int64_t n, int cf, const void *luts, int lf, int nq, int m, int k,
                int topk, void *out_val, int64_t *out_ids) {
    const bool general = opt_int(ctx, PQ_OPT_SCAN_FORCE_GENERAL, 0) != 0;
    if (!general && cf == PQ_CODES_U8 && lf == PQ_LUT_F32 && k == 256 && (m == 8 || m == 16))
        return w16::launch_scan_tuned(ctx, m == 8 ? 0 : 1, codes, n, luts, nq, topk, out_val, out_ids);
    if (!general && cf == PQ_CODES_U4_PACKED && lf == PQ_LUT_U8 && k == 16 && m == 16)
        return w16::launch_scan_tuned(ctx, 2, codes, n, luts, nq, topk, out_val, out_ids);
    if ((int64_t)m * k <= 8192)
        return run_generic(ctx, codes, n, cf, luts, lf == PQ_LUT_U8, nq, m, k, topk, out_val, out_ids);
    return fail(ctx, PQ_EUNSUPPORTED, "scan: no kernel for m=%d k=%d code_fmt=%d lut_fmt=%d", m, k, cf, lf);
}

}  // namespace pq
