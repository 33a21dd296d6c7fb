// IVFADC search (Section 2.3.2; Index, Tables and Scan steps of Section 2.3.3).
//
// Per batch of queries:
//   Index   distances from every query to the nlist coarse centroids (the Tables kernel with
//           one "sub-space" covering all d dimensions), then the nprobe smallest (distance,
//           list id) per query by a histogram select;
//   Tables  residual y - centroid_l for each (query, probed list) pair and its m tables,
//           Eq. (tables), materialised in the workspace;
//   Scan    the pairs are grouped by list, every list is cut into chunks, and one work item
//           = one chunk x up to 4 of the queries probing that list.  Items are ordered by
//           list size class (largest first) and run by the persistent scan kernel; each
//           (pair, chunk) leaves a list of k keys, and a merge kernel picks the k best of all
//           lists of a query.  Bounds and candidate histograms are per query, so what one
//           list establishes prunes the other lists of the same query.
// Everything is sized from upper bounds, so the call enqueues without reading back from the
// device.
#include <string.h>

#include "pq_internal.h"
#include "scan_common.h"
#include "topk_device.h"
#include "lds_walk.h"

namespace pq {

constexpr int IVF_MAX_CHUNKS = 16;            // chunks per list (bounds the lists a query can own)
constexpr int64_t IVF_CHUNK_TARGET = 1 << 18; // rows per chunk aimed at for long lists
// Quick ADC: chunks of at most 2^20 rows, as many as the list needs.  The lists of a query are distinct, so a query owns
// at most nprobe + ntotal / 2^20 chunks whatever it probes: about as many result lists as the cap above allows, and
// no work item is longer than 2^20 rows (an item costs the same whatever the number of its pairs, and the call waits
// for the longest one).
constexpr int64_t IVF_QUICK_CHUNK_ROWS = 1 << 20;
constexpr float IVF_PRUNE_RANGE = 3500.f;      // table units between the sum of a pair's minima and the query's first bound
constexpr int IVF_QB_PLAIN = 4;               // queries per work item: plain float loop
constexpr int IVF_QB_PRUNED = 8;              // and the loop on 16-bit lower bounds
constexpr int IVF_QB_QUICK = 8;               // Quick ADC: pairs whose 8-bit tables lie side by side
constexpr int IVF_SHORT_MAX = 12288;          // lists of fewer codes are scanned by the kernel of short lists (8 tables, plain loop)

// ------------------------------------------------------------------------------------------
// nprobe smallest (distance, list id) of one row of coarse distances.  One block per query.
// Fast path for long rows: a threshold guessed from a sample of 1024 entries (its order statistic aimed at
// three times nprobe entries at or below it, by radix selection), one pass that collects the keys at or below
// it (four 16-byte loads of a thread on their way at a time), sort.
// If the guess caught fewer than nprobe or more than fit: histogram of the top 12 bits of the
// ordered value -> bin holding the nprobe-th; everything in lower bins and in that bin is sorted
// in LDS.  If that is too much (heavy ties), bisection on the 64-bit key over the whole row.
constexpr int SEL_CAP = 4096;
__global__ __launch_bounds__(256) void ivf_select_probes_kernel(const float *__restrict__ dist, int nlist,
                                                                int nprobe, int32_t *__restrict__ probes,
                                                                int32_t *probe_out, const int32_t *__restrict__ only_flagged) {
    __shared__ uint64_t cand[SEL_CAP];
    if (only_flagged && only_flagged[blockIdx.x] == 0) return;   // (rows settled otherwise)
    __shared__ uint32_t part[256];
    __shared__ uint32_t sel_state[2];
    __shared__ int s_bin, s_count;
    // the sample of the fast path and the histogram of the slow one live in the memory of the candidates, which
    // are collected only after either has served its purpose
    uint32_t *sample = reinterpret_cast<uint32_t *>(cand);
    uint32_t *hist = reinterpret_cast<uint32_t *>(cand);
    static_assert(SEL_CAP * 8 >= 4096 * 4, "the histogram fits into the candidates' memory");
    __shared__ unsigned long long s_kth;
    const int q = blockIdx.x, tid = threadIdx.x;
    const float *row = dist + (size_t)q * nlist;
    bool done = false;
    if (nlist >= 8192 && (nlist & 3) == 0 && (size_t)nprobe * 3 * 1024 / nlist + 8 < 1024) {
        const int stride = nlist / 1024;
        for (int i = tid; i < 1024; i += 256) sample[i] = f32_to_ord(row[(size_t)i * stride]);
        if (tid == 0) s_count = 0;
        __syncthreads();
        const uint32_t guess = block_kth_smallest_u32(sample, 1024, (uint32_t)((size_t)nprobe * 3 * 1024 / nlist + 8) + 1u, part, sel_state);
        const float4 *row4 = reinterpret_cast<const float4 *>(row);   // rows start on 16-byte boundaries (nlist % 4 == 0)
        auto collect = [&](int i, const float4 v) {
            const uint32_t o[4] = {f32_to_ord(v.x), f32_to_ord(v.y), f32_to_ord(v.z), f32_to_ord(v.w)};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (o[e] <= guess) {
                    const int pos = atomicAdd(&s_count, 1);
                    if (pos < SEL_CAP) cand[pos] = ((uint64_t)o[e] << 32) | (uint32_t)(4 * i + e);
                }
        };
        const int n4 = nlist / 4;
        int i = tid;
        for (; i + 3 * 256 < n4; i += 4 * 256) {
            const float4 v0 = row4[i], v1 = row4[i + 256], v2 = row4[i + 512], v3 = row4[i + 768];
            collect(i, v0); collect(i + 256, v1); collect(i + 512, v2); collect(i + 768, v3);
        }
        for (; i < n4; i += 256) collect(i, row4[i]);
        __syncthreads();
        done = s_count >= nprobe && s_count <= SEL_CAP;
        __syncthreads();
    }
    int total = done ? s_count : 0;
    if (!done) {
        for (int i = tid; i < 4096; i += 256) hist[i] = 0;
        if (tid == 0) { s_bin = 4095; s_count = 0; }
        __syncthreads();
        for (int i = tid; i < nlist; i += 256) atomicAdd(&hist[f32_to_ord(row[i]) >> 20], 1u);
        __syncthreads();
        // thread t owns bins 16t .. 16t+15
        uint32_t mine = 0;
        for (int b = 0; b < 16; ++b) mine += hist[tid * 16 + b];
        part[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0;
            int t = 0;
            for (; t < 256; ++t) { if (cum + part[t] >= (uint32_t)nprobe) break; cum += part[t]; }
            int b = t * 16;
            for (; b < t * 16 + 16 && b < 4096; ++b) { if (cum + hist[b] >= (uint32_t)nprobe) break; cum += hist[b]; }
            s_bin = b < 4096 ? b : 4095;
        }
        __syncthreads();
        const uint32_t bin = (uint32_t)s_bin;
        for (int i = tid; i < nlist; i += 256) {
            const uint32_t o = f32_to_ord(row[i]);
            if ((o >> 20) <= bin) {
                const int pos = atomicAdd(&s_count, 1);
                if (pos < SEL_CAP) cand[pos] = ((uint64_t)o << 32) | (uint32_t)i;
            }
        }
        __syncthreads();
        total = s_count;
        if (total > SEL_CAP) {
            // bisection: smallest key v with count(key <= v) >= nprobe
            uint64_t v = 0;
            for (int bit = 63; bit >= 0; --bit) {
                const uint64_t trial = v | ((1ull << bit) - 1ull);
                __syncthreads();
                if (tid == 0) s_count = 0;
                __syncthreads();
                int c = 0;
                for (int i = tid; i < nlist; i += 256) c += ((((uint64_t)f32_to_ord(row[i]) << 32) | (uint32_t)i) <= trial) ? 1 : 0;
                atomicAdd(&s_count, c);
                __syncthreads();
                if (s_count < nprobe) v |= (1ull << bit);
            }
            __syncthreads();
            if (tid == 0) { s_kth = v; s_count = 0; }
            __syncthreads();
            const uint64_t kth = s_kth;
            for (int i = tid; i < nlist; i += 256) {
                const uint64_t key = ((uint64_t)f32_to_ord(row[i]) << 32) | (uint32_t)i;
                if (key <= kth) { const int pos = atomicAdd(&s_count, 1); if (pos < SEL_CAP) cand[pos] = key; }
            }
            __syncthreads();
            total = s_count;   // exactly nprobe (keys are unique)
        }
    }
    int n2 = 64;
    while (n2 < total) n2 <<= 1;
    for (int i = total + tid; i < n2; i += 256) cand[i] = KEY_EMPTY;
    block_bitonic_sort(cand, n2);
    for (int r = tid; r < nprobe; r += 256) {
        const int32_t l = (int32_t)(uint32_t)cand[r];
        probes[(size_t)q * nprobe + r] = l;
        if (probe_out) probe_out[(size_t)q * nprobe + r] = l;
    }
}

// residual of query q for its r-th probed list: y - centroid (float)
__global__ __launch_bounds__(256) void ivf_residual_kernel(const float *__restrict__ queries,
                                                           const float *__restrict__ coarse,
                                                           const int32_t *__restrict__ probes, int npairs, int nprobe,
                                                           int d, float *__restrict__ resid) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)npairs * d) return;
    const int p = (int)(i / d), t = (int)(i % d);
    const int q = p / nprobe, l = probes[p];
    resid[i] = queries[(size_t)q * d + t] - coarse[(size_t)l * d + t];
}

// the same, four dimensions per thread (d a multiple of 4, all rows on 16-byte boundaries); d4 = d / 4
__global__ __launch_bounds__(256) void ivf_residual4_kernel(const float4 *__restrict__ queries, const float4 *__restrict__ coarse,
                                                            const int32_t *__restrict__ probes, int npairs, int nprobe, int d4,
                                                            float4 *__restrict__ resid) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)npairs * d4) return;
    const int p = (int)(i / (unsigned int)d4), t = (int)(i - (size_t)p * d4);
    const int q = p / nprobe, l = probes[p];
    const float4 y = queries[(size_t)q * d4 + t], c = coarse[(size_t)l * d4 + t];
    resid[i] = make_float4(y.x - c.x, y.y - c.y, y.z - c.z, y.w - c.w);
}

__global__ void ivf_zero_kernel(uint32_t *p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0;
}

__global__ void ivf_count_pairs_kernel(const int32_t *__restrict__ probes, int npairs, uint32_t *np) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < npairs) atomicAdd(&np[probes[p]], 1u);
}

__device__ __forceinline__ int ivf_chunks_of(int64_t size, int64_t uncapped_rows) {
    if (size <= 0) return 0;
    if (uncapped_rows > 0) return (int)((size + uncapped_rows - 1) / uncapped_rows);
    int64_t nc = (size + IVF_CHUNK_TARGET - 1) / IVF_CHUNK_TARGET;
    return (int)(nc < 1 ? 1 : (nc > IVF_MAX_CHUNKS ? IVF_MAX_CHUNKS : nc));
}

// One round of an exclusive scan by a block of 1024 threads: the sum of the values of the threads before this one
// plus *carry, which is then advanced by the block's total (shuffles inside the waves, the 16 wave totals through
// LDS; three barriers).
__device__ __forceinline__ uint32_t block_scan_round(uint32_t v, uint32_t *wave_tot, uint32_t *carry) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = *carry;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    __syncthreads();
    if (tid == 1023) *carry = before + incl;
    __syncthreads();
    return before + incl - v;
}

// Single block.  From the number of pairs per list: where each list's pairs start
// (pair_off), how many chunks it is cut into (nc), where its items start in the item table
// (item_off; lists of a larger size class come first) and the number of items.
// Lists of fewer than short_max codes go to a table of their own (one item per group of short_qs pairs, the whole
// list, for the kernel of short lists); item_off is then the position in that table and nitems_dev[1] its length.
__global__ __launch_bounds__(1024) void ivf_plan_kernel(const uint32_t *__restrict__ np,
                                                        const int64_t *__restrict__ list_offsets, int nlist,
                                                        uint32_t *pair_off, uint32_t *nc_out, uint32_t *item_off,
                                                        uint32_t *nitems_dev, uint32_t qb, int64_t short_max, uint32_t short_qs,
                                                        int64_t uncapped_rows) {
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t cls_items[64], cls_base[64], cls_cursor[64];   // 32 size classes of the long lists, 32 of the short ones
    __shared__ uint32_t carry;
    const int tid = threadIdx.x;
    if (tid < 64) { cls_items[tid] = 0; cls_cursor[tid] = 0; }
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int l0 = 0; l0 < nlist; l0 += 1024) {
        const int l = l0 + tid;
        const uint32_t v = l < nlist ? np[l] : 0u;
        const uint32_t before = block_scan_round(v, wave_tot, &carry);
        if (l < nlist) {
            pair_off[l] = before;
            const int64_t size = list_offsets[l + 1] - list_offsets[l];
            const int nc = v > 0 ? ivf_chunks_of(size, uncapped_rows) : 0;
            nc_out[l] = (uint32_t)nc;
            const bool is_short = size < short_max;
            const uint32_t items = is_short ? (nc > 0 ? (v + short_qs - 1) / short_qs : 0u) : ((v + qb - 1) / qb) * (uint32_t)nc;
            if (items > 0) atomicAdd(&cls_items[(is_short ? 32 : 0) + 63 - __builtin_clzll((unsigned long long)size)], items);
        }
    }
    __syncthreads();
    if (tid == 0) {
        pair_off[nlist] = carry;
        uint32_t run = 0;
        for (int c = 31; c >= 0; --c) { cls_base[c] = run; run += cls_items[c]; }
        nitems_dev[0] = run;
        run = 0;
        for (int c = 63; c >= 32; --c) { cls_base[c] = run; run += cls_items[c]; }
        nitems_dev[1] = run;
    }
    __syncthreads();
    for (int l = tid; l < nlist; l += 1024) {
        const uint32_t v = np[l];
        const int64_t size = list_offsets[l + 1] - list_offsets[l];
        const bool is_short = size < short_max;
        const uint32_t items = is_short ? (nc_out[l] > 0 ? (v + short_qs - 1) / short_qs : 0u) : ((v + qb - 1) / qb) * nc_out[l];
        if (items > 0) {
            const int c = (is_short ? 32 : 0) + 63 - __builtin_clzll((unsigned long long)size);
            item_off[l] = cls_base[c] + atomicAdd(&cls_cursor[c], items);
        } else {
            item_off[l] = 0;
        }
    }
}

__global__ void ivf_fill_pairs_kernel(const int32_t *__restrict__ probes, int npairs,
                                      const uint32_t *__restrict__ pair_off, uint32_t *fill, int32_t *pairs_by_list) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= npairs) return;
    const int l = probes[p];
    pairs_by_list[pair_off[l] + atomicAdd(&fill[l], 1u)] = p;
}

// one thread per list: write the list's items (group-major, chunks of a group consecutive)
__global__ void ivf_fill_items_kernel(const uint32_t *__restrict__ pair_off, const uint32_t *__restrict__ nc_arr,
                                      const uint32_t *__restrict__ item_off, const int64_t *__restrict__ list_offsets,
                                      int nlist, int rows_per_16b, uint32_t qb, IvfItem *items, int64_t short_max,
                                      const int32_t *__restrict__ pairs_by_list, IvfShortItem *short_items) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlist) return;
    const uint32_t npl = pair_off[l + 1] - pair_off[l];
    const int nc = (int)nc_arr[l];
    if (npl == 0 || nc == 0) return;
    const int64_t beg = list_offsets[l], end = list_offsets[l + 1];
    if (end - beg < short_max) {   // a short list: the whole list for every group of IVF_SHORT_QS pairs
        const int64_t aligned = beg / rows_per_16b * rows_per_16b;
        const int ng = (int)((npl + IVF_SHORT_QS - 1) / IVF_SHORT_QS);
        for (int g = 0; g < ng; ++g) {
            const uint32_t nslots = npl - (uint32_t)g * IVF_SHORT_QS < (uint32_t)IVF_SHORT_QS ? npl - (uint32_t)g * IVF_SHORT_QS : (uint32_t)IVF_SHORT_QS;
            IvfShortItem it;
            it.code_begin = (uint32_t)aligned;
            it.ncodes_skip_slots = (uint32_t)(end - aligned) | ((uint32_t)(beg - aligned) << 24) | (nslots << 28);
            for (int s2 = 0; s2 < IVF_SHORT_QS; ++s2)
                it.pair[s2] = (uint32_t)s2 < nslots ? pairs_by_list[pair_off[l] + (uint32_t)g * IVF_SHORT_QS + s2] : 0;
            it.pad[0] = it.pad[1] = 0u;
            short_items[item_off[l] + (uint32_t)g] = it;
        }
        return;
    }
    int64_t rpc = (end - beg + nc - 1) / nc;
    rpc = (rpc + rows_per_16b - 1) / rows_per_16b * rows_per_16b;
    const int ng = (int)((npl + qb - 1) / qb);
    for (int g = 0; g < ng; ++g) {
        const int nslots = (int)(npl - (uint32_t)g * qb < qb ? npl - (uint32_t)g * qb : qb);
        for (int c = 0; c < nc; ++c) {
            int64_t cb = beg + (int64_t)c * rpc, ce = cb + rpc < end ? cb + rpc : end;
            IvfItem it;
            if (cb >= ce) { cb = ce = beg; }   // empty chunk (rounding): scans nothing, still leaves its empty list
            const int64_t aligned = cb / rows_per_16b * rows_per_16b;
            it.code_begin = (uint32_t)aligned;
            it.ncodes = (uint32_t)(ce - aligned);
            it.pair_pos = pair_off[l] + (uint32_t)g * qb;
            it.skip_slots_chunk = (uint32_t)(cb - aligned) | ((uint32_t)nslots << 8) | ((uint32_t)c << 16);
            items[item_off[l] + (uint32_t)g * nc + c] = it;
        }
    }
}

// one thread per query: lists (pair, chunk) the query owns, and each pair's first list relative to the query
__global__ void ivf_pair_lists_kernel(const int32_t *__restrict__ probes, const uint32_t *__restrict__ nc_arr, int nq,
                                      int nprobe, uint32_t *pair_rel, uint32_t *qlists) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    uint32_t run = 0;
    for (int r = 0; r < nprobe; ++r) {
        pair_rel[(size_t)q * nprobe + r] = run;
        run += nc_arr[probes[(size_t)q * nprobe + r]];
    }
    qlists[q] = run;
}

// single block: exclusive scan of qlists -> qlist_off[nq+1] (1024 values per round: shuffles inside the waves, the
// 16 wave totals through LDS)
__global__ __launch_bounds__(1024) void ivf_qlist_scan_kernel(const uint32_t *__restrict__ qlists, int nq, uint32_t *qlist_off) {
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int q0 = 0; q0 < nq; q0 += 1024) {
        const int q = q0 + tid;
        const uint32_t before = block_scan_round(q < nq ? qlists[q] : 0u, wave_tot, &carry);
        if (q < nq) qlist_off[q] = before;
    }
    if (tid == 0) qlist_off[nq] = carry;
}

// absolute first result list of every (query, probe) pair: its place within the query's lists plus the query's first list
__global__ void ivf_pair_abs_kernel(const uint32_t *__restrict__ qlist_off, size_t npairs, int nprobe, uint32_t *pair_out) {
    const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < npairs) pair_out[p] += qlist_off[p / nprobe];
}

// First bound per query: float ADC (the tables' entries added in an order that depends on the lane) of up to IVF_SEED_CODES codes taken from the
// query's probed lists in probe order, each with the tables of its (query, list) pair.  The greatest
// of the first topk distances is a bound already; the distances at or below it are counted in bins of
// 2^HIST_SHIFT ordered-value units below it (0.2 % of the value each), and the smallest bin edge with
// topk distances at or below it is the bound handed on, enlarged by a few units of fp32 rounding
// because the plain scan loop adds the same entries in another order.  +inf if the lists hold fewer
// than topk codes.  (Every candidate a loose first bound lets through costs the scan far more than a
// code its integer test dismisses, so the sample is generous.)
constexpr int IVF_SEED_CODES = 16384;
template <int M>
__global__ __launch_bounds__(256) void ivf_seed_kernel(const uint8_t *__restrict__ codes,
                                                       const int64_t *__restrict__ list_offsets,
                                                       const int32_t *__restrict__ probes, const float *__restrict__ luts,
                                                       int nprobe, int topk, float *tau0) {
    __shared__ __align__(16) float tab[M * 256];
    __shared__ __align__(16) uint32_t hist[HIST_BINS];
    __shared__ uint32_t ref_s;
    const int q = blockIdx.x, tid = threadIdx.x;
    const uint32_t rot = (uint32_t)tid & (M - 1);
    for (int i = tid; i < HIST_BINS; i += 256) hist[i] = 0;
    if (tid == 0) ref_s = 0;
    // f(ordered distance) for the first `limit` codes of the probed lists; returns how many there were
    auto for_codes = [&](int limit, auto &&f) {
        int count = 0;
        for (int r = 0; r < nprobe && count < limit; ++r) {
            const int l = probes[(size_t)q * nprobe + r];
            const int64_t beg = list_offsets[l], size = list_offsets[l + 1] - beg;
            const int take = (int)(size < limit - count ? size : limit - count);
            if (take <= 0) continue;
            const float *lut = luts + ((size_t)q * nprobe + r) * M * 256;
            __syncthreads();
            // entry b of table j at word b * M + j: a lane walks the tables from its own first one (lane % M), so the lanes
            // that the LDS serves together read M different columns of banks
            {
                float e[M];
#pragma unroll
                for (int j = 0; j < M; ++j) e[j] = lut[j * 256 + tid];
#pragma unroll
                for (int j = 0; j < M; j += 4) *reinterpret_cast<float4 *>(tab + tid * M + j) = make_float4(e[j], e[j + 1], e[j + 2], e[j + 3]);
            }
            __syncthreads();
            struct Code { uint32_t w[M / 4]; };
            auto load_code = [&](int i) {
                const uint8_t *c = codes + (size_t)(beg + i) * M;
                Code k;
                if (M == 8) { const uint2 v = *reinterpret_cast<const uint2 *>(c); k.w[0] = v.x; k.w[1] = v.y; }
                else { const uint4 v = *reinterpret_cast<const uint4 *>(c); k.w[0] = v.x; k.w[1] = v.y; k.w[M / 4 - 2] = v.z; k.w[M / 4 - 1] = v.w; }
                return k;
            };
            auto eval = [&](Code k) {
                if constexpr (M == 8) rot8(k.w[0], k.w[1], (rot & 4u) != 0u, rot & 3u);
                else rot16(k.w, rot);
                float dist = 0.f;   // (the entries of the code's M tables, added from table lane % M on)
#pragma unroll
                for (int st = 0; st < M; ++st) dist += tab[(((k.w[st >> 2] >> (8 * (st & 3))) & 255u) * M) | ((rot + st) & (M - 1))];
                f(f32_to_ord(dist));
            };
            // four codes of a thread on their way at a time (the loop is otherwise a chain of load latencies)
            int i = tid;
            for (; i + 3 * 256 < take; i += 4 * 256) {
                const Code c0 = load_code(i), c1 = load_code(i + 256), c2 = load_code(i + 512), c3 = load_code(i + 768);
                eval(c0); eval(c1); eval(c2); eval(c3);
            }
            for (; i < take; i += 256) eval(load_code(i));
            count += take;
        }
        return count;
    };
    const int first = for_codes(topk, [&](uint32_t ord) { atomicMax(&ref_s, ord); });
    __syncthreads();
    if (first < topk) {
        if (tid == 0) tau0[q] = __builtin_inff();
        return;
    }
    const uint32_t ref = ref_s;
    for_codes(IVF_SEED_CODES, [&](uint32_t ord) {
        if (ord <= ref) {
            const uint32_t below = (ref - ord) >> HIST_SHIFT;
            atomicAdd(&hist[HIST_BINS - 1 - (below < (uint32_t)HIST_BINS ? below : HIST_BINS - 1)], 1u);
        }
    });
    __syncthreads();
    if (tid < 64) {   // one wave reads the bin off the counts
        const int b = hist_threshold(hist, topk);
        if (tid == 0) {
            // every distance counted in bins <= b is at or below this edge
            const uint32_t edge = b < HIST_BINS ? ref - ((uint32_t)(HIST_BINS - 1 - b) << HIST_SHIFT) : ref;
            const float kth = ord_to_f32(edge);
            tau0[q] = kth + fabsf(kth) * 4e-6f;
        }
    }
}

// Pruned scan of inverted lists: per (query, list) pair the minima of its M tables, their sum, and the
// scale of the pair's 16-bit lower-bound tables (see scan_flush_pruned): PRUNE_RANGE table units between
// the sum of the minima and the query's first bound tau0.  A pair whose minima already add up to tau0 or
// more cannot contribute a result and gets a negative scale; no first bound gives scale 0 (no pruning);
// the scale is capped so that the bound converts to table units to a fraction of a unit in fp32.
// One wave per pair.
template <int M>
__global__ __launch_bounds__(256) void ivf_prune_prep_kernel(const float *__restrict__ luts, const float *__restrict__ tau0,
                                                             int npairs, int nprobe, float range_units, float *pair_min,
                                                             float *pair_off, float *pair_scale, const int32_t *__restrict__ probes,
                                                             const int64_t *__restrict__ list_offsets, int64_t short_max) {
    const int pair = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (pair >= npairs) return;
    if (short_max > 0) {   // pairs of lists that the kernel of short lists scans need none of this
        const int l = probes[pair];
        if (list_offsets[l + 1] - list_offsets[l] < short_max) return;
    }
    const float4 *t = reinterpret_cast<const float4 *>(luts + (size_t)pair * M * 256);
    float off = 0.f;
    for (int j = 0; j < M; ++j) {
        const float4 v = t[j * 64 + lane];
        float mn = fminf(fminf(v.x, v.y), fminf(v.z, v.w));
        for (int o = 32; o > 0; o >>= 1) mn = fminf(mn, __shfl_xor(mn, o));
        if (lane == 0) pair_min[(size_t)pair * M + j] = mn;
        off += mn;
    }
    if (lane == 0) {
        const float bound = tau0[pair / nprobe];
        float scale = 0.f;
        if (bound < 3.0e38f) {
            const float range = bound - off;
            if (!(range > 0.f)) {
                scale = -1.f;
            } else {
                scale = range_units / range;
                const float cap = 0.99e6f / bound;   // bound * scale * 1e-6 stays below 1
                if (!(scale < cap)) scale = cap;
                if (!(scale > 0.f) || !(scale < 3.0e38f)) scale = 0.f;
            }
        }
        pair_off[pair] = off;
        pair_scale[pair] = scale;
    }
}

// ------------------------------------------------------------------------------------------
// Index step through approximate distances (fp32 matrix cores, every value within eps * (||y||^2 + ||c||^2) of the
// exact one): the ncand > nprobe lists nearest by approximate distance are measured exactly (the plain definition in
// double, rounded to float once), and if the nprobe-th of these exact distances lies below what any list outside the
// candidates can have (the greatest approximate distance among the candidates minus the error bound), the nprobe
// nearest of the candidates are the nprobe nearest of all lists, in (distance, list) order.  Queries for which this
// cannot be shown are flagged; their rows of exact distances are computed and selected from as without the short cut.

// Greatest squared norm of the rows of `v`, as the bits of a float not below it (squared norms are not negative, so
// the bits order like the values).  *out_bits starts at 0.
__global__ __launch_bounds__(256) void ivf_max_norm_kernel(const float *__restrict__ v, int rows, int d, unsigned int *out_bits) {
    __shared__ float red[4];
    const int row = blockIdx.x * 256 + threadIdx.x;
    double n = 0.0;
    if (row < rows)
        for (int t = 0; t < d; ++t) { const double x = v[(size_t)row * d + t]; n += x * x; }
    float f = (float)n * 1.0000002f;
    for (int o = 32; o > 0; o >>= 1) f = fmaxf(f, __shfl_xor(f, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = f;
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(out_bits, __float_as_uint(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]))));
}

// Bound per query for the pass that keeps only near lists, from the query's approximate distances to a sample of the
// lists: one wave per query, lane l takes the smallest of the entries l, l + 64, ..., and the bound is the r-th smallest
// of the 64 lane minima (r <= 64).  That is the value of rank about -64 ln(1 - r / 64) among all the entries (r minima at
// or below it lie in r different lanes), and never below the r-th smallest entry.
__global__ __launch_bounds__(256) void ivf_theta_kernel(const float *__restrict__ sample, int ks, int r, int nq, float *theta) {
    const int q = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (q >= nq) return;
    const float *row = sample + (size_t)q * ks;
    float mine = __builtin_inff();
    for (int i = lane; i < ks; i += 64) mine = fminf(mine, row[i]);
    int before = 0;   // lanes whose minimum comes before this lane's (equal values by lane number)
#pragma unroll
    for (int l = 0; l < 64; ++l) {
        const float other = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine), l));
        before += (other < mine || (other == mine && l < lane)) ? 1 : 0;
    }
    if (before == r - 1) theta[q] = mine;
}

// The keys that the filtering pass kept for a query are gathered from its places (`nslots` of them, ~0: unused) and
// from the entries beyond the places (ov_keys[q][ov_cap], ov_cnt[q] of them), sorted, and written to kept_keys[q][] with
// their number in kept_cnt[q] (0 if there are more than IVF_PICK_CAP or some were lost for lack of room).  The ncand
// smallest are the query's candidates, far[q] the approximate distance of the last of them; queries with fewer than ncand
// keys or more than IVF_PICK_CAP are flagged instead.
constexpr int IVF_PICK_CAP = 2048;
constexpr int IVF_OV_CAP = 256;
__global__ __launch_bounds__(256) void ivf_pick_candidates_kernel(const unsigned long long *__restrict__ slot_keys, int nslots,
                                                                  const unsigned long long *__restrict__ ov_keys,
                                                                  const unsigned int *__restrict__ ov_cnt, int ncand,
                                                                  unsigned long long *__restrict__ kept_keys, unsigned int *__restrict__ kept_cnt,
                                                                  int32_t *__restrict__ cand, float *__restrict__ far, int32_t *__restrict__ flags) {
    __shared__ uint64_t keys[IVF_PICK_CAP];
    __shared__ unsigned int total;
    const int q = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) total = 0u;
    __syncthreads();
    const unsigned int ov = ov_cnt[q];
    const ulonglong2 *places = reinterpret_cast<const ulonglong2 *>(slot_keys + (size_t)q * nslots);   // (nslots is a multiple of 4)
    for (int i = tid; i < nslots / 2; i += 256) {
        const ulonglong2 two = places[i];
        if (two.x != ~0ull) { const unsigned int at = atomicAdd(&total, 1u); if (at < (unsigned int)IVF_PICK_CAP) keys[at] = two.x; }
        if (two.y != ~0ull) { const unsigned int at = atomicAdd(&total, 1u); if (at < (unsigned int)IVF_PICK_CAP) keys[at] = two.y; }
    }
    if (ov <= (unsigned int)IVF_OV_CAP)
        for (int i = tid; i < (int)ov; i += 256) {
            const unsigned int at = atomicAdd(&total, 1u);
            if (at < (unsigned int)IVF_PICK_CAP) keys[at] = ov_keys[(size_t)q * IVF_OV_CAP + i];
        }
    __syncthreads();
    const unsigned int cnt = total;
    const bool whole = ov <= (unsigned int)IVF_OV_CAP && cnt <= (unsigned int)IVF_PICK_CAP;
    if (!whole) {
        if (tid == 0) { kept_cnt[q] = 0u; flags[q] = 1; }
        return;
    }
    int n2 = 128;
    while (n2 < (int)cnt) n2 <<= 1;
    for (int i = (int)cnt + tid; i < n2; i += 256) keys[i] = ~0ull;
    block_bitonic_sort(keys, n2);
    for (int i = tid; i < (int)cnt; i += 256) kept_keys[(size_t)q * IVF_PICK_CAP + i] = keys[i];
    if (tid == 0) kept_cnt[q] = cnt;
    if (cnt < (unsigned int)ncand) {
        if (tid == 0) flags[q] = 1;
        return;
    }
    if (tid < ncand) cand[(size_t)q * ncand + tid] = (int32_t)(uint32_t)keys[tid];
    if (tid == 0) {
        far[q] = ord_to_f32((uint32_t)(keys[ncand - 1] >> 32));
        flags[q] = 0;
    }
}

constexpr int IVF_REFINE_MAX = 128;   // candidates per query (nprobe and a margin)
__global__ __launch_bounds__(IVF_REFINE_MAX) void ivf_refine_probes_kernel(const float *__restrict__ queries, const float *__restrict__ cents,
                                                                          const float *__restrict__ approx, const int32_t *__restrict__ cand,
                                                                          const float *__restrict__ far_in, int ncand, int nlist, int d,
                                                                          int nprobe, float eps, const unsigned int *__restrict__ max_norm_bits,
                                                                          int32_t *__restrict__ probes, int32_t *probe_out,
                                                                          int32_t *__restrict__ flags) {
    extern __shared__ float ys[];   // the query, d floats (d is a multiple of 4)
    __shared__ uint64_t keys[IVF_REFINE_MAX];
    __shared__ double red[2];
    const int q = blockIdx.x, tid = threadIdx.x;
    if (far_in && flags[q] != 0) return;   // (no candidates for this query: it takes the exact row)
    const float *y = queries + (size_t)q * d;
    double ny = 0.0;
    for (int t = tid; t < d; t += IVF_REFINE_MAX) { const float x = y[t]; ys[t] = x; ny += (double)x * (double)x; }
    for (int o = 32; o > 0; o >>= 1) ny += __shfl_xor(ny, o);
    if ((tid & 63) == 0) red[tid >> 6] = ny;
    __syncthreads();
    uint64_t key = ~0ull;
    if (tid < ncand) {
        const int l = cand[(size_t)q * ncand + tid];
        const float4 *c4 = reinterpret_cast<const float4 *>(cents + (size_t)l * d);   // rows start on 16-byte boundaries
        const float4 *y4 = reinterpret_cast<const float4 *>(ys);
        double s = 0.0;   // dimension by dimension, as the definition has it
        for (int t = 0; t < d / 4; t += 4) {   // four loads of 16 bytes on their way at a time
            float4 c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) c[u] = t + u < d / 4 ? c4[t + u] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (t + u >= d / 4) break;
                const float4 yy = y4[t + u];
                double df = (double)yy.x - (double)c[u].x; s += df * df;
                df = (double)yy.y - (double)c[u].y; s += df * df;
                df = (double)yy.z - (double)c[u].z; s += df * df;
                df = (double)yy.w - (double)c[u].w; s += df * df;
            }
        }
        key = ((uint64_t)f32_to_ord((float)s) << 32) | (uint32_t)l;
    }
    keys[tid] = key;
    block_bitonic_sort(keys, IVF_REFINE_MAX);
    __syncthreads();
    if (tid == 0) {
        ny = red[0] + red[1];
        // no list outside the candidates is nearer than this (its approximate distance is at least that of the last candidate)
        const double far = far_in ? (double)far_in[q] : (double)approx[(size_t)q * nlist + cand[(size_t)q * ncand + ncand - 1]];
        const double low = (far - (double)eps * (ny + (double)__uint_as_float(*max_norm_bits))) * (1.0 - 1.2e-7);
        const double kth = (double)ord_to_f32((uint32_t)(keys[nprobe - 1] >> 32));
        flags[q] = kth < low ? 0 : 1;   // (false for a NaN anywhere as well)
    }
    __syncthreads();
    if (flags[q] == 0 && tid < nprobe) {
        const int32_t l = (int32_t)(uint32_t)keys[tid];
        probes[(size_t)q * nprobe + tid] = l;
        if (probe_out) probe_out[(size_t)q * nprobe + tid] = l;
    }
}

// Second attempt for the queries that ivf_refine_probes_kernel left flagged (the gap behind their nprobe-th list is smaller
// than the error bound of the approximations times a handful of lists): exact distances to ALL lists that the filtering pass
// kept for the query.  Their approximate distances are at or below theta[q] and those of every other list above it, so the
// same proof holds against theta[q], some hundreds of lists further out.  Queries with fewer than nprobe kept lists, with more
// than the lists' room, or still without proof (equal distances far out) stay flagged and take the exact row.
__global__ __launch_bounds__(256) void ivf_refine_kept_kernel(const float *__restrict__ queries, const float *__restrict__ cents,
                                                              const unsigned long long *__restrict__ keys_in,
                                                              const unsigned int *__restrict__ cnt_in, const float *__restrict__ theta,
                                                              int d, int nprobe, float eps, const unsigned int *__restrict__ max_norm_bits,
                                                              int32_t *__restrict__ probes, int32_t *probe_out, int32_t *__restrict__ flags) {
    extern __shared__ float ys[];   // the query
    __shared__ uint64_t keys[IVF_PICK_CAP];
    __shared__ double red[4];
    __shared__ int proved;
    const int q = blockIdx.x, tid = threadIdx.x;
    if (flags[q] == 0) return;
    const unsigned int cnt = cnt_in[q];
    if (cnt < (unsigned int)nprobe || cnt > (unsigned int)IVF_PICK_CAP) return;
    const float *y = queries + (size_t)q * d;
    double ny = 0.0;
    for (int t = tid; t < d; t += 256) { const float x = y[t]; ys[t] = x; ny += (double)x * (double)x; }
    for (int o = 32; o > 0; o >>= 1) ny += __shfl_xor(ny, o);
    if ((tid & 63) == 0) red[tid >> 6] = ny;
    __syncthreads();
    int n2 = 128;
    while (n2 < (int)cnt) n2 <<= 1;
    for (int i = tid; i < n2; i += 256) {
        uint64_t key = ~0ull;
        if (i < (int)cnt) {
            const uint32_t l = (uint32_t)keys_in[(size_t)q * IVF_PICK_CAP + i];
            const float *c = cents + (size_t)l * d;
            double s = 0.0;   // dimension by dimension, as the definition has it
            for (int t = 0; t < d; ++t) { const double df = (double)ys[t] - (double)c[t]; s += df * df; }
            key = ((uint64_t)f32_to_ord((float)s) << 32) | l;
        }
        keys[i] = key;
    }
    block_bitonic_sort(keys, n2);
    if (tid == 0) {
        ny = red[0] + red[1] + red[2] + red[3];
        const double low = ((double)theta[q] - (double)eps * (ny + (double)__uint_as_float(*max_norm_bits))) * (1.0 - 1.2e-7);
        const double kth = (double)ord_to_f32((uint32_t)(keys[nprobe - 1] >> 32));
        proved = kth < low ? 1 : 0;   // (false for a NaN anywhere as well)
    }
    __syncthreads();
    if (proved == 0) return;
    if (tid < nprobe) {
        const int32_t l = (int32_t)(uint32_t)keys[tid];
        probes[(size_t)q * nprobe + tid] = l;
        if (probe_out) probe_out[(size_t)q * nprobe + tid] = l;
    }
    if (tid == 0) flags[q] = 0;
}

// Exact distances (the plain definition in double, rounded to float once) of the flagged queries to every list.
__global__ __launch_bounds__(256) void ivf_exact_rows_kernel(const float *__restrict__ queries, const float *__restrict__ cents,
                                                             int nlist, int d, const int32_t *__restrict__ flags,
                                                             float *__restrict__ dist) {
    const int q = blockIdx.x;
    if (flags[q] == 0) return;
    const float *y = queries + (size_t)q * d;
    for (int l = threadIdx.x; l < nlist; l += 256) {
        const float *c = cents + (size_t)l * d;
        double s = 0.0;
        for (int t = 0; t < d; ++t) { const double df = (double)y[t] - (double)c[t]; s += df * df; }
        dist[(size_t)q * nlist + l] = (float)s;
    }
}

// ------------------------------------------------------------------------------------------
int launch_ivf(pq_ctx *ctx, const ivf_lists *L, const float *codebooks, int m, int k, int cf, const float *queries,
               int nq, int nprobe, int topk, float *out_dist, int64_t *out_ids, int32_t *probe_out, int init, int kprime) {
    const int d = L->d, nlist = L->nlist;
    // Packed 4-bit codes: Quick ADC in the Scan step (ivf_quick_kernels.hip), eight pairs per work item, every list
    // cut into work items the same way.
    const bool quick = cf == PQ_CODES_U4_PACKED;
    // Short lists (8 tables, plain loop, blocks of 8 waves): a kernel of their own, see ivf_short_kernels.hip.
    // Option ivf_short_max: lists of fewer codes than this take it (default IVF_SHORT_MAX, 0: none, at most 2^18).
    int64_t short_max = !quick && m == 8 && opt_int(ctx, PQ_OPT_IVF_BLOCK_WAVES, 8) != 16 ? opt_int(ctx, PQ_OPT_IVF_SHORT_MAX, IVF_SHORT_MAX) : 0;
    if (short_max < 0) short_max = 0;
    if (short_max > IVF_CHUNK_TARGET) short_max = IVF_CHUNK_TARGET;
    // The other lists: the loop on 16-bit lower bounds (8 pairs per item, one preparation kernel over the pairs of
    // these lists) where the short lists have their own kernel, so that the preparation touches the tables of few
    // pairs; else the plain float loop (4 pairs per item), which measured the same scan time and a shorter call
    // when every pair needs the preparation.  Option ivf_prune = 0 / 1 fixes the choice.
    const int prune_opt = opt_int(ctx, PQ_OPT_IVF_PRUNE, -1);
    const bool prune = !quick && (prune_opt < 0 ? short_max > 0 : prune_opt != 0);
    const int kind = prune ? (m == 8 ? 3 : 4) : (m == 8 ? 0 : 1);
    const uint32_t item_qb = quick ? IVF_QB_QUICK : prune ? IVF_QB_PRUNED : IVF_QB_PLAIN;   // (query, list) pairs per work item
    const int kpad = 128;
    const int rows_per_16b = 16 / (quick ? m / 2 : m);
    hipStream_t s = ctx->stream;

    // queries per batch: keeps the per-query part of the workspace (coarse distances, residuals and
    // tables of the nprobe pairs, upper bound of their result lists, histogram) within PQ_IVF_WS_GIB
    // GiB (default 24); the more queries share a batch, the more of them share a pass over a list
    // result lists a query can own: one per chunk of each of its lists
    int64_t quick_rows = opt_int(ctx, PQ_OPT_IVF_QUICK_CHUNK_ROWS, (int)IVF_QUICK_CHUNK_ROWS);
    if (quick_rows < 1024) quick_rows = 1024;
    if (quick_rows > (1 << 20)) quick_rows = 1 << 20;
    const size_t lists_per_query = quick ? (size_t)nprobe + (size_t)(L->ntotal / quick_rows) + 1 : (size_t)nprobe * IVF_MAX_CHUNKS;
    const size_t per_query = (size_t)nlist * 4 + (size_t)nprobe * ((size_t)m * k * 4 + (size_t)d * 4 + 64) +
                             lists_per_query * kpad * 8 + (size_t)HIST_BINS * 4 + 64;
    int ws_gib = opt_int(ctx, PQ_OPT_IVF_WS_GIB, 24);
    if (ws_gib < 1) ws_gib = 1;
    if (ws_gib > 128) ws_gib = 128;
    int qbatch = (int)(((size_t)ws_gib << 30) / per_query);
    if (qbatch < 1) qbatch = 1;
    if (qbatch > nq) qbatch = nq;
    const size_t npairs_max = (size_t)qbatch * nprobe;
    const size_t max_lists = (size_t)qbatch * lists_per_query;
    // items of a list: (groups of its pairs) x chunks <= (pairs / item_qb + 1) x chunks
    const size_t max_items = quick ? max_lists / item_qb + (size_t)nlist + (size_t)(L->ntotal / quick_rows) + 1
                                   : (npairs_max / item_qb + (size_t)nlist + 1) * IVF_MAX_CHUNKS;

    // workspace carving (all offsets 256-byte aligned)
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes, 256); return o; };
    const size_t o_dist = take((size_t)qbatch * nlist * 4);
    const size_t o_probes = take(npairs_max * 4);
    const int ncand = nprobe + 16;   // lists measured exactly when the Index step goes through approximate distances
    const size_t o_cand = take((size_t)qbatch * ncand * 4);
    const size_t o_flags = take((size_t)qbatch * 4);
    const size_t o_maxnorm = take(256);
    const size_t o_theta = take((size_t)qbatch * 4);
    const size_t o_far = take((size_t)qbatch * 4);
    const size_t o_ccnt = take((size_t)qbatch * 4);
    const size_t o_ckeys = take((size_t)qbatch * IVF_PICK_CAP * 8);
    const size_t o_kcnt = take((size_t)qbatch * 4);
    const size_t o_ovkeys = take((size_t)qbatch * IVF_OV_CAP * 8);
    const size_t o_slots = take((size_t)qbatch * coarse_filter_slots(nlist) * 8);
    const size_t o_resid = take(npairs_max * d * 4);
    const size_t o_luts = take(npairs_max * m * k * 4);
    const size_t o_np = take((size_t)nlist * 4);
    const size_t o_fill = take((size_t)nlist * 4);
    const size_t o_pairoff = take((size_t)(nlist + 1) * 4);
    const size_t o_nc = take((size_t)nlist * 4);
    const size_t o_itemoff = take((size_t)nlist * 4);
    const size_t o_nitems = take(8);   // (long lists' items, short lists' items)
    const size_t o_pairs = take(npairs_max * 4);
    const size_t o_items = take(max_items * sizeof(IvfItem));
    const size_t max_short_items = short_max > 0 ? npairs_max / IVF_SHORT_QS + (size_t)nlist + 1 : 0;
    const size_t o_sitems = take(max_short_items * sizeof(IvfShortItem));
    const size_t o_pairout = take(npairs_max * 4);
    const size_t o_qlists = take((size_t)qbatch * 4);
    const size_t o_qlistoff = take((size_t)(qbatch + 1) * 4);
    const size_t o_tau0 = take((size_t)qbatch * 4);
    const size_t o_pmin = take(prune ? npairs_max * m * 4 : 0);
    const size_t o_poff = take(prune ? npairs_max * 4 : 0);
    const size_t o_pscale = take(prune ? npairs_max * 4 : 0);
    const size_t o_partial = take(max_lists * kpad * 8);
    // blocks of 8 waves, two per CU, unless PQ_IVF_BLOCK_WAVES=16 asks for the flat scan's shape
    const bool w8_blocks = opt_int(ctx, PQ_OPT_IVF_BLOCK_WAVES, 8) != 16;
    const size_t state_bytes = quick ? 0 : w8_blocks ? w8::tuned_state_bytes(kind, qbatch, topk, ctx->num_cu)
                                                     : w16::tuned_state_bytes(kind, qbatch, topk, ctx->num_cu);
    const size_t o_state = take(state_bytes);
    const size_t o_qmaxp = take(quick ? npairs_max * 4 : 0);
    const size_t o_qluts = take(quick ? npairs_max * (size_t)m * k : 0);
    const size_t o_tauq = take(quick ? (size_t)qbatch * 8 : 0);
    const size_t o_qrows = take(quick ? ivf_quick_saved_bytes(ctx, quick_rows) : 0);
    int rc = ws_reserve(ctx, off);
    if (rc) return rc;
    if (!ctx->aux_stream) {   // second stream of the context and the two events that fork to it and join from it
        PQ_HIP(ctx, hipStreamCreateWithFlags(&ctx->aux_stream, hipStreamNonBlocking));
        PQ_HIP(ctx, hipEventCreateWithFlags(&ctx->aux_fork, hipEventDisableTiming));
        PQ_HIP(ctx, hipEventCreateWithFlags(&ctx->aux_join, hipEventDisableTiming));
    }
    uint8_t *ws = (uint8_t *)ctx->ws;
    float *dist = (float *)(ws + o_dist);
    int32_t *probes = (int32_t *)(ws + o_probes);
    float *resid = (float *)(ws + o_resid);
    float *luts = (float *)(ws + o_luts);
    uint32_t *np = (uint32_t *)(ws + o_np), *fill = (uint32_t *)(ws + o_fill);
    uint32_t *pair_off = (uint32_t *)(ws + o_pairoff), *nc = (uint32_t *)(ws + o_nc);
    uint32_t *item_off = (uint32_t *)(ws + o_itemoff), *nitems_dev = (uint32_t *)(ws + o_nitems);
    int32_t *pairs_by_list = (int32_t *)(ws + o_pairs);
    IvfItem *items = (IvfItem *)(ws + o_items);
    IvfShortItem *short_items = (IvfShortItem *)(ws + o_sitems);
    uint32_t *pair_out = (uint32_t *)(ws + o_pairout), *qlists = (uint32_t *)(ws + o_qlists);
    uint32_t *qlist_off = (uint32_t *)(ws + o_qlistoff);
    uint64_t *partial = (uint64_t *)(ws + o_partial);

    for (int q0 = 0; q0 < nq; q0 += qbatch) {
        const int nqb = nq - q0 < qbatch ? nq - q0 : qbatch;
        const int npairs = nqb * nprobe;
        const float *qb = queries + (size_t)q0 * d;
        // Index step
        int32_t *pout = probe_out ? probe_out + (size_t)q0 * nprobe : nullptr;
        if (opt_int(ctx, PQ_OPT_IVF_COARSE_F32, 1) != 0 && ncand <= IVF_REFINE_MAX && (int64_t)ncand * 8 <= nlist && d <= 8192 &&
            coarse_f32_usable(ctx, qb, L->coarse_centroids, nqb, d, nlist, dist)) {
            int32_t *cand = (int32_t *)(ws + o_cand), *flags = (int32_t *)(ws + o_flags);
            unsigned int *maxnorm = (unsigned int *)(ws + o_maxnorm);
            ivf_zero_kernel<<<1, 64, 0, s>>>(maxnorm, (size_t)1);
            ivf_max_norm_kernel<<<(nlist + 255) / 256, 256, 0, s>>>(L->coarse_centroids, nlist, d, maxnorm);
            PQ_HIP(ctx, hipGetLastError());
            // With many lists the matrix of approximate distances is not written at all: a sample of the lists (every
            // 16th) gives each query a bound below which some hundreds of lists are expected, and the pass over all
            // lists keeps the entries at or below it (a query left with fewer than ncand of them takes the exact row).
            const int ks = (nlist + 15) / 16, rank = 6 * ncand / 16 > 8 ? 6 * ncand / 16 : 8;
            const int lane_rank = (int)(64.0 * (1.0 - exp(-(double)rank / 64.0)) + 0.5);   // (of the 64 lane minima that ivf_theta_kernel ranks)
            if (nlist >= 16384 && rank <= ncand && coarse_f32_usable(ctx, qb, L->coarse_centroids, nqb, d, ks, dist)) {
                float *theta = (float *)(ws + o_theta), *far = (float *)(ws + o_far);
                unsigned int *ccnt = (unsigned int *)(ws + o_ccnt);
                unsigned long long *ckeys = (unsigned long long *)(ws + o_ckeys), *ovkeys = (unsigned long long *)(ws + o_ovkeys);
                unsigned long long *slots = (unsigned long long *)(ws + o_slots);
                unsigned int *kcnt = (unsigned int *)(ws + o_kcnt);
                ivf_zero_kernel<<<64, 256, 0, s>>>(ccnt, (size_t)nqb);
                rc = launch_coarse_f32(ctx, qb, L->coarse_centroids, (size_t)16 * d, nqb, d, ks, dist);
                if (rc) return rc;
                ivf_theta_kernel<<<(nqb + 3) / 4, 256, 0, s>>>(dist, ks, lane_rank, nqb, theta);
                PQ_HIP(ctx, hipGetLastError());
                // (the pass over all lists on the fp16 matrix cores, every operand as two halves; option 0: on the fp32 ones)
                const bool split16 = opt_int(ctx, PQ_OPT_IVF_COARSE_F16, 1) != 0;
                rc = split16 ? launch_coarse_split16_filter(ctx, qb, L->coarse_centroids, nqb, d, nlist, theta, slots, ovkeys, ccnt, IVF_OV_CAP)
                             : launch_coarse_f32_filter(ctx, qb, L->coarse_centroids, nqb, d, nlist, theta, slots, ovkeys, ccnt, IVF_OV_CAP);
                if (rc) return rc;
                ivf_pick_candidates_kernel<<<nqb, 256, 0, s>>>(slots, coarse_filter_slots(nlist), ovkeys, ccnt, ncand, ckeys, kcnt, cand, far, flags);
                ivf_refine_probes_kernel<<<nqb, IVF_REFINE_MAX, (size_t)d * 4, s>>>(qb, L->coarse_centroids, nullptr, cand, far, ncand, nlist, d,
                                                                                   nprobe, split16 ? coarse_split16_error(d) : coarse_f32_error(d),
                                                                                   maxnorm, probes, pout, flags);
                ivf_refine_kept_kernel<<<nqb, 256, (size_t)d * 4, s>>>(qb, L->coarse_centroids, ckeys, kcnt, theta, d, nprobe,
                                                                      split16 ? coarse_split16_error(d) : coarse_f32_error(d), maxnorm,
                                                                      probes, pout, flags);
            } else {
                rc = launch_coarse_f32(ctx, qb, L->coarse_centroids, (size_t)d, nqb, d, nlist, dist);
                if (rc) return rc;
                ivf_select_probes_kernel<<<nqb, 256, 0, s>>>(dist, nlist, ncand, cand, nullptr, nullptr);
                ivf_refine_probes_kernel<<<nqb, IVF_REFINE_MAX, (size_t)d * 4, s>>>(qb, L->coarse_centroids, dist, cand, nullptr, ncand, nlist, d,
                                                                                   nprobe, coarse_f32_error(d), maxnorm, probes, pout, flags);
            }
            // (queries that the short cut could not settle: normally none)
            ivf_exact_rows_kernel<<<nqb, 256, 0, s>>>(qb, L->coarse_centroids, nlist, d, flags, dist);
            ivf_select_probes_kernel<<<nqb, 256, 0, s>>>(dist, nlist, nprobe, probes, pout, flags);
            PQ_HIP(ctx, hipGetLastError());
        } else {
            rc = launch_build_luts(ctx, qb, L->coarse_centroids, nqb, d, 1, nlist, dist);
            if (rc) return rc;
            ivf_select_probes_kernel<<<nqb, 256, 0, s>>>(dist, nlist, nprobe, probes, pout, nullptr);
            PQ_HIP(ctx, hipGetLastError());
        }
        // The grouping of the pairs needs the probed lists only: it runs on a stream of the context's own (same priority)
        // beside the residuals and their tables, and joins the caller's stream before the first bounds.
        hipStream_t g = ctx->aux_stream;
        PQ_HIP(ctx, hipEventRecord(ctx->aux_fork, s));
        PQ_HIP(ctx, hipStreamWaitEvent(g, ctx->aux_fork, 0));
        ivf_zero_kernel<<<256, 256, 0, g>>>(np, (size_t)nlist);
        ivf_zero_kernel<<<256, 256, 0, g>>>(fill, (size_t)nlist);
        ivf_count_pairs_kernel<<<(npairs + 255) / 256, 256, 0, g>>>(probes, npairs, np);
        ivf_plan_kernel<<<1, 1024, 0, g>>>(np, L->list_offsets, nlist, pair_off, nc, item_off, nitems_dev, item_qb, short_max, (uint32_t)IVF_SHORT_QS,
                                           quick ? quick_rows : (int64_t)0);
        ivf_fill_pairs_kernel<<<(npairs + 255) / 256, 256, 0, g>>>(probes, npairs, pair_off, fill, pairs_by_list);
        ivf_fill_items_kernel<<<(nlist + 255) / 256, 256, 0, g>>>(pair_off, nc, item_off, L->list_offsets, nlist,
                                                                  rows_per_16b, item_qb, items, short_max, pairs_by_list, short_items);
        ivf_pair_lists_kernel<<<(nqb + 255) / 256, 256, 0, g>>>(probes, nc, nqb, nprobe, pair_out, qlists);
        ivf_qlist_scan_kernel<<<1, 1024, 0, g>>>(qlists, nqb, qlist_off);
        ivf_pair_abs_kernel<<<(unsigned)(((size_t)nqb * nprobe + 255) / 256), 256, 0, g>>>(qlist_off, (size_t)nqb * nprobe, nprobe, pair_out);
        PQ_HIP(ctx, hipGetLastError());
        PQ_HIP(ctx, hipEventRecord(ctx->aux_join, g));
        // Tables step on the residuals
        {
            const size_t n = (size_t)npairs * d;
            const bool by4 = (d & 3) == 0 && (((uintptr_t)qb | (uintptr_t)L->coarse_centroids | (uintptr_t)resid) & 15) == 0;
            if (by4)
                ivf_residual4_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, s>>>((const float4 *)qb, (const float4 *)L->coarse_centroids, probes,
                                                                                     npairs, nprobe, d / 4, (float4 *)resid);
            else
                ivf_residual_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(qb, L->coarse_centroids, probes, npairs, nprobe, d, resid);
            PQ_HIP(ctx, hipGetLastError());
        }
        rc = launch_build_luts(ctx, resid, codebooks, npairs, d, m, k, luts);
        if (rc) return rc;
        PQ_HIP(ctx, hipStreamWaitEvent(s, ctx->aux_join, 0));   // the work items are laid out
        if (quick) {
            unsigned long long *tau_q = (unsigned long long *)(ws + o_tauq);
            rc = launch_ivf_quick(ctx, L->codes, L->list_offsets, probes, luts, nqb, nprobe, init, kprime, topk,
                                  (float *)(ws + o_qmaxp), ws + o_qluts, items, nitems_dev, pairs_by_list, pair_out, nc,
                                  partial, tau_q, (uint32_t *)(ws + o_qrows), quick_rows);
            if (rc) return rc;
            rc = launch_merge_filtered(ctx, partial, qlist_off, 0, 0, 1, tau_q, kpad, nqb, topk, L->ids, false,
                                       out_dist + (size_t)q0 * topk, out_ids + (size_t)q0 * topk);
            if (rc) return rc;
            continue;
        }
        // Scan step, seeded with a first bound per query
        float *tau0 = (float *)(ws + o_tau0);
        if (m == 8) ivf_seed_kernel<8><<<nqb, 256, 0, s>>>(L->codes, L->list_offsets, probes, luts, nprobe, topk, tau0);
        else ivf_seed_kernel<16><<<nqb, 256, 0, s>>>(L->codes, L->list_offsets, probes, luts, nprobe, topk, tau0);
        PQ_HIP(ctx, hipGetLastError());
        float *pmin = nullptr, *poff = nullptr, *pscale = nullptr;
        if (prune) {
            pmin = (float *)(ws + o_pmin); poff = (float *)(ws + o_poff); pscale = (float *)(ws + o_pscale);
            if (m == 8) ivf_prune_prep_kernel<8><<<(npairs + 3) / 4, 256, 0, s>>>(luts, tau0, npairs, nprobe, IVF_PRUNE_RANGE, pmin, poff, pscale, probes, L->list_offsets, short_max);
            else ivf_prune_prep_kernel<16><<<(npairs + 3) / 4, 256, 0, s>>>(luts, tau0, npairs, nprobe, IVF_PRUNE_RANGE, pmin, poff, pscale, probes, L->list_offsets, short_max);
            PQ_HIP(ctx, hipGetLastError());
        }
        unsigned long long *tau_key = nullptr;
        rc = w8_blocks ? w8::launch_scan_items(ctx, kind, pmin, poff, pscale, L->codes, luts, nqb, nprobe, topk, items, nitems_dev,
                                               pairs_by_list, pair_out, partial, ws + o_state, state_bytes, tau0, &tau_key)
                       : w16::launch_scan_items(ctx, kind, pmin, poff, pscale, L->codes, luts, nqb, nprobe, topk, items, nitems_dev,
                                                pairs_by_list, pair_out, partial, ws + o_state, state_bytes, tau0, &tau_key);
        if (rc) return rc;
        // the short lists after the long ones: by then a query's bound has seen the lists that hold most of its codes
        if (short_max > 0) {
            rc = launch_ivf_short_scan(ctx, L->codes, luts, short_items, nitems_dev + 1, pair_out, nprobe, topk, tau_key, partial);
            if (rc) return rc;
            if (ctx->profiling) {   // the measured "scan kernel" is both kernels
                PQ_HIP(ctx, hipEventRecord(ctx->ev_end, s));
                const size_t len = strlen(ctx->last_scan_name);
                snprintf(ctx->last_scan_name + len, sizeof(ctx->last_scan_name) - len, " (lists of %lld codes and more) + ivf_short_scan_kernel (shorter lists, 4 pairs per pass, blocks of 4 waves)", (long long)short_max);
            }
        }
        rc = launch_merge_filtered(ctx, partial, qlist_off, 0, 0, 1, tau_key, kpad, nqb, topk, L->ids, false,
                                   out_dist + (size_t)q0 * topk, out_ids + (size_t)q0 * topk);
        if (rc) return rc;
    }
    return PQ_OK;
}

}  // namespace pq
