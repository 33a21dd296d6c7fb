// IVFADC search with Quick ADC in the Scan step (chapter 5: packed 4-bit codes, m = 16 sub-quantizers of 16
// centroids, tables quantised to 8 bits, Section 5.2; Section 5.3 evaluates it inside the inverted index of
// Section 2.3.2).  Per query:
//   qmax     float ADC of the first `init` codes met when the probed lists are walked in probe order (each code with
//            the float tables of its own (query, list) pair); qmax = the topk-th smallest of these distances, the
//            distance to a temporary topk-th neighbour (Section 5.2.1, as Section 4.2.4);
//   8 bits   every pair's tables quantised between the pair's own smallest entry and the query's qmax
//            (launch_quantize_luts);
//   Scan     integer sums of the 8-bit entries (Alg. 3, plain sums) over the codes of the list; the kprime smallest
//            (sum, row) of a pair are its candidates;
//   Rerank   float ADC of the candidates with the pair's float tables; the topk smallest (distance, row) of the query.
// Sums of different pairs are not comparable (own qmin and scale each), so the candidates are chosen per pair.
//
// Where the thesis keeps the 16 tables of 16 bytes in SIMD registers and looks 16 codes up at once, the scan kernel
// here keeps the tables of EIGHT (query, list) pairs that probe the same list side by side in LDS: the entry for
// (sub-quantizer j, index i) is one 16-byte slot of eight 16-bit values, so one LDS read serves eight pairs and the
// eight sums are formed by four packed 16-bit additions per sub-quantizer.  The 16 slots of a sub-quantizer cover
// all 64 LDS banks once: lanes with different indexes never collide and lanes with equal indexes read one address.
//
// The kprime smallest sums of a work item (a chunk of a list x up to 8 pairs) are found by counting instead of
// sorting, because sums are small integers (at most 16 * 255): a first pass over the codes counts the sums of each
// pair in 512 bins, which gives the kprime-th smallest sum T of the pair exactly; a second pass collects the codes
// below T (fewer than kprime) and, in row order, those equal to T.  Every float sum of this file is formed in
// double in table order and rounded once, so that the bound, the 8-bit tables, the candidates and the distances are
// those of the plain definition bit for bit.
#include <type_traits>
#include "pq_internal.h"
#include "scan_common.h"
#include "topk_device.h"

namespace pq {

constexpr int QK_QS = 8;          // (query, list) pairs per work item
constexpr int QK_LONG_MIN = 65536;   // work items of this many rows and more take the blocks of 8 waves
constexpr int QK_BINS = 512;      // sums counted per pass: base .. base + 510, and one bin for everything above
constexpr int QK_KP = 128;        // kprime at most (the length of a result list)
constexpr int QK_BATCH = 4;       // codes of a thread on their way at a time

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pk_add_u16(uint32_t a, uint32_t b) {
    const u16x2 r = __builtin_bit_cast(u16x2, a) + __builtin_bit_cast(u16x2, b);
    return __builtin_bit_cast(uint32_t, r);
}
// per 16-bit half: a - b, 0 where b > a
__device__ __forceinline__ uint32_t pk_sub_sat_u16(uint32_t a, uint32_t b) {
    const u16x2 r = __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    return __builtin_bit_cast(uint32_t, r);
}

// index j (0 .. 15) of a packed code: component 2i in the low half of byte i
__device__ __forceinline__ uint32_t code_index4(const uint2 c, int j) { return ((j < 8 ? c.x : c.y) >> (4 * (j & 7))) & 15u; }

// float ADC in double, table order, rounded once (tab: [16][16] floats)
__device__ __forceinline__ float adc16x4_exact(const float *tab, const uint2 c) {
    double s = 0.0;
#pragma unroll
    for (int j = 0; j < 16; ++j) s += (double)tab[j * 16 + code_index4(c, j)];
    return (float)s;
}

// ------------------------------------------------------------------------------------------
// qmax of every query, written once per (query, list) pair, and the query's bound for the final merge set to "none".
// One block per query.
constexpr int QK_INIT_MAX = 4096;
__global__ __launch_bounds__(256) void ivf_quick_qmax_kernel(const uint8_t *__restrict__ codes,
                                                             const int64_t *__restrict__ list_offsets,
                                                             const int32_t *__restrict__ probes, const float *__restrict__ luts,
                                                             int nprobe, int init, int topk, float *qmax_pair,
                                                             unsigned long long *tau_key) {
    __shared__ float tab[256];
    __shared__ uint32_t vals[QK_INIT_MAX];
    __shared__ uint32_t bins[256], state[2];
    const int q = blockIdx.x, tid = threadIdx.x;
    int count = 0;
    for (int r = 0; r < nprobe && count < init; ++r) {
        const int l = probes[(size_t)q * nprobe + r];
        const int64_t beg = list_offsets[l], size = list_offsets[l + 1] - beg;
        const int take = (int)(size < init - count ? size : init - count);
        if (take <= 0) continue;
        __syncthreads();
        tab[tid] = luts[((size_t)q * nprobe + r) * 256 + tid];
        __syncthreads();
        for (int i = tid; i < take; i += 256) {
            const uint2 c = *reinterpret_cast<const uint2 *>(codes + (size_t)(beg + i) * 8);
            vals[count + i] = f32_to_ord(adc16x4_exact(tab, c));
        }
        count += take;
    }
    __syncthreads();
    float qmax = __builtin_inff();
    if (count > 0) qmax = ord_to_f32(block_kth_smallest_u32(vals, count, (uint32_t)(topk < count ? topk : count), bins, state));
    for (int r = tid; r < nprobe; r += 256) qmax_pair[(size_t)q * nprobe + r] = qmax;
    if (tid == 0) tau_key[q] = KEY_EMPTY;
}

// ------------------------------------------------------------------------------------------
template <int QK_WAVES, typename TieRow>
struct __align__(16) QuickSmem {
    uint4 tab[256];                              // slot j * 16 + i: the 8-bit entries (j, i) of the 8 pairs as 16-bit values
    uint32_t hist[QK_QS][QK_BINS];
    unsigned long long sure[QK_QS][QK_KP];       // keys below the pair's T (fewer than kprime)
    TieRow tie[QK_WAVES][QK_QS][QK_KP];          // rows (within the item) with sum T, per wave in ascending order
    int sure_cnt[QK_QS];
    int tie_cnt[QK_WAVES][QK_QS];
    uint32_t tstar[QK_QS];                       // T: the kprime-th smallest sum (0xffff: every code is a candidate)
    uint32_t below[QK_QS];                       // sums below `base` (counted in earlier attempts)
    uint32_t base[QK_QS];                        // first sum of bin 0 in the current counting pass
    int found[QK_QS];
    uint32_t cap[QK_QS];                         // sums above it are not counted (the kprime-th smallest sum so far)
    uint32_t cum_t[QK_QS];                       // sums from `base` on below the cap (all counted sums while none is reached)
    int reached[QK_QS];
    int pair[QK_QS];
    uint32_t out_idx[QK_QS];
    int pending;                                 // pairs whose T is not known yet
};
// (items of the blocks of 4 waves have fewer than QK_LONG_MIN = 2^16 rows: 16 bits hold a row within the item)
typedef QuickSmem<4, uint16_t> QuickSmemShort;
typedef QuickSmem<8, uint32_t> QuickSmemLong;
static_assert(QK_LONG_MIN <= 65536, "rows of short items fit 16 bits");
static_assert(sizeof(QuickSmemShort) <= 40 * 1024, "four blocks of 4 waves share the 160 KB of a compute unit");
static_assert(sizeof(QuickSmemLong) <= 80 * 1024, "two blocks of 8 waves per compute unit");

// Blocks of QK_WAVES waves.  LONG: the kernel takes the work items of QK_LONG_MIN rows and more (8 waves, two blocks
// per compute unit: the longest item of a skewed index is what the call waits for), else the shorter ones (4 waves,
// four blocks per compute unit).  Items are dealt in a stride of the grid; an item of the other kind is passed over.
template <int QK_WAVES, bool LONG>
__global__ __launch_bounds__(QK_WAVES * 64, LONG ? 2 : 4) void ivf_quick_scan_kernel(const uint8_t *__restrict__ codes,
                                                                       const uint8_t *__restrict__ qluts,
                                                                       const IvfItem *__restrict__ items,
                                                                       const uint32_t *__restrict__ nitems_dev,
                                                                       const int32_t *__restrict__ pairs_by_list,
                                                                       const uint32_t *__restrict__ pair_out, int kprime,
                                                                       uint64_t *partial, uint32_t *saved_rows, int saved_cap) {
    constexpr int QK_THREADS = QK_WAVES * 64;
    extern __shared__ __align__(16) unsigned char quick_smem[];
    typedef typename std::conditional<LONG, uint32_t, uint16_t>::type TieRow;
    QuickSmem<QK_WAVES, TieRow> &sm = *reinterpret_cast<QuickSmem<QK_WAVES, TieRow> *>(quick_smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nitems = (int)*nitems_dev;
    // rows of the item that the counting pass found at or below some pair's cap of the moment, per wave in the order
    // the wave met them (ascending): the only rows the collecting pass has to look at again
    uint32_t *my_saved = saved_rows + ((size_t)blockIdx.x * QK_WAVES + wave) * (size_t)saved_cap;
    for (int item = (int)blockIdx.x; item < nitems; item += (int)gridDim.x) {
        const IvfItem it = items[item];
        if (((int)it.ncodes >= QK_LONG_MIN) != LONG) continue;   // (uniform)
        const int skip = (int)(it.skip_slots_chunk & 255u);
        const int nslots = (int)((it.skip_slots_chunk >> 8) & 255u);
        const uint32_t chunk = it.skip_slots_chunk >> 16;
        const int ncodes = (int)it.ncodes;            // rows from code_begin; the first `skip` belong to the list before
        const int nvalid = ncodes - skip;
        const uint32_t row0 = it.code_begin;
        const uint8_t *base_ptr = codes + (size_t)row0 * 8;
        __syncthreads();   // the item before is done with the shared state
        if (tid < QK_QS) {
            const int pair = tid < nslots ? pairs_by_list[it.pair_pos + tid] : -1;
            sm.pair[tid] = pair;
            sm.out_idx[tid] = pair >= 0 ? pair_out[pair] + chunk : 0u;
            sm.sure_cnt[tid] = 0;
            sm.below[tid] = 0u;
            sm.base[tid] = 0u;
            sm.tstar[tid] = 0xffffu;
            sm.found[tid] = (tid >= nslots || nvalid <= kprime) ? 1 : 0;
        }
        __syncthreads();
        // ---- the 8-bit tables of the item's pairs, widened to 16 bits, pair s in half s of the slot
        if (tid < 256) {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int s = 0; s < QK_QS; ++s) {
                const int pair = sm.pair[s];
                const uint32_t e = pair >= 0 ? (uint32_t)qluts[(size_t)pair * 256 + tid] : 0u;
                w[s >> 1] |= e << (16 * (s & 1));
            }
            sm.tab[tid] = make_uint4(w[0], w[1], w[2], w[3]);
        }
        __syncthreads();

        // sums of one code for the eight pairs: four registers of two 16-bit sums
        uint32_t tab_lds = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)sm.tab;   // LDS address of the tables
        asm volatile("" : "+v"(tab_lds));
        // Returns, per lane, whether some pair's sum is below its limit (`limit` holds the limits per 16-bit half; 0:
        // nothing passes).
        auto sums_below = [&](const uint2 c, bool valid, const uint32_t (&limit)[4], uint32_t (&acc)[4]) {
            acc[0] = acc[1] = acc[2] = acc[3] = 0u;
            // byte b of lo4 / hi4: index 2 b / 2 b + 1 of the code times 16, the offset of its slot within a sub-quantizer's 256 bytes
            uint32_t lo4[2] = {(c.x << 4) & 0xf0f0f0f0u, (c.y << 4) & 0xf0f0f0f0u};
            uint32_t hi4[2] = {c.x & 0xf0f0f0f0u, c.y & 0xf0f0f0f0u};
            // (kept as they are: the compiler would otherwise go back to a shift, a mask and an addition per entry)
            asm volatile("" : "+v"(lo4[0]), "+v"(lo4[1]), "+v"(hi4[0]), "+v"(hi4[1]));
            auto entry = [&](int j) {
                const uint32_t word = (j & 1) ? hi4[j >> 3] : lo4[j >> 3];
                const uint32_t addr = tab_lds | ((word >> (8 * ((j >> 1) & 3))) & 0xffu);   // (the tables start on a 256-byte boundary)
                return *(const __attribute__((address_space(3))) u32x4 *)(uintptr_t)(addr + (uint32_t)j * 256u);
            };
            // two 16-bit sums per register, added as 32-bit words (no half ever carries: a sum is at most 16 * 255), two
            // entries per three-operand addition
#pragma unroll
            for (int j = 0; j < 16; j += 2) {
                const u32x4 e0 = entry(j), e1 = entry(j + 1);
                acc[0] = acc[0] + e0.x + e1.x; acc[1] = acc[1] + e0.y + e1.y;
                acc[2] = acc[2] + e0.z + e1.z; acc[3] = acc[3] + e0.w + e1.w;
            }
            const uint32_t any = pk_sub_sat_u16(limit[0], acc[0]) | pk_sub_sat_u16(limit[1], acc[1]) |
                                 pk_sub_sat_u16(limit[2], acc[2]) | pk_sub_sat_u16(limit[3], acc[3]);
            return valid && any != 0u;
        };
        // f(row index within the item, code) for every code of the item; a thread meets its rows in ascending order,
        // and so does a wave (lane by lane within a step, step by step)
        auto for_codes = [&](int begin, int end, auto &&f) {
            for (int i0 = begin + tid; i0 < end; i0 += QK_BATCH * QK_THREADS) {
                uint2 c[QK_BATCH];
#pragma unroll
                for (int u = 0; u < QK_BATCH; ++u) {
                    const int i = i0 + u * QK_THREADS;
                    c[u] = i < end ? *reinterpret_cast<const uint2 *>(base_ptr + (size_t)i * 8) : make_uint2(0u, 0u);
                }
#pragma unroll
                for (int u = 0; u < QK_BATCH; ++u) {
                    const int i = i0 + u * QK_THREADS;
                    f(i, c[u], i < end);
                }
            }
        };

        // ---- counting passes: T of every pair.  Sums of base .. base + 510 are counted (one pass unless fewer than
        // kprime sums lie in that range: then the next 511 values are counted in another pass).  The codes are taken
        // in segments of 1024, 2048, 4096, ... rows (twice that in blocks of 8 waves); after each segment the kprime-th smallest sum so far becomes the
        // pair's cap, and greater sums are no longer counted: the final T cannot exceed it.
        int scnt = 0;            // rows saved by this wave (uniform among the lanes still in the loop; lane 0 stays longest)
        bool use_saved = nvalid > kprime;
        if (nvalid > kprime) {
            for (int attempt = 0;; ++attempt) {
                if (attempt > 0) use_saved = false;   // (rows of a second counting pass would be saved twice: all rows are looked at again)
                for (int i = tid; i < QK_QS * QK_BINS; i += QK_THREADS) (&sm.hist[0][0])[i] = 0u;
                if (tid < QK_QS) {
                    sm.cap[tid] = sm.base[tid] + (uint32_t)(QK_BINS - 2);
                    sm.reached[tid] = 0;
                    sm.cum_t[tid] = 0u;
                }
                if (tid == 0) sm.pending = 0;
                __syncthreads();
                uint32_t lo[QK_QS];
                bool open[QK_QS];
#pragma unroll
                for (int s = 0; s < QK_QS; ++s) { lo[s] = sm.base[s]; open[s] = sm.found[s] == 0; }
                for (int seg_begin = skip, seg_len = QK_BATCH * QK_THREADS; seg_begin < ncodes; seg_len *= 2) {
                    const int seg_end = ncodes - seg_begin < seg_len ? ncodes : seg_begin + seg_len;
                    uint32_t capv[QK_QS], capplus[4] = {0u, 0u, 0u, 0u};   // cap + 1 per pair (0: pair not counted)
#pragma unroll
                    for (int s = 0; s < QK_QS; ++s) {
                        capv[s] = sm.cap[s];
                        if (open[s]) capplus[s >> 1] |= (capv[s] + 1u) << (16 * (s & 1));
                    }
                    for_codes(seg_begin, seg_end, [&](int i, const uint2 c, bool valid) {
                        uint32_t acc[4];
                        const bool pass = sums_below(c, valid, capplus, acc);
                        const uint64_t mask = __ballot(pass);
                        if (mask == 0ull) return;
                        {
                            const int pos = scnt + mask_prefix(mask);
                            if (pass && pos < saved_cap) my_saved[pos] = (uint32_t)i;
                            scnt += __popcll(mask);
                        }
                        if (!pass) return;
#pragma unroll
                        for (int s = 0; s < QK_QS; ++s) {
                            const uint32_t sum = (acc[s >> 1] >> (16 * (s & 1))) & 0xffffu;
                            if (open[s] && sum >= lo[s] && sum <= capv[s]) atomicAdd(&sm.hist[s][sum - lo[s]], 1u);
                        }
                    });
                    __syncthreads();
                    // a wave reads the bins of a pair: lane l owns bins 8 l .. 8 l + 7 (the last bin stays empty)
                    for (int s = wave; s < QK_QS; s += QK_WAVES) {
                        if (sm.found[s]) continue;   // (uniform)
                        uint32_t b8[8], tot = 0u;
#pragma unroll
                        for (int t = 0; t < 8; ++t) { b8[t] = sm.hist[s][lane * 8 + t]; tot += b8[t]; }
                        uint32_t incl = tot;
#pragma unroll
                        for (int o = 1; o < 64; o <<= 1) {
                            const uint32_t up = __shfl_up(incl, o);
                            if (lane >= o) incl += up;
                        }
                        const uint32_t want = (uint32_t)kprime - sm.below[s];
                        const uint64_t reach = __ballot(incl >= want);
                        if (reach != 0ull) {
                            if (lane == __builtin_ctzll(reach)) {
                                uint32_t cum = incl - tot;
                                int t = 0;
                                while (cum + b8[t] < want) { cum += b8[t]; ++t; }   // (ends within the lane's bins)
                                sm.cap[s] = sm.base[s] + (uint32_t)(lane * 8 + t);   // the kprime-th smallest sum so far
                                sm.cum_t[s] = cum;                                    // sums below it, from base on
                                sm.reached[s] = 1;
                            }
                        } else if (lane == 63) {
                            sm.cum_t[s] = incl;   // all sums counted so far
                        }
                    }
                    __syncthreads();
                    seg_begin = seg_end;
                }
                if (tid < QK_QS && sm.found[tid] == 0) {
                    sm.below[tid] += sm.cum_t[tid];
                    if (sm.reached[tid]) {
                        sm.tstar[tid] = sm.cap[tid];
                        sm.found[tid] = 1;
                    } else {   // fewer than kprime sums up to base + 510: count the next 511 values
                        sm.base[tid] += (uint32_t)(QK_BINS - 1);
                        atomicAdd(&sm.pending, 1);
                    }
                }
                __syncthreads();
                if (sm.pending == 0) break;
                __syncthreads();   // (pending is cleared by thread 0 at the top of the next pass)
            }
        }

        // ---- collecting pass: keys below T, and the rows at T in ascending order per wave
        {
            uint32_t tplus[4] = {0u, 0u, 0u, 0u};   // T + 1 per pair (0 for empty slots: nothing passes)
            uint32_t tval[QK_QS];
            int need[QK_QS], tcnt[QK_QS];
#pragma unroll
            for (int s = 0; s < QK_QS; ++s) {
                tval[s] = sm.tstar[s];
                const uint32_t tp = s < nslots ? (tval[s] < 0xffffu ? tval[s] + 1u : 0xffffu) : 0u;
                tplus[s >> 1] |= tp << (16 * (s & 1));
                // rows at T that can still be candidates: kprime less the sums below T (none when every code is taken)
                need[s] = (s < nslots && tval[s] < 0xffffu) ? kprime - (int)sm.below[s] : 0;
                tcnt[s] = 0;
            }
            scnt = __builtin_amdgcn_readfirstlane(scnt);
            if (scnt > saved_cap) use_saved = false;   // (cannot happen: a wave saves at most the rows it meets)
            use_saved = __syncthreads_or(use_saved ? 0 : 1) == 0;   // (the same decision in every wave)
            // f(row, code, valid) for the rows to look at: the wave's saved rows in their order, or every row of the item
            auto for_rows = [&](auto &&f) {
                if (!use_saved) { for_codes(skip, ncodes, f); return; }
                for (int e0 = lane; e0 < scnt; e0 += QK_BATCH * 64) {
                    uint32_t r[QK_BATCH];
                    uint2 c[QK_BATCH];
#pragma unroll
                    for (int u = 0; u < QK_BATCH; ++u) r[u] = e0 + u * 64 < scnt ? my_saved[e0 + u * 64] : 0u;
#pragma unroll
                    for (int u = 0; u < QK_BATCH; ++u)
                        c[u] = e0 + u * 64 < scnt ? *reinterpret_cast<const uint2 *>(base_ptr + (size_t)r[u] * 8) : make_uint2(0u, 0u);
#pragma unroll
                    for (int u = 0; u < QK_BATCH; ++u) f((int)r[u], c[u], e0 + u * 64 < scnt);
                }
            };
            for_rows([&](int i, const uint2 c, bool valid) {
                uint32_t acc[4];
                const bool some = sums_below(c, valid, tplus, acc);
                if (__ballot(some) == 0ull) return;
#pragma unroll
                for (int s = 0; s < QK_QS; ++s) {
                    const uint32_t sum = (acc[s >> 1] >> (16 * (s & 1))) & 0xffffu;
                    const bool in = valid && s < nslots;
                    if (in && sum < tval[s]) {
                        const int at = atomicAdd(&sm.sure_cnt[s], 1);   // (fewer than kprime such codes exist)
                        sm.sure[s][at] = ((unsigned long long)sum << 32) | (row0 + (uint32_t)i);
                    }
                    const bool at_t = in && sum == tval[s] && tval[s] < 0xffffu;
                    const uint64_t mask = __ballot(at_t);
                    if (mask != 0ull) {
                        const int pos = tcnt[s] + mask_prefix(mask);
                        if (at_t && pos < need[s]) sm.tie[wave][s][pos] = (TieRow)i;
                        tcnt[s] += __popcll(mask);
                        if (tcnt[s] > need[s]) tcnt[s] = need[s];   // (later rows of this wave are greater: not needed)
                    }
                }
            });
            if (lane == 0) {
#pragma unroll
                for (int s = 0; s < QK_QS; ++s) sm.tie_cnt[wave][s] = tcnt[s];
            }
        }
        __syncthreads();

        // ---- result lists: the keys below T, then the smallest rows at T up to kprime keys, then empty slots; put
        // together in LDS (the list of keys below T has room for kprime keys), then written out
        for (int e = tid; e < QK_QS * QK_KP; e += QK_THREADS) {
            const int s = e / QK_KP, idx = e % QK_KP;
            if (idx >= sm.sure_cnt[s]) sm.sure[s][idx] = KEY_EMPTY;
        }
        __syncthreads();
        for (int s = 0; s < nslots; ++s) {
            const int c = sm.sure_cnt[s];
            const uint32_t t = sm.tstar[s];
            const int need = t < 0xffffu ? kprime - c : 0;
            if (need <= 0) continue;
            // entry e of wave w's list: its rank among the rows at T of all waves (rows are distinct)
            for (int e = tid; e < QK_WAVES * QK_KP; e += QK_THREADS) {
                const int w = e / QK_KP, idx = e % QK_KP;
                if (idx >= sm.tie_cnt[w][s]) continue;
                const uint32_t row = (uint32_t)sm.tie[w][s][idx];
                int rank = idx;
#pragma unroll
                for (int w2 = 0; w2 < QK_WAVES; ++w2) {
                    if (w2 == w) continue;
                    int lo = 0, hi = sm.tie_cnt[w2][s];   // rows of w2 below `row`
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if ((uint32_t)sm.tie[w2][s][mid] < row) lo = mid + 1; else hi = mid;
                    }
                    rank += lo;
                }
                if (rank < need) sm.sure[s][c + rank] = ((unsigned long long)t << 32) | (row0 + row);
            }
        }
        __syncthreads();
        for (int e = tid; e < nslots * QK_KP; e += QK_THREADS) {
            const int s = e / QK_KP, idx = e % QK_KP;
            partial[(size_t)sm.out_idx[s] * QK_KP + idx] = sm.sure[s][idx];
        }
    }
}

// ------------------------------------------------------------------------------------------
// Rerank: one block per (query, list) pair.  The kprime smallest integer keys over the pair's result lists (one list
// per chunk of the inverted list, any number of them) are its candidates; their float distances replace them in the pair's first list,
// in ascending order, the other lists are emptied, and the pair's topk-th key (if it has one) bounds the query's result.
__global__ __launch_bounds__(128) void ivf_quick_rerank_kernel(const uint8_t *__restrict__ codes, const float *__restrict__ luts,
                                                               const int32_t *__restrict__ probes, const uint32_t *__restrict__ nc_arr,
                                                               const uint32_t *__restrict__ pair_out, int nprobe, int kprime,
                                                               int topk, uint64_t *partial, unsigned long long *tau_key) {
    __shared__ float tab[256];
    __shared__ uint64_t keys[2 * QK_KP];
    const int pair = blockIdx.x, tid = threadIdx.x;
    const int nc = (int)nc_arr[probes[pair]];
    uint64_t *lists = partial + (size_t)pair_out[pair] * QK_KP;
    tab[tid] = luts[(size_t)pair * 256 + tid];
    tab[tid + 128] = luts[(size_t)pair * 256 + 128 + tid];
    uint64_t key;
    if (nc <= 1) {
        key = nc == 1 ? lists[tid] : KEY_EMPTY;
    } else {   // a list of several chunks: the smallest keys so far in keys[0 .. 127], the next chunk's list sorted in beside them
        keys[tid] = lists[tid];
        for (int c = 1; c < nc; ++c) {
            keys[QK_KP + tid] = lists[(size_t)c * QK_KP + tid];
            block_bitonic_sort(keys, 2 * QK_KP);
        }
        key = tid < kprime ? keys[tid] : KEY_EMPTY;
        __syncthreads();
    }
    __syncthreads();
    uint64_t fkey = KEY_EMPTY;
    if (key != KEY_EMPTY) {
        const uint32_t row = (uint32_t)key;
        const uint2 c = *reinterpret_cast<const uint2 *>(codes + (size_t)row * 8);
        fkey = ((uint64_t)f32_to_ord(adc16x4_exact(tab, c)) << 32) | row;
    }
    keys[tid] = fkey;
    block_bitonic_sort(keys, 128);
    if (nc >= 1) lists[tid] = keys[tid];
    for (size_t i = 128 + tid; i < (size_t)nc * QK_KP; i += 128) lists[i] = KEY_EMPTY;
    if (tid == 0 && keys[topk - 1] != KEY_EMPTY) atomicMin(&tau_key[pair / nprobe], (unsigned long long)keys[topk - 1]);
}

// ------------------------------------------------------------------------------------------
// Rows a wave can meet in a work item of at most `rows` rows (+ the rows of alignment in front) scanned by `waves` waves.
static int ivf_quick_saved_cap(int64_t rows, int waves) { return (int)(((rows + 16) / (waves * 64) + 2) * 64); }

size_t ivf_quick_saved_bytes(const pq_ctx *ctx, int64_t max_item_rows) {
    return ((size_t)ctx->num_cu * 2 * 8 * ivf_quick_saved_cap(max_item_rows, 8) + (size_t)ctx->num_cu * 4 * 4 * ivf_quick_saved_cap(QK_LONG_MIN, 4)) * 4;
}

int launch_ivf_quick(pq_ctx *ctx, const uint8_t *codes, const int64_t *list_offsets, const int32_t *probes,
                     const float *luts, int nq, int nprobe, int init, int kprime, int topk, float *qmax_pair,
                     uint8_t *qluts, const IvfItem *items, const uint32_t *nitems_dev, const int32_t *pairs_by_list,
                     const uint32_t *pair_out, const uint32_t *nc_arr, uint64_t *partial, unsigned long long *tau_key,
                     uint32_t *saved_rows, int64_t max_item_rows) {
    if (kprime < 1 || kprime > QK_KP || topk < 1 || topk > QK_KP || init < 1 || init > QK_INIT_MAX)
        return fail(ctx, PQ_EUNSUPPORTED, "ivf quick adc: kprime and topk must be 1..%d, init 1..%d", QK_KP, QK_INIT_MAX);
    hipStream_t s = ctx->stream;
    const int npairs = nq * nprobe;
    ivf_quick_qmax_kernel<<<nq, 256, 0, s>>>(codes, list_offsets, probes, luts, nprobe, init, topk, qmax_pair, tau_key);
    PQ_HIP(ctx, hipGetLastError());
    int rc = launch_quantize_luts(ctx, luts, npairs, 16, 16, qmax_pair, qluts, nullptr, nullptr);
    if (rc) return rc;
    if (ctx->profiling) {
        PQ_HIP(ctx, hipEventRecord(ctx->ev_begin, s));
        snprintf(ctx->last_scan_name, sizeof(ctx->last_scan_name),
                 "ivf_quick_scan_kernel (16x4 codes, 8-bit tables of 8 (query, list) pairs per work item; blocks of 8 waves for items of %d rows and more, of 4 waves for the others)", QK_LONG_MIN);
        ctx->last_scan_qpp = QK_QS;
        ctx->last_scan_passes = 2;
        ctx->stat_parked = nullptr;
        ctx->stat_ncand = nullptr;
        ctx->stat_ncand_len = 0;
    }
    {
        auto long_kernel = ivf_quick_scan_kernel<8, true>;
        auto short_kernel = ivf_quick_scan_kernel<4, false>;
        PQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(long_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)sizeof(QuickSmemLong)));
        PQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(short_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)sizeof(QuickSmemShort)));
        // the long items first (longest lists come first in the table of items), then the many short ones
        const int cap_long = ivf_quick_saved_cap(max_item_rows, 8), cap_short = ivf_quick_saved_cap(QK_LONG_MIN, 4);
        long_kernel<<<ctx->num_cu * 2, 8 * 64, sizeof(QuickSmemLong), s>>>(codes, qluts, items, nitems_dev, pairs_by_list, pair_out,
                                                                       kprime, partial, saved_rows, cap_long);
        PQ_HIP(ctx, hipGetLastError());
        short_kernel<<<ctx->num_cu * 4, 4 * 64, sizeof(QuickSmemShort), s>>>(codes, qluts, items, nitems_dev, pairs_by_list, pair_out,
                                                                          kprime, partial,
                                                                          saved_rows + (size_t)ctx->num_cu * 2 * 8 * cap_long, cap_short);
        PQ_HIP(ctx, hipGetLastError());
    }
    if (ctx->profiling) {
        PQ_HIP(ctx, hipEventRecord(ctx->ev_end, s));
        ctx->ev_valid = 1;
    }
    ivf_quick_rerank_kernel<<<npairs, 128, 0, s>>>(codes, luts, probes, nc_arr, pair_out, nprobe, kprime, topk, partial, tau_key);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

}  // namespace pq
