// Search with derived quantizers (chapter 6; Section 6.2.3, Alg. 5) for 64-bit codes of four
// 16-bit indexes whose low 8 bits name the centroid of the derived 8-bit quantizer (property P1
// of Section 6.2.2).
//
//   Step 1.1  compact tables from the derived codebooks      -> the Tables kernel (lut_kernels.hip)
//   Step 1.2  qmax = greatest compact distance of the first r2 codes (derived_qmax_kernel),
//             8-bit tables                                   -> the quantiser (lut_kernels.hip)
//   Step 1.3  adc_low_bits over the whole database into buckets indexed by the integer distance
//   Step 2    precise distances from the full codebooks for the vectors of the buckets taken in
//             increasing order until r2 vectors are in (the bucket of the r2-th is finished)
//
// Capped buckets on a GPU.  The thesis appends every vector to the list of its bucket and keeps
// an upper bound on the bucket index so that the lists stay short.  Here the lists are replaced
// by counts: a first pass over the codes counts, per query, the vectors of every bucket up to a
// bound that is lowered in the same way (the smallest bucket below which r2 counted vectors lie
// bounds the bucket of the r2-th from above, so every vector at or below the final bucket is
// always counted); the bucket b* of the r2-th vector and the exact number of vectors in the
// buckets 0..b* follow from the counts.  A second pass over the codes, with b* fixed, writes the
// ids of exactly those vectors into a list whose size is known beforehand.  Both passes run the
// same loop: 8 queries per pass over a chunk of codes, tables in LDS as 16-bit entries (8 queries
// per 16-byte slot, the four tables stored four times in the rotated slot order of lds_walk.h,
// so every read is conflict-free), four lookups and three packed adds per code, one packed
// compare for 8 queries x 2 codes.

#include "pq_internal.h"
#include "scan_common.h"
#include "topk_device.h"
#include "lds_walk.h"

namespace pq {
namespace {

constexpr int DQ_WAVES = 16;
constexpr int DQ_THREADS = DQ_WAVES * 64;
constexpr int DQ_QB = 8;            // queries per pass
constexpr int DQ_M = 4;             // sub-quantizers (16-bit indexes per code)
constexpr int DQ_BINS = 1024;       // buckets: integer distances are at most 4 * 255
constexpr int DQ_SUB = 128;         // codes per wave sub-tile (16 bytes = two codes per lane)
constexpr uint32_t DQ_THR_MAX = 0x7fffu;   // "every sum passes" (sums stay below 1024)
constexpr int DQ_DEPTH = 4;         // sub-tiles per group of a wave
constexpr int DQ_RING = 64 * (DQ_DEPTH + 1);   // parked rows per wave: a group's worth behind an unflushed rest

struct DqArgs {
    const uint8_t *codes;        // [n][8]
    int64_t n, chunk_codes;
    int nchunks, ngroups, nitems, nq, r2;
    const uint8_t *qluts;        // [nq][4][256]
    uint32_t *work_counter;
    uint32_t *g_hist;            // [nq][DQ_BINS] vectors counted per bucket
    uint32_t *g_bound;           // [nq] bucket bound shared by the blocks (counting pass)
    const uint32_t *bucket;      // [nq] b* (collecting pass)
    const uint64_t *cand_off;    // [nq + 1]
    uint32_t *cand_cnt;          // [nq]
    uint64_t *cand;              // keys (integer distance << 32 | row)
};

struct __align__(16) DqSmem {
    uint4 lut[4096];                   // row b: 16 slots; slot s = table s >> 2 (four copies)
    uint32_t hist[DQ_QB][DQ_BINS];     // this block's counts of the current item
    uint32_t thr[DQ_QB];               // a vector is kept for query q if its sum is below thr[q]
    uint32_t ring[DQ_WAVES][DQ_RING];  // rows whose sums passed a threshold, waiting to be counted or listed
    int item;
};

// first bin at which the running count reaches k, and that count; DQ_BINS if it never does.
// `load(i)` returns the count of bin i.  One wave.
template <class Load>
__device__ __forceinline__ int first_bin_reaching(Load load, uint32_t k, uint32_t *count_out) {
    const int lane = lane_id();
    uint32_t carry = 0;
    for (int j = 0; j < DQ_BINS / 64; ++j) {
        uint32_t v = load(j * 64 + lane);
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(v, o);
            if (lane >= o) v += up;
        }
        v += carry;
        const uint64_t reached = __ballot(v >= k);
        if (reached != 0ull) {
            const int first = __builtin_ctzll(reached);
            if (count_out) *count_out = __shfl(v, first);
            return j * 64 + first;
        }
        carry = __shfl(v, 63);
    }
    if (count_out) *count_out = carry;
    return DQ_BINS;
}

// MODE 0: counting pass (buckets), MODE 1: collecting pass (ids of the buckets 0..b*)
template <int MODE>
__global__ __launch_bounds__(DQ_THREADS) void derived_scan_kernel(DqArgs a) {
    __shared__ DqSmem sm;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = lane_id();
    const uint32_t lane15 = (uint32_t)lane & 15u;
    // Lane l reads slot ((l & 15) + 4 s) & 15 at step s, which holds table ((l >> 2) + s) & 3;
    // rotating the code right by 2 * ((l >> 2) & 3) bytes brings that table's index byte to
    // byte 2 s.  bases[g]: slot offsets of steps 2g (byte 0) and 2g + 1 (byte 2).
    const uint32_t rot = 2u * ((lane15 >> 2) & 3u);
    uint32_t bases[2];
#pragma unroll
    for (int g = 0; g < 2; ++g)
        bases[g] = (((lane15 + 4u * (2 * g)) & 15u) << 4) | ((((lane15 + 4u * (2 * g + 1)) & 15u) << 4) << 16);
    const char *lut_bytes = reinterpret_cast<const char *>(sm.lut);

    for (;;) {
        if (threadIdx.x == 0) sm.item = (int)atomicAdd(a.work_counter, 1u);
        __syncthreads();
        const int item = sm.item;
        if (item >= a.nitems) break;
        const int group = item % a.ngroups, chunk = item / a.ngroups;
        const int64_t cbeg = (int64_t)chunk * a.chunk_codes;
        const int64_t cend = cbeg + a.chunk_codes < a.n ? cbeg + a.chunk_codes : a.n;
        const int ncodes = cend > cbeg ? (int)(cend - cbeg) : 0;

        if (threadIdx.x < DQ_QB) {
            const int gq = group * DQ_QB + threadIdx.x;
            uint32_t thr = 0;   // empty slot: nothing passes
            if (gq < a.nq) {
                const uint32_t b = MODE == 0 ? __hip_atomic_load(&a.g_bound[gq], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                             : a.bucket[gq];
                thr = b + 1u < DQ_THR_MAX ? b + 1u : DQ_THR_MAX;
            }
            sm.thr[threadIdx.x] = thr;
        }
        if (MODE == 0)
            for (int i = threadIdx.x; i < DQ_QB * DQ_BINS; i += DQ_THREADS) (&sm.hist[0][0])[i] = 0u;
        {   // tables of the group's queries: entry (byte b, table t) of all 8 queries in one slot
            const int b = threadIdx.x >> 2, t = threadIdx.x & 3;
            uint32_t v[DQ_QB];
#pragma unroll
            for (int q = 0; q < DQ_QB; ++q) {
                const int gq = group * DQ_QB + q;
                v[q] = gq < a.nq ? (uint32_t)a.qluts[((size_t)gq * DQ_M + t) * 256 + b] : 0u;
            }
            const uint4 pk = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
#pragma unroll
            for (int c = 0; c < 4; ++c) sm.lut[b * 16 + t * 4 + c] = pk;
        }
        __syncthreads();

        const uint8_t *chunk_ptr = a.codes + cbeg * 8;
        const int nfull = ncodes / DQ_SUB;                       // sub-tiles with every code present
        const int nsub = (ncodes + DQ_SUB - 1) / DQ_SUB;         // the last one may be ragged
        uint32_t tau[4];   // thresholds of the 8 queries, two per register
        auto reload_tau = [&]() {
            const uint32_t t = sm.thr[lane & (DQ_QB - 1)];
#pragma unroll
            for (int p = 0; p < 4; ++p)
                tau[p] = __builtin_amdgcn_readlane(t, 2 * p) | (__builtin_amdgcn_readlane(t, 2 * p + 1) << 16);
        };
        typedef uint32_t v4u __attribute__((ext_vector_type(4)));
        typedef const __attribute__((address_space(1))) v4u *global_v4u;
        auto load_full = [&](int t) -> uint4 {
            const v4u v = *(global_v4u)(chunk_ptr + (size_t)t * (DQ_SUB * 8) + lane * 16);
            return make_uint4(v.x, v.y, v.z, v.w);
        };
        // the two codes at rows pos, pos + 1 of the chunk (zeros for rows past its end)
        auto load_pair = [&](int pos) -> uint4 {
            uint4 c = make_uint4(0, 0, 0, 0);
            const uint8_t *p = chunk_ptr + (size_t)pos * 8;
            if (pos + 2 <= ncodes) {
                c = *reinterpret_cast<const uint4 *>(p);
            } else if (pos < ncodes) {
                const uint2 half = *reinterpret_cast<const uint2 *>(p);
                c.x = half.x; c.y = half.y;
            }
            return c;
        };

        // the eight table reads of the lane's two codes (four tables each, in the lane's rotated order)
        auto issue = [&](const uint4 c, uint4 (&v)[8]) {
            uint32_t w[4] = {c.x, c.y, c.z, c.w};
            rot8(w[0], w[1], (rot & 4u) != 0, rot & 3u);
            rot8(w[2], w[3], (rot & 4u) != 0, rot & 3u);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint32_t word = w[2 * h + (s >> 1)];
                    const uint32_t off = (s & 1) ? lut_offset<2>(word, bases[s >> 1]) : lut_offset<0>(word, bases[s >> 1]);
                    v[4 * h + s] = *reinterpret_cast<const uint4 *>(lut_bytes + off);
                }
            }
        };
        // integer distances of the two codes for the 8 queries, as four packed pairs per code
        auto add_up = [&](const uint4 (&v)[8], uint32_t (&d)[2][4]) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                d[h][0] = v[4 * h].x + v[4 * h + 1].x + v[4 * h + 2].x + v[4 * h + 3].x;
                d[h][1] = v[4 * h].y + v[4 * h + 1].y + v[4 * h + 2].y + v[4 * h + 3].y;
                d[h][2] = v[4 * h].z + v[4 * h + 1].z + v[4 * h + 2].z + v[4 * h + 3].z;
                d[h][3] = v[4 * h].w + v[4 * h + 1].w + v[4 * h + 2].w + v[4 * h + 3].w;
            }
        };

        // One sub-tile whose reads are on their way: sums, one packed test for 8 queries x 2 codes,
        // and the rows of the lanes with a sum below a threshold parked in the wave's ring.
        int ring_cnt = 0;
        auto finish = [&](const uint4 (&v)[8], const int sidx) {
            uint32_t d[2][4];
            add_up(v, d);
            // 16-bit fields below 0x8000: the smaller of the two sums minus the threshold wraps
            // (sets bit 15) iff one of them is below the threshold
            typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
            uint32_t below = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const u16x2 mn = __builtin_elementwise_min(__builtin_bit_cast(u16x2, d[0][p]), __builtin_bit_cast(u16x2, d[1][p]));
                below |= __builtin_bit_cast(uint32_t, (u16x2)(mn - __builtin_bit_cast(u16x2, tau[p])));
            }
            const uint64_t hit = __ballot((below & 0x80008000u) != 0u);
            if (__builtin_expect(hit != 0ull, 0)) {
                if ((hit >> lane) & 1ull) sm.ring[wave][ring_cnt + mask_prefix(hit)] = (uint32_t)(sidx * DQ_SUB + lane * 2);
                ring_cnt += __popcll(hit);
            }
        };
        auto scan_sub = [&](const uint4 c, const int sidx) {
            uint4 v[8];
            issue(c, v);
            asm volatile("" : : : "memory");   // all eight reads are issued before the first add
            finish(v, sidx);
        };

        // Parked rows, 64 at a time: the sums again, the test against the thresholds of now, and
        // for every (code, query) that passes the bucket count or the list append.
        auto flush = [&](const int count) {
            reload_tau();
            for (int base = 0; base < count; base += 64) {
                const bool have = base + lane < count;
                const int pos = have ? (int)sm.ring[wave][base + lane] : ncodes;
                uint32_t d[2][4];
                {
                    uint4 v[8];
                    issue(load_pair(pos), v);
                    add_up(v, d);
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const bool valid = pos + h < ncodes;
#pragma unroll
                    for (int q = 0; q < DQ_QB; ++q) {
                        const uint32_t sum = (d[h][q >> 1] >> (16 * (q & 1))) & 0xffffu;
                        const uint32_t thr = (tau[q >> 1] >> (16 * (q & 1))) & 0xffffu;
                        const bool pass = valid && sum < thr;
                        if (MODE == 0) {
                            if (pass) atomicAdd(&sm.hist[q][sum], 1u);
                        } else {
                            const uint64_t mask = __ballot(pass);
                            if (mask != 0ull) {
                                const int gq = group * DQ_QB + q;
                                const int first = __builtin_ctzll(mask);
                                uint32_t slot = 0;
                                if (lane == first) slot = atomicAdd(&a.cand_cnt[gq], (uint32_t)__popcll(mask));
                                slot = __shfl(slot, first);
                                // (the list holds exactly the vectors the first pass counted; the
                                // comparison only keeps a disagreement from writing past it)
                                const uint64_t at = a.cand_off[gq] + slot + (uint32_t)mask_prefix(mask);
                                if (pass && at < a.cand_off[gq + 1]) a.cand[at] = ((uint64_t)sum << 32) | (uint32_t)(cbeg + pos + h);
                            }
                        }
                    }
                }
            }
        };

        // Counting pass: the bound of a query is lowered from the block's own counts while the item
        // runs (waves 0..7, one query each), early and then every 16 groups.
        auto refresh = [&]() {
            const int q = wave;
            if (group * DQ_QB + q >= a.nq) return;
            const int b = first_bin_reaching([&](int i) { return sm.hist[q][i]; }, (uint32_t)a.r2, nullptr);
            if (b < DQ_BINS && lane == 0) atomicMin(&sm.thr[q], (uint32_t)b + 1u);
        };

        // A wave works through groups of DQ_DEPTH full sub-tiles (group g = sub-tiles g * DEPTH ...);
        // the codes of its next group are requested into the registers of the sub-tile just scanned;
        // full batches of parked rows are flushed between groups.
        const int ngroups_t = nfull / DQ_DEPTH;
        int it = 0;
        uint4 cur[DQ_DEPTH];
#pragma unroll
        for (int u = 0; u < DQ_DEPTH; ++u) cur[u] = make_uint4(0, 0, 0, 0);
        // this lane's 16 bytes of sub-tile 0 of the wave's current group, then of its next group
        const uint8_t *gp = chunk_ptr + (size_t)wave * (DQ_DEPTH * DQ_SUB * 8) + lane * 16;
        auto load_group_sub = [&](const uint8_t *p, int u) -> uint4 {
            const v4u v = *(global_v4u)(p + u * (DQ_SUB * 8));
            return make_uint4(v.x, v.y, v.z, v.w);
        };
        if (wave < ngroups_t) {
#pragma unroll
            for (int u = 0; u < DQ_DEPTH; ++u) cur[u] = load_group_sub(gp, u);
        }
        reload_tau();
        for (int g = wave; g < ngroups_t; g += DQ_WAVES) {
            const bool more = g + DQ_WAVES < ngroups_t;
            gp += (size_t)DQ_WAVES * (DQ_DEPTH * DQ_SUB * 8);
            // the table reads of sub-tile u + 1 are issued before the sums of sub-tile u are formed
            uint4 va[8], vb[8];
            issue(cur[0], va);
            if (more) cur[0] = load_group_sub(gp, 0);
#pragma unroll
            for (int u = 0; u < DQ_DEPTH; ++u) {
                if (u + 1 < DQ_DEPTH) {
                    issue(cur[u + 1], (u & 1) ? va : vb);
                    if (more) cur[u + 1] = load_group_sub(gp, u + 1);
                }
                asm volatile("" : : : "memory");
                finish((u & 1) ? vb : va, g * DQ_DEPTH + u);
            }
            if (__builtin_expect(ring_cnt >= 64, 0)) {
                const int whole = ring_cnt & ~63;
                flush(whole);
                for (int i = lane; i < ring_cnt - whole; i += 64) {   // the rest moves to the front
                    const uint32_t v = sm.ring[wave][whole + i];
                    sm.ring[wave][i] = v;
                }
                ring_cnt -= whole;
            }
            if (MODE == 0) {
                if (wave < DQ_QB && ((it & (it + 1)) == 0 || (it & 15) == 15)) refresh();
                reload_tau();
            }
            ++it;
        }
        // sub-tiles past the last whole group, the ragged one included
        for (int sidx = ngroups_t * DQ_DEPTH + wave; sidx < nsub; sidx += DQ_WAVES)
            scan_sub(load_pair(sidx * DQ_SUB + lane * 2), sidx);
        if (ring_cnt > 0) flush(ring_cnt);

        if (MODE == 0) {
            // the block's counts join the query's device-wide buckets, whose bound then serves
            // every block that starts an item of this query later
            __syncthreads();
            for (int i = threadIdx.x; i < DQ_QB * DQ_BINS; i += DQ_THREADS) {
                const int q = i / DQ_BINS, bin = i % DQ_BINS;
                const uint32_t v = sm.hist[q][bin];
                const int gq = group * DQ_QB + q;
                if (v != 0u && gq < a.nq) atomicAdd(&a.g_hist[(size_t)gq * DQ_BINS + bin], v);
            }
            __syncthreads();
            if (wave < DQ_QB && group * DQ_QB + wave < a.nq) {
                const int gq = group * DQ_QB + wave;
                const uint32_t *gh = a.g_hist + (size_t)gq * DQ_BINS;
                const int b = first_bin_reaching(
                    [&](int i) { return __hip_atomic_load(&gh[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); },
                    (uint32_t)a.r2, nullptr);
                if (b < DQ_BINS && lane == 0) atomicMin(&a.g_bound[gq], (uint32_t)b);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// The same loop for many queries (640 and more; used by the collecting pass): 16 queries per pass over the codes.  The entries of the
// 8-bit tables are bytes, so the entries of 16 queries for one (table, byte) fill a 16-byte LDS slot exactly;
// their sums of four do not fit a byte, so the scan loop adds 5-bit lower bounds instead,
//   L[t][b] = min(31, floor((Q[t][b] - min_b Q[t][b]) * scale)),   scale = DQ16_RANGE / (thr - off),
// (off = the sum of the four minima, thr = the query's threshold: sums below it are wanted), four of which stay
// below 128: the 16 sums of a code add up byte-wise in four 32-bit adds per table, and one add per word tests them
// against 0x80 - threshold (bit 7 of a byte stays clear iff that sum is below its threshold).  A code with
// sum <= thr - 1 has a bound of at most floor((thr - 1 - off) * scale) + 1 (fp32 rounding of the products), so
// testing "bound < that + 2" loses none.  Lanes that pass park their rows; the parked rows get their exact sums
// from the exact tables, which wait in LDS as well (16 KB), and are counted or listed as in the 8-query kernel.
// In the counting pass the thresholds fall quickly at the start of an item; the bounds are rebuilt from the
// exact tables at the thresholds of the moment after 4, 16 and 64 groups of a wave.
constexpr int DQ16_QB = 16;
constexpr int DQ16_DEPTH = 2;
constexpr int DQ16_RING = 64 * (DQ16_DEPTH + 1);
constexpr float DQ16_RANGE = 48.f;
constexpr float DQ16_ENTRY_MAX = 31.f;

template <int MODE>
struct __align__(16) DqSmem16 {
    uint4 lut[4096];                   // lower bounds: row b, 16 slots; slot s = table s >> 2 (four copies); 16 queries per slot
    uint4 lutx[DQ_M][256];             // exact entries: table t, byte b, 16 queries
    uint32_t hist[MODE == 0 ? DQ16_QB : 1][DQ_BINS];   // this block's counts of the current item (counting pass)
    uint32_t thr[DQ16_QB];             // a vector is kept for query q if its sum is below thr[q] (0: empty slot)
    uint32_t tmin[DQ16_QB][DQ_M];      // minima of the exact tables
    float off[DQ16_QB], scale[DQ16_QB];
    uint32_t ring[DQ_WAVES][DQ16_RING];
    int item;
};

template <int MODE>
__global__ __launch_bounds__(DQ_THREADS) void derived_scan16_kernel(DqArgs a) {
    typedef DqSmem16<MODE> SM;
    __shared__ SM sm;
    static_assert(sizeof(SM) <= 160 * 1024, "LDS of a CU");
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = lane_id();
    const uint32_t lane15 = (uint32_t)lane & 15u;
    // the walk over the slots of a row is that of the 8-query kernel (same layout of the rows)
    const uint32_t rot = 2u * ((lane15 >> 2) & 3u);
    uint32_t bases[2];
#pragma unroll
    for (int g = 0; g < 2; ++g)
        bases[g] = (((lane15 + 4u * (2 * g)) & 15u) << 4) | ((((lane15 + 4u * (2 * g + 1)) & 15u) << 4) << 16);
    const char *lut_bytes = reinterpret_cast<const char *>(sm.lut);

    for (;;) {
        if (threadIdx.x == 0) sm.item = (int)atomicAdd(a.work_counter, 1u);
        __syncthreads();
        const int item = sm.item;
        if (item >= a.nitems) break;
        const int group = item % a.ngroups, chunk = item / a.ngroups;
        const int64_t cbeg = (int64_t)chunk * a.chunk_codes;
        const int64_t cend = cbeg + a.chunk_codes < a.n ? cbeg + a.chunk_codes : a.n;
        const int ncodes = cend > cbeg ? (int)(cend - cbeg) : 0;

        if (threadIdx.x < DQ16_QB) {
            const int gq = group * DQ16_QB + threadIdx.x;
            uint32_t thr = 0;   // empty slot: nothing passes
            if (gq < a.nq) {
                const uint32_t b = MODE == 0 ? __hip_atomic_load(&a.g_bound[gq], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                             : a.bucket[gq];
                thr = b + 1u;   // at most DQ_BINS
            }
            sm.thr[threadIdx.x] = thr;
        }
        if (MODE == 0)
            for (int i = threadIdx.x; i < DQ16_QB * DQ_BINS; i += DQ_THREADS) (&sm.hist[0][0])[i] = 0u;
        {   // exact tables of the group's queries: entry (table t, byte b) of all 16 queries in one slot
            const int b = threadIdx.x >> 2, t = threadIdx.x & 3;
            uint32_t v[DQ16_QB];
#pragma unroll
            for (int q = 0; q < DQ16_QB; ++q) {
                const int gq = group * DQ16_QB + q;
                v[q] = gq < a.nq ? (uint32_t)a.qluts[((size_t)gq * DQ_M + t) * 256 + b] : 255u;
            }
            sm.lutx[t][b] = make_uint4(v[0] | (v[1] << 8) | (v[2] << 16) | (v[3] << 24), v[4] | (v[5] << 8) | (v[6] << 16) | (v[7] << 24),
                                       v[8] | (v[9] << 8) | (v[10] << 16) | (v[11] << 24), v[12] | (v[13] << 8) | (v[14] << 16) | (v[15] << 24));
        }
        __syncthreads();
        {   // minima: wave w takes rows (q, t) = 4w .. 4w + 3 of the 64, four entries per lane
            const uint8_t *xb = reinterpret_cast<const uint8_t *>(sm.lutx);
            for (int row = wave * 4; row < wave * 4 + 4; ++row) {
                const int q = row >> 2, t = row & 3;
                uint32_t mn = 255u;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t v = xb[((size_t)t * 256 + lane + 64 * i) * 16 + q];
                    mn = v < mn ? v : mn;
                }
                for (int o = 32; o > 0; o >>= 1) { const uint32_t other = __shfl_xor(mn, o); mn = other < mn ? other : mn; }
                if (lane == 0) sm.tmin[q][t] = mn;
            }
        }
        __syncthreads();
        // lower-bound tables from the exact ones at the thresholds of the moment (all threads; ends with a barrier)
        auto build_bounds = [&]() {
            if (threadIdx.x < DQ16_QB) {
                const int q = threadIdx.x;
                const uint32_t off = sm.tmin[q][0] + sm.tmin[q][1] + sm.tmin[q][2] + sm.tmin[q][3];
                const uint32_t thr = sm.thr[q];
                float scale = 0.f;   // every bound 0: every code goes to the exact test
                if (thr > off) scale = DQ16_RANGE / (float)(thr - off);
                sm.off[q] = (float)off;
                sm.scale[q] = scale;
            }
            __syncthreads();
            {
                const int b = threadIdx.x >> 2, t = threadIdx.x & 3;
                const uint4 x = sm.lutx[t][b];
                const uint32_t xw[4] = {x.x, x.y, x.z, x.w};
                uint32_t l[DQ16_QB];
#pragma unroll
                for (int q = 0; q < DQ16_QB; ++q) {
                    const uint32_t e = (xw[q >> 2] >> (8 * (q & 3))) & 255u;
                    const float v = (float)(e - sm.tmin[q][t]) * sm.scale[q];
                    l[q] = sm.thr[q] != 0u ? (uint32_t)fminf(floorf(v), DQ16_ENTRY_MAX) : (uint32_t)DQ16_ENTRY_MAX;
                }
                const uint4 pk = make_uint4(l[0] | (l[1] << 8) | (l[2] << 16) | (l[3] << 24), l[4] | (l[5] << 8) | (l[6] << 16) | (l[7] << 24),
                                            l[8] | (l[9] << 8) | (l[10] << 16) | (l[11] << 24), l[12] | (l[13] << 8) | (l[14] << 16) | (l[15] << 24));
#pragma unroll
                for (int c = 0; c < 4; ++c) sm.lut[b * 16 + t * 4 + c] = pk;
            }
            __syncthreads();
        };
        build_bounds();

        const uint8_t *chunk_ptr = a.codes + cbeg * 8;
        const int nfull = ncodes / DQ_SUB;                       // sub-tiles with every code present
        const int nsub = (ncodes + DQ_SUB - 1) / DQ_SUB;         // the last one may be ragged
        uint32_t tau[4];   // 0x80 minus the threshold (in units of the bounds) of the 16 queries, four per register
        auto reload_tau = [&]() {
            const int ql = lane & (DQ16_QB - 1);
            const uint32_t thr = sm.thr[ql];
            const float t = floorf(((float)thr - 1.f - sm.off[ql]) * sm.scale[ql]) + 2.f;
            const uint32_t t8 = thr != 0u ? (uint32_t)fmaxf(fminf(t, 127.f), 0.f) : 0u;
#pragma unroll
            for (int p = 0; p < 4; ++p)
                tau[p] = 0x80808080u - (__builtin_amdgcn_readlane(t8, 4 * p) | (__builtin_amdgcn_readlane(t8, 4 * p + 1) << 8) |
                                        (__builtin_amdgcn_readlane(t8, 4 * p + 2) << 16) | (__builtin_amdgcn_readlane(t8, 4 * p + 3) << 24));
        };
        typedef uint32_t v4u __attribute__((ext_vector_type(4)));
        typedef const __attribute__((address_space(1))) v4u *global_v4u;
        // the two codes at rows pos, pos + 1 of the chunk (zeros for rows past its end)
        auto load_pair = [&](int pos) -> uint4 {
            uint4 c = make_uint4(0, 0, 0, 0);
            const uint8_t *p = chunk_ptr + (size_t)pos * 8;
            if (pos + 2 <= ncodes) {
                c = *reinterpret_cast<const uint4 *>(p);
            } else if (pos < ncodes) {
                const uint2 half = *reinterpret_cast<const uint2 *>(p);
                c.x = half.x; c.y = half.y;
            }
            return c;
        };
        // the eight table reads of the lane's two codes (four tables each, in the lane's rotated order)
        auto issue = [&](const uint4 c, uint4 (&v)[8]) {
            uint32_t w[4] = {c.x, c.y, c.z, c.w};
            rot8(w[0], w[1], (rot & 4u) != 0, rot & 3u);
            rot8(w[2], w[3], (rot & 4u) != 0, rot & 3u);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint32_t word = w[2 * h + (s >> 1)];
                    const uint32_t off = (s & 1) ? lut_offset<2>(word, bases[s >> 1]) : lut_offset<0>(word, bases[s >> 1]);
                    v[4 * h + s] = *reinterpret_cast<const uint4 *>(lut_bytes + off);
                }
            }
        };
        // One sub-tile whose reads are on their way: the bounds of the two codes for the 16 queries (four bytes per
        // word), one add per word against the thresholds, the rows of the lanes with a bound below one parked.
        int ring_cnt = 0;
        auto finish = [&](const uint4 (&v)[8], const int sidx) {
            uint32_t keep = 0x80808080u;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                keep &= v[4 * h].x + v[4 * h + 1].x + v[4 * h + 2].x + v[4 * h + 3].x + tau[0];
                keep &= v[4 * h].y + v[4 * h + 1].y + v[4 * h + 2].y + v[4 * h + 3].y + tau[1];
                keep &= v[4 * h].z + v[4 * h + 1].z + v[4 * h + 2].z + v[4 * h + 3].z + tau[2];
                keep &= v[4 * h].w + v[4 * h + 1].w + v[4 * h + 2].w + v[4 * h + 3].w + tau[3];
            }
            const uint64_t hit = __ballot(keep != 0x80808080u);
            if (__builtin_expect(hit != 0ull, 0)) {
                if ((hit >> lane) & 1ull) sm.ring[wave][ring_cnt + mask_prefix(hit)] = (uint32_t)(sidx * DQ_SUB + lane * 2);
                ring_cnt += __popcll(hit);
            }
        };
        auto scan_sub = [&](const uint4 c, const int sidx) {
            uint4 v[8];
            issue(c, v);
            asm volatile("" : : : "memory");   // all eight reads are issued before the first add
            finish(v, sidx);
        };

        // Parked rows, 64 at a time: the exact sums of the two codes of a row for the 16 queries (the 16 bytes of a
        // slot split into even and odd queries, two 16-bit sums per word: word p of `ev` holds queries 4p and 4p + 2,
        // word p of `od` queries 4p + 1 and 4p + 3), the test against the thresholds of now, and for every
        // (code, query) that passes the bucket count or the list append.
        auto flush = [&](const int count) {
            const uint32_t thr_lane = sm.thr[lane & (DQ16_QB - 1)];
            uint32_t comp_ev[4], comp_od[4];   // 0x8000 - threshold (thresholds are at most 1024)
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                comp_ev[p] = 0x80008000u - (__builtin_amdgcn_readlane(thr_lane, 4 * p) | (__builtin_amdgcn_readlane(thr_lane, 4 * p + 2) << 16));
                comp_od[p] = 0x80008000u - (__builtin_amdgcn_readlane(thr_lane, 4 * p + 1) | (__builtin_amdgcn_readlane(thr_lane, 4 * p + 3) << 16));
            }
            for (int base = 0; base < count; base += 64) {
                const bool have = base + lane < count;
                const int pos = have ? (int)sm.ring[wave][base + lane] : ncodes;
                const uint4 c = load_pair(pos);
                uint32_t ev[2][4], od[2][4];
                uint32_t m = 0;   // bit h * 16 + q: code h of the row is wanted by query q
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t w0 = h == 0 ? c.x : c.z, w1 = h == 0 ? c.y : c.w;
                    const uint32_t idx[4] = {w0 & 255u, (w0 >> 16) & 255u, w1 & 255u, (w1 >> 16) & 255u};
#pragma unroll
                    for (int p = 0; p < 4; ++p) { ev[h][p] = 0; od[h][p] = 0; }
#pragma unroll
                    for (int t = 0; t < DQ_M; ++t) {
                        const uint4 x = sm.lutx[t][idx[t]];
                        const uint32_t xw[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                        for (int p = 0; p < 4; ++p) {
                            ev[h][p] += xw[p] & 0x00ff00ffu;
                            od[h][p] += (xw[p] >> 8) & 0x00ff00ffu;
                        }
                    }
                    if (pos + h < ncodes) {
#pragma unroll
                        for (int p = 0; p < 4; ++p) {
                            // bit 15 / 31 of sum + (0x8000 - threshold) is clear iff the sum is below the threshold
                            const uint32_t fe = ~(ev[h][p] + comp_ev[p]), fo = ~(od[h][p] + comp_od[p]);
                            const uint32_t nib = ((fe >> 15) & 1u) | (((fo >> 15) & 1u) << 1) | (((fe >> 31) & 1u) << 2) | (((fo >> 31) & 1u) << 3);
                            m |= nib << (h * 16 + 4 * p);
                        }
                    }
                }
                if (MODE == 0) {
                    uint32_t bits = m;
                    while (bits != 0u) {
                        const int bit = __builtin_ctz(bits);
                        bits &= bits - 1u;
                        const int q = bit & 15, h = bit >> 4, p = q >> 2;
                        uint32_t word = (q & 1) ? (h == 0 ? od[0][0] : od[1][0]) : (h == 0 ? ev[0][0] : ev[1][0]);
#pragma unroll
                        for (int i = 1; i < 4; ++i)
                            word = p == i ? ((q & 1) ? (h == 0 ? od[0][i] : od[1][i]) : (h == 0 ? ev[0][i] : ev[1][i])) : word;
                        const uint32_t sum = (q & 2) ? word >> 16 : word & 0xffffu;
                        atomicAdd(&sm.hist[q][sum], 1u);
                    }
                } else {
                    if (__ballot(m != 0u) == 0ull) continue;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
#pragma unroll
                        for (int q = 0; q < DQ16_QB; ++q) {
                            const bool pass = ((m >> (h * 16 + q)) & 1u) != 0u;
                            const uint64_t mask = __ballot(pass);
                            if (mask != 0ull) {
                                const uint32_t word = (q & 1) ? od[h][q >> 2] : ev[h][q >> 2];
                                const uint32_t sum = (q & 2) ? word >> 16 : word & 0xffffu;
                                const int gq = group * DQ16_QB + q;
                                const int first = __builtin_ctzll(mask);
                                uint32_t slot = 0;
                                if (lane == first) slot = atomicAdd(&a.cand_cnt[gq], (uint32_t)__popcll(mask));
                                slot = __shfl(slot, first);
                                // (the list holds exactly the vectors the first pass counted; the
                                // comparison only keeps a disagreement from writing past it)
                                const uint64_t at = a.cand_off[gq] + slot + (uint32_t)mask_prefix(mask);
                                if (pass && at < a.cand_off[gq + 1]) a.cand[at] = ((uint64_t)sum << 32) | (uint32_t)(cbeg + pos + h);
                            }
                        }
                    }
                }
            }
        };

        // Counting pass: the bound of a query is lowered from the block's own counts while the item
        // runs (one wave per query), early and then every 16 groups.
        auto refresh = [&]() {
            const int q = wave;
            if (group * DQ16_QB + q >= a.nq) return;
            const int b = first_bin_reaching([&](int i) { return sm.hist[q][i]; }, (uint32_t)a.r2, nullptr);
            if (b < DQ_BINS && lane == 0) atomicMin(&sm.thr[q], (uint32_t)b + 1u);
        };

        const int ngroups_t = nfull / DQ16_DEPTH;
        int it = 0;
        uint4 cur[DQ16_DEPTH];
#pragma unroll
        for (int u = 0; u < DQ16_DEPTH; ++u) cur[u] = make_uint4(0, 0, 0, 0);
        const uint8_t *gp = chunk_ptr + (size_t)wave * (DQ16_DEPTH * DQ_SUB * 8) + lane * 16;
        auto load_group_sub = [&](const uint8_t *p, int u) -> uint4 {
            const v4u v = *(global_v4u)(p + u * (DQ_SUB * 8));
            return make_uint4(v.x, v.y, v.z, v.w);
        };
        if (wave < ngroups_t) {
#pragma unroll
            for (int u = 0; u < DQ16_DEPTH; ++u) cur[u] = load_group_sub(gp, u);
        }
        reload_tau();
        for (int g = wave; g < ngroups_t; g += DQ_WAVES) {
            const bool more = g + DQ_WAVES < ngroups_t;
            gp += (size_t)DQ_WAVES * (DQ16_DEPTH * DQ_SUB * 8);
            // the table reads of sub-tile u + 1 are issued before the sums of sub-tile u are formed
            uint4 va[8], vb[8];
            issue(cur[0], va);
            if (more) cur[0] = load_group_sub(gp, 0);
#pragma unroll
            for (int u = 0; u < DQ16_DEPTH; ++u) {
                if (u + 1 < DQ16_DEPTH) {
                    issue(cur[u + 1], (u & 1) ? va : vb);
                    if (more) cur[u + 1] = load_group_sub(gp, u + 1);
                }
                asm volatile("" : : : "memory");
                finish((u & 1) ? vb : va, g * DQ16_DEPTH + u);
            }
            if (__builtin_expect(ring_cnt >= 64, 0)) {
                const int whole = ring_cnt & ~63;
                flush(whole);
                for (int i = lane; i < ring_cnt - whole; i += 64) {   // the rest moves to the front
                    const uint32_t v = sm.ring[wave][whole + i];
                    sm.ring[wave][i] = v;
                }
                ring_cnt -= whole;
            }
            if (MODE == 0) {
                if ((it & (it + 1)) == 0 || (it & 15) == 15) refresh();
                // every wave of the block runs iteration `it` iff its last wave does: then all of them meet here
                if ((it == 3 || it == 15 || it == 63) && DQ_WAVES * it + DQ_WAVES - 1 < ngroups_t) {
                    __syncthreads();
                    build_bounds();
                }
                reload_tau();
            }
            ++it;
        }
        // sub-tiles past the last whole group, the ragged one included
        for (int sidx = ngroups_t * DQ16_DEPTH + wave; sidx < nsub; sidx += DQ_WAVES)
            scan_sub(load_pair(sidx * DQ_SUB + lane * 2), sidx);
        if (ring_cnt > 0) flush(ring_cnt);

        if (MODE == 0) {
            // the block's counts join the query's device-wide buckets, whose bound then serves
            // every block that starts an item of this query later
            __syncthreads();
            for (int i = threadIdx.x; i < DQ16_QB * DQ_BINS; i += DQ_THREADS) {
                const int q = i / DQ_BINS, bin = i % DQ_BINS;
                const uint32_t v = sm.hist[q][bin];
                const int gq = group * DQ16_QB + q;
                if (v != 0u && gq < a.nq) atomicAdd(&a.g_hist[(size_t)gq * DQ_BINS + bin], v);
            }
            __syncthreads();
            if (group * DQ16_QB + wave < a.nq) {
                const int gq = group * DQ16_QB + wave;
                const uint32_t *gh = a.g_hist + (size_t)gq * DQ_BINS;
                const int b = first_bin_reaching(
                    [&](int i) { return __hip_atomic_load(&gh[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); },
                    (uint32_t)a.r2, nullptr);
                if (b < DQ_BINS && lane == 0) atomicMin(&a.g_bound[gq], (uint32_t)b);
            }
        }
    }
}

__global__ void derived_init_kernel(uint32_t *work_counter, uint32_t *g_hist, size_t nhist, uint32_t *g_bound,
                                    uint32_t *cand_cnt, int nq) {
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    if (i0 == 0) *work_counter = 0;
    for (size_t i = i0; i < nhist; i += stride) g_hist[i] = 0u;
    for (size_t i = i0; i < (size_t)nq; i += stride) {
        if (g_bound) g_bound[i] = DQ_BINS - 1;   // no bound yet: every bucket is counted
        if (cand_cnt) cand_cnt[i] = 0u;
    }
}

// One wave per query: the bucket in which the r2-th vector falls (all vectors if there are fewer)
// and the number of vectors in the buckets up to it.
__global__ __launch_bounds__(64) void derived_bucket_kernel(const uint32_t *g_hist, int64_t n, int r2, uint32_t *bucket,
                                                            uint32_t *count) {
    const int q = blockIdx.x;
    const uint32_t *gh = g_hist + (size_t)q * DQ_BINS;
    const uint32_t want = (int64_t)r2 < n ? (uint32_t)r2 : (uint32_t)n;
    uint32_t cnt = 0;
    int b = 0;
    if (want > 0) b = first_bin_reaching([&](int i) { return gh[i]; }, want, &cnt);
    if (threadIdx.x == 0) {
        bucket[q] = (uint32_t)(b < DQ_BINS ? b : DQ_BINS - 1);
        count[q] = cnt;
    }
}

// Offsets of the candidate lists (exclusive prefix sum of the nq counts, one block) and what the host
// needs of them: summary[0] = total, summary[1] = the first query whose count exceeds `cap` (nq if
// none), summary[2] = that query's count.
__global__ __launch_bounds__(1024) void derived_offsets_kernel(const uint32_t *__restrict__ count, int nq, long long cap,
                                                                unsigned long long *__restrict__ cand_off,
                                                                unsigned long long *__restrict__ summary) {
    __shared__ unsigned long long wsum[16];
    __shared__ unsigned long long carry;
    __shared__ int bad;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { carry = 0; bad = nq; }
    __syncthreads();
    for (int base = 0; base < nq; base += 1024) {
        const int q = base + tid;
        const unsigned long long c = q < nq ? count[q] : 0;
        if (q < nq && cap >= 0 && (long long)c > cap) atomicMin(&bad, q);
        unsigned long long incl = c;   // inclusive scan over the wave
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long other = __shfl_up(incl, o);
            if (lane >= o) incl += other;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        unsigned long long before = carry;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        if (q < nq) cand_off[q] = before + incl - c;
        __syncthreads();
        if (tid == 1023) carry = before + incl;
        __syncthreads();
    }
    if (tid == 0) {
        cand_off[nq] = carry;
        summary[0] = carry;
        summary[1] = (unsigned long long)bad;
        summary[2] = bad < nq ? count[bad] : 0;
    }
}

// Step 1.2: greatest compact distance (float tables of the derived quantizers, low bits of the
// indexes; entries added in double in table order, rounded once) among the first `init` codes.
__global__ __launch_bounds__(256) void derived_qmax_kernel(const uint8_t *codes, int init, const float *dluts, float *qmax) {
    __shared__ float red[256];
    const int q = blockIdx.x;
    const float *lut = dluts + (size_t)q * DQ_M * 256;
    float best = 0.f;   // distances are not negative; no code at all gives 0
    for (int i = threadIdx.x; i < init; i += 256) {
        const uint2 c = *reinterpret_cast<const uint2 *>(codes + (size_t)i * 8);
        const double s = (double)lut[c.x & 255u] + (double)lut[256 + ((c.x >> 16) & 255u)] +
                         (double)lut[512 + (c.y & 255u)] + (double)lut[768 + ((c.y >> 16) & 255u)];
        best = fmaxf(best, (float)s);
    }
    red[threadIdx.x] = best;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) qmax[q] = red[0];
}

// Step 2 for one query per block: precise distance of every candidate from the full codebooks
// (each of the four terms ||y^j - C^j[c[j]]||^2 summed in double and rounded to float as the table
// entry of Eq. (tables) would be, the four entries added in double and rounded once, Eq. (adc1)),
// and the topk smallest (distance, row).  Candidates are taken in tiles; a tile's keys below the
// current topk-th are sorted in LDS together with the best so far.
constexpr int RR_THREADS = 1024;
constexpr int RR_KEEP = 128;            // best keys carried from tile to tile (topk <= 128)
constexpr int RR_TILE = 2 * RR_THREADS; // candidates per tile
__global__ __launch_bounds__(RR_THREADS) void derived_rerank_kernel(const uint8_t *codes, const float *codebooks, int k,
                                                                   int dsub, const float *queries, const uint64_t *cand,
                                                                   const uint64_t *cand_off, const int64_t *ids, int topk,
                                                                   float *out_dist, int64_t *out_ids) {
    __shared__ uint64_t keys[RR_KEEP + RR_TILE + RR_KEEP * 15];   // 4096 keys: a power of two above KEEP + TILE
    __shared__ float y[4096];
    __shared__ int nnew;
    const int q = blockIdx.x, tid = threadIdx.x;
    const int d = DQ_M * dsub;
    for (int i = tid; i < d; i += RR_THREADS) y[i] = queries[(size_t)q * d + i];
    for (int i = tid; i < RR_KEEP; i += RR_THREADS) keys[i] = KEY_EMPTY;
    if (tid == 0) nnew = 0;
    __syncthreads();
    const uint64_t begin = cand_off[q], end = cand_off[q + 1];
    for (uint64_t base = begin; base < end; base += RR_TILE) {
        const uint64_t bound = keys[topk - 1];
        for (int u = 0; u < 2; ++u) {
            const uint64_t ci = base + (uint64_t)u * RR_THREADS + tid;
            if (ci >= end) continue;
            const uint32_t row = (uint32_t)cand[ci];
            const uint2 c = *reinterpret_cast<const uint2 *>(codes + (size_t)row * 8);
            uint32_t idx[4] = {c.x & 0xffffu, c.x >> 16, c.y & 0xffffu, c.y >> 16};
#pragma unroll
            for (int j = 0; j < DQ_M; ++j) idx[j] = idx[j] < (uint32_t)k ? idx[j] : (uint32_t)k - 1u;   // indexes are below k by contract
            double total = 0.0;
#pragma unroll
            for (int j = 0; j < DQ_M; ++j) {
                const float *cent = codebooks + ((size_t)j * k + idx[j]) * dsub;
                const float *yj = y + j * dsub;
                double s = 0.0;
                for (int t = 0; t < dsub; ++t) {
                    const double diff = (double)yj[t] - (double)cent[t];
                    s += diff * diff;
                }
                total += (double)(float)s;
            }
            const uint64_t key = ((uint64_t)f32_to_ord((float)total) << 32) | row;
            if (key < bound) keys[RR_KEEP + atomicAdd(&nnew, 1)] = key;
        }
        __syncthreads();
        const int total = RR_KEEP + nnew;
        if (nnew > 0) {
            int n2 = 256;
            while (n2 < total) n2 <<= 1;
            for (int i = total + tid; i < n2; i += RR_THREADS) keys[i] = KEY_EMPTY;
            block_bitonic_sort(keys, n2);
        }
        __syncthreads();
        if (tid == 0) nnew = 0;
        __syncthreads();
    }
    for (int i = tid; i < topk; i += RR_THREADS) {
        const uint64_t key = keys[i];
        const bool have = key != KEY_EMPTY;
        out_dist[(size_t)q * topk + i] = have ? ord_to_f32((uint32_t)(key >> 32)) : __builtin_inff();
        const uint32_t row = (uint32_t)key;
        out_ids[(size_t)q * topk + i] = have ? (ids ? ids[row] : (int64_t)row) : -1;
    }
}

// candidate rows of every query as [nq][cap] ids (ascending positions in the list are not sorted), padded with -1
__global__ void derived_export_kernel(const uint64_t *cand, const uint64_t *cand_off, int64_t cap, int64_t *out) {
    const int q = blockIdx.y;
    const uint64_t begin = cand_off[q], cnt = cand_off[q + 1] - begin;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cap; i += (int64_t)gridDim.x * blockDim.x)
        out[(size_t)q * cap + i] = (uint64_t)i < cnt ? (int64_t)(uint32_t)cand[begin + i] : -1;
}

__global__ void derived_widen_kernel(const uint32_t *src, int n, int64_t *dst) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (int64_t)src[i];
}

}  // namespace

int launch_derived_search(pq_ctx *ctx, const uint16_t *codes16, int64_t n, const float *derived_codebooks,
                          const float *codebooks, int k, const float *queries, int nq, int d, int r2, int topk,
                          float *out_dist, int64_t *out_ids, uint32_t *bucket_out, int64_t *ncand_out,
                          int64_t *cand_ids_out, int64_t cand_cap) {
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(codes16);
    const int dsub = d / DQ_M;
    hipStream_t s = ctx->stream;
    // 640 queries and more (measured on 25 M codes: 512 queries 4.45 -> 4.90 ms per call, 700 queries 6.23 -> 6.06 ms,
    // 1000 queries 8.30 -> 7.87 ms): the collecting pass takes 16 queries per pass over the codes (PQ_SCAN_Q8=0: 8, as
    // for fewer queries).  The counting pass stays with 8: its bound is the loose one of the block's own counts for most of
    // an item, so a large share of the codes needs exact sums, which the 8-query loop has at hand and the 16-query
    // loop fetches again (measured: 3.7 ms against 5.0 ms, 4.7 ms with a first bound from a sample).
    const bool wide = nq >= 640 && opt_int(ctx, PQ_OPT_SCAN_Q8, 1) != 0;

    // work items: chunk of codes x group of 8 or 16 queries, chunk-major (blocks running together share chunks)
    struct Geometry { int ngroups, nblocks; int64_t nchunks, chunk_codes, nitems; };
    auto geometry = [&](int qb) {
        Geometry g;
        g.ngroups = (nq + qb - 1) / qb;
        const int64_t block_tile = (int64_t)DQ_SUB * DQ_WAVES;
        int nblocks_max = opt_int(ctx, PQ_OPT_SCAN_BLOCKS, ctx->num_cu);
        if (nblocks_max < 1) nblocks_max = 1;
        int64_t nchunks = ((int64_t)opt_int(ctx, PQ_OPT_SCAN_ITEMS_PER_BLOCK, 4) * nblocks_max + g.ngroups - 1) / g.ngroups;
        const int64_t max_by_n = (n + 8 * block_tile - 1) / (8 * block_tile);
        if (nchunks > max_by_n) nchunks = max_by_n;
        const int64_t min_chunks = (n + ((int64_t)1 << 30) - 1) >> 30;   // a chunk's rows are counted in 32 bits
        if (nchunks < min_chunks) nchunks = min_chunks;
        if (nchunks < 1) nchunks = 1;
        int64_t chunk_codes = (n + nchunks - 1) / nchunks;
        chunk_codes = (chunk_codes + block_tile - 1) / block_tile * block_tile;
        if (chunk_codes < block_tile) chunk_codes = block_tile;
        g.chunk_codes = chunk_codes;
        g.nchunks = n > 0 ? (n + chunk_codes - 1) / chunk_codes : 0;
        g.nitems = g.nchunks * g.ngroups;
        g.nblocks = (int)(g.nitems < nblocks_max ? g.nitems : nblocks_max);
        return g;
    };
    const Geometry g_count = geometry(DQ_QB), g_collect = geometry(wide ? DQ16_QB : DQ_QB);
    if (g_count.nitems > 0x3fffffff) return fail(ctx, PQ_EUNSUPPORTED, "derived_search: too many work items (%lld)", (long long)g_count.nitems);
    auto bind_geometry = [&](DqArgs &a, const Geometry &g) {
        a.chunk_codes = g.chunk_codes; a.nchunks = (int)g.nchunks; a.ngroups = g.ngroups; a.nitems = (int)g.nitems;
    };

    // workspace, first part: tables and counts
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes, 256); return o; };
    const size_t o_counter = take(256);
    const size_t o_dluts = take((size_t)nq * DQ_M * 256 * 4);
    const size_t o_qmax = take((size_t)nq * 4);
    const size_t o_qmin = take((size_t)nq * 4);
    const size_t o_scale = take((size_t)nq * 4);
    const size_t o_qluts = take((size_t)nq * DQ_M * 256);
    const size_t o_hist = take((size_t)nq * DQ_BINS * 4);
    const size_t o_bound = take((size_t)nq * 4);
    const size_t o_bucket = take((size_t)nq * 4);
    const size_t o_count = take((size_t)nq * 4);
    const size_t o_candcnt = take((size_t)nq * 4);
    const size_t o_candoff = take((size_t)(nq + 1) * 8);

    auto prepare = [&](uint8_t *ws) -> int {   // Steps 1.1 and 1.2
        float *dluts = (float *)(ws + o_dluts), *qmax = (float *)(ws + o_qmax);
        int rc = launch_build_luts(ctx, queries, derived_codebooks, nq, d, DQ_M, 256, dluts);
        if (rc) return rc;
        const int init = (int)((int64_t)r2 < n ? (int64_t)r2 : n);
        derived_qmax_kernel<<<nq, 256, 0, s>>>(codes, init, dluts, qmax);
        PQ_HIP(ctx, hipGetLastError());
        return launch_quantize_luts(ctx, dluts, nq, DQ_M, 256, qmax, ws + o_qluts, (float *)(ws + o_qmin),
                                    (float *)(ws + o_scale));
    };

    const size_t o_summary = take(256);
    const size_t first_part_all = off;
    int rc = ws_reserve(ctx, first_part_all);
    if (rc) return rc;
    if (!ctx->host_pin) {   // a few words of pinned host memory, kept by the context
        void *p = nullptr;
        PQ_HIP(ctx, hipHostMalloc(&p, 256, hipHostMallocDefault));
        ctx->host_pin = p;
    }
    DqArgs a;
    a.codes = codes; a.n = n; a.nq = nq; a.r2 = r2;
    // Steps 1.1 to 1.3 (counting pass) in the workspace `ws`; leaves the buckets, the counts and the
    // offsets of the candidate lists there and brings their total (and the first list beyond
    // cand_cap, if any) to the host: three words through pinned memory.
    auto count_pass = [&](uint8_t *ws, unsigned long long *total) -> int {
        int rc = prepare(ws);
        if (rc) return rc;
        bind_geometry(a, g_count);
        a.qluts = ws + o_qluts;
        a.work_counter = (uint32_t *)(ws + o_counter);
        a.g_hist = (uint32_t *)(ws + o_hist);
        a.g_bound = (uint32_t *)(ws + o_bound);
        a.bucket = nullptr; a.cand_off = nullptr; a.cand_cnt = nullptr; a.cand = nullptr;
        derived_init_kernel<<<256, 256, 0, s>>>(a.work_counter, a.g_hist, (size_t)nq * DQ_BINS, a.g_bound, nullptr, nq);
        PQ_HIP(ctx, hipGetLastError());
        if (ctx->profiling) {
            note_plain_scan(ctx, "derived_scan_kernel<count> (8 queries per pass)", 8, g_count.ngroups);
            PQ_HIP(ctx, hipEventRecord(ctx->ev_begin, s));
        }
        if (g_count.nblocks > 0) {
            derived_scan_kernel<0><<<g_count.nblocks, DQ_THREADS, 0, s>>>(a);
            PQ_HIP(ctx, hipGetLastError());
        }
        if (ctx->profiling) {
            PQ_HIP(ctx, hipEventRecord(ctx->ev_end, s));
            ctx->ev_valid = 1;
        }
        derived_bucket_kernel<<<nq, 64, 0, s>>>(a.g_hist, n, r2, (uint32_t *)(ws + o_bucket), (uint32_t *)(ws + o_count));
        PQ_HIP(ctx, hipGetLastError());
        derived_offsets_kernel<<<1, 1024, 0, s>>>((const uint32_t *)(ws + o_count), nq, cand_ids_out ? (long long)cand_cap : -1,
                                                  (unsigned long long *)(ws + o_candoff), (unsigned long long *)(ws + o_summary));
        PQ_HIP(ctx, hipGetLastError());
        unsigned long long *pin = (unsigned long long *)ctx->host_pin;
        PQ_HIP(ctx, hipMemcpyAsync(pin, ws + o_summary, 24, hipMemcpyDeviceToHost, s));
        PQ_HIP(ctx, hipStreamSynchronize(s));
        if (pin[1] < (unsigned long long)nq)
            return fail(ctx, PQ_ESHAPE, "derived_search: query %d has %u candidates, cand_cap is %lld", (int)pin[1], (unsigned)pin[2],
                        (long long)cand_cap);
        *total = pin[0];
        return PQ_OK;
    };
    uint8_t *ws = (uint8_t *)ctx->ws;
    unsigned long long total = 0;
    rc = count_pass(ws, &total);
    if (rc) return rc;
    // the sizes of the candidate lists decide the rest of the workspace
    const size_t o_cand = take((size_t)total * 8);
    if (off > ctx->ws_bytes) {   // a new workspace: the counting pass is made again there (same bits)
        rc = ws_reserve(ctx, off);
        if (rc) return rc;
        ws = (uint8_t *)ctx->ws;
        unsigned long long again = 0;
        rc = count_pass(ws, &again);
        if (rc) return rc;
        if (again != total) return fail(ctx, PQ_EHIP, "derived_search: the counting pass gave %llu candidates, then %llu", total, again);
    }

    // Step 1.3, collecting pass
    a.qluts = ws + o_qluts;
    a.work_counter = (uint32_t *)(ws + o_counter);
    a.g_hist = nullptr; a.g_bound = nullptr;
    a.bucket = (const uint32_t *)(ws + o_bucket);
    a.cand_off = (const uint64_t *)(ws + o_candoff);
    a.cand_cnt = (uint32_t *)(ws + o_candcnt);
    a.cand = (uint64_t *)(ws + o_cand);
    derived_init_kernel<<<256, 256, 0, s>>>(a.work_counter, nullptr, 0, nullptr, a.cand_cnt, nq);
    PQ_HIP(ctx, hipGetLastError());
    bind_geometry(a, g_collect);
    if (g_collect.nblocks > 0) {
        if (wide) derived_scan16_kernel<1><<<g_collect.nblocks, DQ_THREADS, 0, s>>>(a);
        else derived_scan_kernel<1><<<g_collect.nblocks, DQ_THREADS, 0, s>>>(a);
        PQ_HIP(ctx, hipGetLastError());
    }
    // Step 2
    derived_rerank_kernel<<<nq, RR_THREADS, 0, s>>>(codes, codebooks, k, dsub, queries, a.cand, a.cand_off, nullptr, topk,
                                                    out_dist, out_ids);
    PQ_HIP(ctx, hipGetLastError());
    if (bucket_out) PQ_HIP(ctx, hipMemcpyAsync(bucket_out, ws + o_bucket, (size_t)nq * 4, hipMemcpyDeviceToDevice, s));
    if (ncand_out) {
        derived_widen_kernel<<<(nq + 255) / 256, 256, 0, s>>>((const uint32_t *)(ws + o_count), nq, ncand_out);
        PQ_HIP(ctx, hipGetLastError());
    }
    if (cand_ids_out && cand_cap > 0) {
        derived_export_kernel<<<dim3(64, nq), 256, 0, s>>>(a.cand, a.cand_off, cand_cap, cand_ids_out);
        PQ_HIP(ctx, hipGetLastError());
    }
    return PQ_OK;
}

}  // namespace pq
