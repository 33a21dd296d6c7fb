// Tuned scan kernels (Alg. 1 `scan`/`adc`, Eq. (adc1); Alg. 3 for packed 4-bit codes):
//   F32_M8  : 8 float tables of 256 entries, 8-byte codes, 4 queries per block
//   F32_M16 : 16 float tables of 256 entries, 16-byte codes, 4 queries per block
//   U4_M16  : 16 tables of 16 bytes merged in pairs to 8 tables of 256 16-bit entries,
//             8-byte packed codes, 8 queries per block
//
// LDS layout (64 KB).  Row b (256 bytes) holds, for code-byte value b, 16 slots of 16 bytes.
// A slot is the entry of one table for all queries of the block (4 floats, or 8 x u16).
// With 8 tables every table owns two slots (two copies), with 16 tables one.  The LDS
// serves a 16-byte read of a wave in passes of 16 lanes that differ in the low four lane
// bits, and two lanes of a pass collide unless they hit different 16-byte bank groups
// (or the same address).  Lane l therefore reads slot ((l & 15) + S*s) & 15 at step s
// (S = 2 with copies, 1 without): the 16 lanes of a pass always hit 16 different slots, so
// every read is conflict-free whatever the code bytes are.  Each lane walks the tables in
// its own rotated order, which only permutes the order of the float additions.
//
// Work distribution.  A fixed number of persistent blocks (one per CU) take work items
// (chunk of codes x group of queries) from a device counter, chunk-major, so that blocks
// running at the same time share code chunks in L2 and later chunks start with the bounds
// the earlier ones found.
//
// Top-k.  Per wave and query a bounded candidate list in device scratch, as in the general
// kernel, plus a per-query histogram of the values of the candidates inserted by any wave.
// The smallest bin edge below which k candidates have been counted is a valid bound on the
// k-th smallest value of the whole scan and is shared through one word per query.  Integer
// sums index the bins directly.  Float values are binned by their distance, in ordered-bit
// units, below a per-query reference (the first bound any wave publishes): bin width 2^14
// units (about 0.2 % of the value), 4096 bins reaching down to 1/256 of the reference, smaller
// values lumped in the first bin; candidates seen before the reference exists are not counted.
#include <stddef.h>
#include <type_traits>

#include "pq_internal.h"
#include "scan_common.h"
#include "topk_device.h"
#include "lds_walk.h"

// This file is compiled as is (blocks of 16 waves, namespace pq::w16) and once more through
// scan_items_w8.hip (blocks of 8 waves, namespace pq::w8, work items of inverted lists only).
#ifndef PQ_TUNED_NS
#define PQ_TUNED_NS w16
#endif
#ifndef PQ_TUNED_ITEMS_ONLY
#define PQ_TUNED_ITEMS_ONLY 0
#endif

namespace pq {
namespace PQ_TUNED_NS {

// Per-wave selection state kept in LDS: the scan loop itself only holds the thresholds in
// registers; everything else is touched on the rare paths below.
struct WaveState {
    int cnt[16];
    uint32_t own_ord[16];   // k-th smallest value of the wave's own list, ord_inf while not full
};

// wave list capacity in units of 64 keys: 384 keys for results of up to 128, 2048 for up to 1024
constexpr int E_SMALL = 6, E_LARGE = 32;
constexpr int RING_FLUSH = TUNED_WAVES == 8 ? 64 : 192;    // flush when more than this many positions are parked
constexpr int RING_PERIOD = 256;  // and, if anything is parked, every this many iterations

// RING: ring entries per wave
// WIDE16: room for a second set of tables (16-bit entries of 16 queries, 64 KB) beside the scan's own
template <int RING, bool WIDE16 = false>
struct __align__(16) TunedSmemT {
    uint4 lut[4096];
    uint4 lut16[WIDE16 ? 4096 : 1];   // entry (byte b, table j): two 16-byte halves at (b * 8 + j) * 2
    uint8_t qstage[WIDE16 ? 16 : 8][256];
    // Per wave: lanes that found a candidate park the position of their 16 code bytes here; the
    // positions are turned into list inserts in batches (scan_flush), which recomputes the values.
    uint32_t ring[TUNED_WAVES][RING];
    float prune_off[16];      // per slot: sum of the table minima, and the scale of the 16-bit tables
    float prune_scale[16];    // (0: no pruning for this slot, negative: nothing of this slot can qualify)
    float prune_scale16[16];  // 16 queries per pass: scale of the 16-bit tables of the second test
    float pmin[8][16];       // inverted lists: minima of the slot's tables
    uint32_t umin[WIDE16 ? 16 : 1][8];    // integer scan on 8-bit lower bounds: minima of the slot's pair-merged tables
    uint32_t eff_tmp[TUNED_WAVES][16];   // 16-query insert path: the float bounds of the batch being inserted
    WaveState ws[TUNED_WAVES];
    uint32_t tau_blk[16];   // best bound known to the block per query (prunes with "<=")
    unsigned long long tau_key_blk[16];   // the same as a whole key (value, row): keys above it are no candidates
    unsigned long long *tau_key_global[16];
    int out_cnt[16];        // keys handed to the item's result list of each query so far
    uint32_t ncand_blk[16]; // candidates inserted by the block and not yet added to the query's device counter
    uint32_t tau_ref[16];   // histogram reference per query (float path)
    uint32_t hwin_base[16]; // first bin of the query's histogram window (see hist_count)
    unsigned long long stat_parked;   // measurement aid: positions the block's waves have parked
    uint32_t hwin_pending[16];   // keys the block has counted for the query since it last moved the window to device memory
    // per item, written at its start: where the state of the query in each slot lives
    uint32_t *hist[16];
    uint32_t *ncand[16];
    uint32_t *refresh_mark[16];
    uint32_t *tau_ref_global[16];
    const void *slot_lut[16];   // tables of the slot's query (nullptr: empty slot)
    uint64_t *slot_out[16];     // where the slot's KPAD result keys go
    const uint8_t *chunk_ptr;  // first row scanned by the item
    int64_t code_begin;        // its row number
    int ncodes;                // rows scanned
    int skip;                  // leading rows that are not part of the item
    int nvalid;                // slots in use
    int topk;
    int item;
    int next_group;            // next group of sub-tiles to hand to a wave
    int group;                 // flat scan: query group of the item
};

// The helpers below are real functions (kept out of line so that their registers do not weigh on
// the scan loop); they address the block's shared structure (SM, one of the TunedSmemT types)
// through an LDS-qualified pointer.
#define LDS_PTR(T) __attribute__((address_space(3))) T *
typedef __attribute__((address_space(3))) WaveState LdsWaveState;


// Candidate histograms.  Every inserted key is counted in a bin of its query's histogram in device memory, from
// which the shared bound is read.  The keys a block inserts during an item lie at or below the bound the item
// started with and crowd just under it (on encoded data thousands of codes share a handful of integer sums), and
// device-scope atomic adds to one word serialise at the memory side.  The block therefore counts the HWIN bins
// up to that bound in LDS (in the memory that staged the 8-bit tables, which is idle while codes are scanned)
// and adds the window to the device histogram when one of its waves is about to read it (scan_refresh) and at
// the end of the item; keys below the window go to the device histogram directly.  A bound read from counts
// that miss another block's window is looser than it could be, never wrong.
constexpr int HWIN = 64;
typedef __attribute__((address_space(3))) uint32_t LdsU32;
template <class SM>
__device__ __forceinline__ LdsU32 *hist_window(LDS_PTR(SM) sm, int q) {

    return (LdsU32 *)&sm->qstage[0][0] + q * HWIN;
}
template <class SM>
__device__ __forceinline__ void hist_count(LDS_PTR(SM) sm, int q, uint32_t bin) {
    const uint32_t rel = bin - sm->hwin_base[q];
    if (rel < (uint32_t)HWIN) __hip_atomic_fetch_add(hist_window(sm, q) + rel, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __hip_atomic_fetch_add(sm->hist[q] + bin, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// one wave: move the window of query q into the device histogram
template <class SM>
__device__ __forceinline__ void hist_window_flush(LDS_PTR(SM) sm, int q) {
    const int lane = lane_id();
    const uint32_t v = __hip_atomic_exchange(hist_window(sm, q) + lane, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (v != 0u) __hip_atomic_fetch_add(sm->hist[q] + sm->hwin_base[q] + lane, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// KIND_F32P_M8 / _M16: the 8 x 256 and 16 x 256 float scans with pruning by 16-bit lower bounds
// (see scan_flush_pruned)
enum { KIND_F32_M8 = 0, KIND_F32_M16 = 1, KIND_U4_M16 = 2, KIND_F32P_M8 = 3, KIND_F32P_M16 = 4, KIND_F32Q_M8 = 5, KIND_U4Q_M16 = 6 };
constexpr int SEED_CODES_BATCH = 1 << 15;   // codes looked at for the first bound of a float scan of many query groups
constexpr int SEED_CODES_STREAM = 1 << 16;  // codes looked at for the first bound when few groups share the GPU (<= PRUNE_MIN_N)
constexpr int STREAM_GROUPS = 32;          // flat scans of fewer query groups fetch like streaming scans
constexpr int64_t PRUNE_MIN_N = 1 << 16;   // smaller databases take the plain float scan
constexpr int PRUNE_INIT = 4096;           // codes looked at for the first bound of every query
constexpr int PRUNE_MARGIN = 8;      // slack of the integer threshold, in table units
constexpr float PRUNE_RANGE = 3500.f;  // table units between the sum of the minima and the first bound
// KIND_F32Q_M8: the same with 8-bit entries, 16 queries per 16-byte slot: entries of at most 15 (eight of them add
// up to less than 128, so the sums of 16 queries add up byte-wise in four 32-bit words without carries and one
// subtraction per word tests four of them), 64 units between the sum of the minima and the first bound (measured
// optimum: fewer units blur the bound, more let codes with a few saturated entries through)
constexpr float PRUNE_RANGE_Q8 = 64.f;
constexpr float PRUNE_RANGE_U4Q = 48.f;   // the same for the integer scan (measured: 40 .. 56 within 2 % of one another, 64: +4 .. 8 %, 32: +6 .. 16 %)
constexpr int PRUNE_MARGIN_Q8 = 2;   // a candidate's sum is at most floor(bound in units) up to fp32 rounding of that conversion
constexpr float PRUNE_ENTRY_MAX_Q8 = 15.f;

// What a lane needs to walk the tables in its own rotated order (see the layout note on top):
// derived from the low four bits of the lane that holds the code bytes.
template <int NT>
struct LaneWalk {
    uint32_t rot;            // bytes to rotate the code by
    uint32_t bases[NT / 4];  // slot offsets of the NT steps, four per word
    __device__ __forceinline__ explicit LaneWalk(uint32_t lane15) {
        constexpr int SSTEP = NT == 8 ? 2 : 1;   // slot stride per step
        rot = NT == 8 ? lane15 >> 1 : lane15;
#pragma unroll
        for (int g = 0; g < NT / 4; ++g) {
            bases[g] = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) bases[g] |= (((lane15 + SSTEP * (4 * g + p)) & 15u) << 4) << (8 * p);
        }
    }
};

// Accumulated values of the codes in the 16 bytes `c` (two 8-byte codes or one 16-byte code),
// four accumulators per code: d[h][0..3] = the four queries' float sums, or the eight queries'
// integer sums as four packed pairs.  `ld(offset)` returns the 16-byte LDS slot at that offset.
// READS: table reads issued back to back before their results are added up (16, or 8 where the
// registers are needed for codes on their way).
template <int NT, bool IS_U4, int READS = 16, class Ld>
__device__ __forceinline__ void code_values(const uint4 c, const LaneWalk<NT> &lw, Ld ld, uint32_t (&d)[16 / NT][4]) {
    constexpr int CPL = 16 / NT;
    static_assert(READS == 16 || READS == 8, "a sub-tile is 16 reads per lane");
    uint32_t w[4] = {c.x, c.y, c.z, c.w};
    if constexpr (NT == 8) {
        const bool swap = (lw.rot & 4u) != 0;
        rot8(w[0], w[1], swap, lw.rot & 3u);
        rot8(w[2], w[3], swap, lw.rot & 3u);
    } else {
        rot16(w, lw.rot);
    }
    // read r of the lane: table step r % NT of code r / NT
#pragma unroll
    for (int r0 = 0; r0 < 16; r0 += READS) {
        uint4 v[READS];
#pragma unroll
        for (int r = 0; r < READS; ++r) {
            const int h = (r0 + r) / NT, s = (r0 + r) % NT;
            uint32_t off;
            const uint32_t word = w[h * (NT / 4) + (s >> 2)], bs = lw.bases[s >> 2];
            switch (s & 3) {
                case 0: off = lut_offset<0>(word, bs); break;
                case 1: off = lut_offset<1>(word, bs); break;
                case 2: off = lut_offset<2>(word, bs); break;
                default: off = lut_offset<3>(word, bs); break;
            }
            v[r] = ld(off);
        }
        // every read above is issued before any addition below: the LDS serves them back to back
        // while the first results are already being added up
        asm volatile("" : : : "memory");
#pragma unroll
        for (int r = 0; r < READS; ++r) {
            const int h = (r0 + r) / NT, s = (r0 + r) % NT;
            const uint4 e = v[r];
            if constexpr (IS_U4) {
                if (s == 0) { d[h][0] = e.x; d[h][1] = e.y; d[h][2] = e.z; d[h][3] = e.w; }
                else { d[h][0] += e.x; d[h][1] += e.y; d[h][2] += e.z; d[h][3] += e.w; }
            } else {
                if (s == 0) { d[h][0] = e.x; d[h][1] = e.y; d[h][2] = e.z; d[h][3] = e.w; }
                else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t add = i == 0 ? e.x : i == 1 ? e.y : i == 2 ? e.z : e.w;
                        d[h][i] = __float_as_uint(__uint_as_float(d[h][i]) + __uint_as_float(add));
                    }
                }
            }
        }
    }
}

template <class SM>
__device__ __forceinline__ void publish_bound(LDS_PTR(SM) sm, int q, uint32_t ord) {
    // a bound on the value alone is the key (value, last row)
    const unsigned long long key = ((unsigned long long)ord << 32) | 0xffffffffull;
    __hip_atomic_fetch_min(&sm->tau_blk[q], ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_min(&sm->tau_key_blk[q], key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    atomicMin(sm->tau_key_global[q], key);
}
// `key` is the k-th smallest key of some set of the query's codes: no key above it belongs to the result
template <class SM>
__device__ __forceinline__ void publish_key_bound(LDS_PTR(SM) sm, int q, uint64_t key) {
    __hip_atomic_fetch_min(&sm->tau_blk[q], (uint32_t)(key >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_min(&sm->tau_key_blk[q], (unsigned long long)key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    atomicMin(sm->tau_key_global[q], (unsigned long long)key);
}

// Rare path: the candidate list of query q of this wave is nearly full.  Keep its k smallest
// keys, make the k-th the wave's own bound and share it.  Returns the new count.
template <class SM, int E, bool INTVAL>
__device__ __noinline__ int scan_compact(LDS_PTR(SM) sm, uint64_t *buf, int cnt, int q) {
    const int lane = lane_id();
    LdsWaveState *ws = &sm->ws[threadIdx.x >> 6];
    const uint64_t kth = wave_compact<E>(buf, cnt, sm->topk);
    if (kth != KEY_EMPTY) {
        const uint32_t kord = (uint32_t)(kth >> 32);
        if (lane == 0) {
            ws->own_ord[q] = kord;
            publish_key_bound(sm, q, kth);
        }
        if (!INTVAL && sm->tau_ref[q] == TAU_REF_UNSET) {
            // the first bound published for a query becomes the reference of its histogram
            uint32_t expected = TAU_REF_UNSET;
            __hip_atomic_compare_exchange_strong(sm->tau_ref_global[q], &expected, kord, __ATOMIC_RELAXED,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t now = expected == TAU_REF_UNSET ? kord : expected;
            if (lane == 0) sm->tau_ref[q] = now;
        }
    }
    return cnt;
}

// Rare path of the scan loop: turn the `n` positions parked in the wave's ring into list inserts.
// Lane e takes entry e (64 at a time): it reloads the 16 code bytes at that position and
// recomputes their values exactly as the lane that parked them did (same rotation, same order
// of additions).  Every lane then appends the (value, id) keys of its own codes that are below
// the current bound of a query to the wave's list of that query (slot from an LDS counter) and
// counts them in the query's histogram.  Before a batch, a list that the batch could overflow
// is cut to its k smallest keys.
template <class SM, int KIND, int E>
__device__ __noinline__ int scan_flush(LDS_PTR(SM) sm, uint64_t *wave_buf, int n) {
    constexpr bool IS_U4 = KIND == KIND_U4_M16;
    constexpr int QB = IS_U4 ? 8 : 4;
    constexpr int NT = KIND == KIND_F32_M16 ? 16 : 8;
    constexpr int CPL = 16 / NT;
    constexpr int CAP = 64 * E;
    static_assert(CAP - 64 * CPL >= 128 && (E <= 8 || CAP - 64 * CPL >= 1024), "a compacted list must leave room for one batch");
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    LdsWaveState *ws = &sm->ws[wave];
    const int nvalid = sm->nvalid, skip = sm->skip, ncodes = sm->ncodes;
    const uint32_t row0 = (uint32_t)sm->code_begin;
    const uint8_t *chunk_ptr = sm->chunk_ptr;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const __attribute__((address_space(3))) char *lut_bytes = (const __attribute__((address_space(3))) char *)sm->lut;
    const int ql = lane & (QB - 1);
    int appended = 0;   // keys added to the wave's lists (returned)
    for (int base = 0; base < n; base += 64) {
        // room for 64 * CPL more keys in every list
        uint32_t full = (uint32_t)__ballot(ws->cnt[ql] > CAP - 64 * CPL) & ((1u << QB) - 1u);
        while (full != 0u) {
            const int q = __builtin_ctz(full);
            full &= full - 1u;
            const int cnt = scan_compact<SM, E, IS_U4>(sm, wave_buf + (size_t)q * CAP, ws->cnt[q], q);
            if (lane == 0) ws->cnt[q] = cnt;
        }
        const bool have = base + lane < n;
        const int pos = have ? (int)sm->ring[wave][base + lane] : 0;   // position of the 16 bytes' first code
        uint4 c = make_uint4(0, 0, 0, 0);
        if (have) {
            const uint8_t *p = chunk_ptr + (size_t)(pos / CPL) * 16;
            if (pos + CPL <= ncodes) {
                c = *reinterpret_cast<const uint4 *>(p);
            } else if (CPL == 2 && pos < ncodes) {   // last lane of a ragged chunk: only its first code exists
                const uint2 half = *reinterpret_cast<const uint2 *>(p);
                c.x = half.x; c.y = half.y;
            }   // (lanes past the end of a ragged chunk park positions too: nothing to load, never inserted)
        }
        const LaneWalk<NT> lw((uint32_t)(pos / CPL) & 15u);   // the parking lane's walk
        uint32_t acc[CPL][4];
        code_values<NT, IS_U4>(c, lw, [&](uint32_t off) {
            const v4u v = *(const __attribute__((address_space(3))) v4u *)(lut_bytes + off);
            return make_uint4(v.x, v.y, v.z, v.w);
        }, acc);
        // codes outside the item (and lanes without an entry) never qualify
        bool ok[CPL];
#pragma unroll
        for (int h = 0; h < CPL; ++h) ok[h] = have && pos + h >= skip && pos + h < ncodes;
        // candidates satisfy value < eff: the wave's own bound is strict, the block's is "<=".
        // Lane q works out the bound of query q; the loop below picks it up with a lane read.
        uint32_t eff_lane;
        {
            const uint32_t shared = sm->tau_blk[ql];
            const uint32_t loose = shared == 0xffffffffu ? shared : shared + 1u;
            const uint32_t own = ws->own_ord[ql];
            eff_lane = own < loose ? own : loose;
        }
        // bit h * QB + q of m: code h of this lane qualifies for query q
        uint32_t m = 0;
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const uint32_t eff = __builtin_amdgcn_readlane(eff_lane, q);
#pragma unroll
            for (int h = 0; h < CPL; ++h) {
                uint32_t ord;
                if constexpr (IS_U4) ord = (acc[h][q >> 1] >> (16 * (q & 1))) & 0xffffu;
                else ord = f32_to_ord(__uint_as_float(acc[h][q]));
                if (ok[h] && q < nvalid && ord < eff) m |= 1u << (h * QB + q);
            }
        }
        // per lane: one key per set bit
        uint32_t bits = m;
        while (bits != 0u) {
            const int b = __builtin_ctz(bits);
            bits &= bits - 1u;
            const int q = b & (QB - 1), h = b / QB;
            const uint32_t lo = h == 0 ? acc[0][0] : acc[CPL - 1][0], l1 = h == 0 ? acc[0][1] : acc[CPL - 1][1];
            const uint32_t l2 = h == 0 ? acc[0][2] : acc[CPL - 1][2], l3 = h == 0 ? acc[0][3] : acc[CPL - 1][3];
            uint32_t ord;
            if constexpr (IS_U4) {
                const int pp = q >> 1;
                const uint32_t pk = pp == 0 ? lo : pp == 1 ? l1 : pp == 2 ? l2 : l3;
                ord = (pk >> (16 * (q & 1))) & 0xffffu;
            } else {
                ord = f32_to_ord(__uint_as_float(q == 0 ? lo : q == 1 ? l1 : q == 2 ? l2 : l3));
            }
            const uint64_t key = ((uint64_t)ord << 32) | (row0 + (uint32_t)(pos + h));
            if (key > sm->tau_key_blk[q]) { m &= ~(1u << b); continue; }   // ties with the k-th value beyond the k-th row
            const int slot = __hip_atomic_fetch_add(&ws->cnt[q], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            key_store(wave_buf + (size_t)q * CAP + slot, key);
            const uint32_t ref = IS_U4 ? 0u : sm->tau_ref[q];
            if (IS_U4 || (ref != TAU_REF_UNSET && ord <= ref)) {
                uint32_t bin;
                if (IS_U4) {
                    bin = ord < HIST_BINS ? ord : HIST_BINS - 1;
                } else {
                    const uint32_t below = (ref - ord) >> HIST_SHIFT;
                    bin = HIST_BINS - 1 - (below < HIST_BINS ? below : HIST_BINS - 1);
                }
                hist_count(sm, q, bin);
            }
        }
        // candidates seen per query (paces the histogram evaluations)
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            int added = __popcll(__ballot((m >> q) & 1u));
            if (CPL == 2) added += __popcll(__ballot((m >> (QB + q)) & 1u));
            appended += added;
            if (added != 0 && lane == 0)
                __hip_atomic_fetch_add(&sm->ncand_blk[q], (uint32_t)added, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    return appended;
}

// Sixteen "not below the bound" flags of sixteen queries at once.
// 8-bit sums (four per word, below 0x80) against 8-bit bounds of at most 0x7f: `comp` holds 0x80 - bound in every byte,
// so sum + comp has bit 7 set iff the sum is not below its bound, and no byte carries.  The set bits 7 of four words are
// gathered into bits 0 .. 15 by byte-wise dot products with powers of two (every byte is 0x80 or 0: 128 x the flags).
__device__ __forceinline__ uint32_t fail_flags_8bit(const uint32_t (&sums)[4], const uint32_t (&comp)[4]) {
    uint32_t lo = __builtin_amdgcn_udot4((sums[0] + comp[0]) & 0x80808080u, 0x08040201u, 0u, false);
    lo = __builtin_amdgcn_udot4((sums[1] + comp[1]) & 0x80808080u, 0x80402010u, lo, false);
    uint32_t hi = __builtin_amdgcn_udot4((sums[2] + comp[2]) & 0x80808080u, 0x08040201u, 0u, false);
    hi = __builtin_amdgcn_udot4((sums[3] + comp[3]) & 0x80808080u, 0x80402010u, hi, false);
    return (lo >> 7) | ((hi >> 7) << 8);
}
// 16-bit sums (two per word, below 0x8000) against 16-bit bounds of at most 0x8000: `comp` holds 0x8000 - bound in
// both halves; bits 15 and 31 of sum + comp are the flags.
__device__ __forceinline__ uint32_t fail_flags_16bit(const uint32_t (&sums)[8], const uint32_t (&comp)[8]) {
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t weights = (1u << (8 + 2 * w)) | (1u << (24 + 2 * w + 1));   // byte 1: query 2w, byte 3: query 2w + 1
        lo = __builtin_amdgcn_udot4((sums[w] + comp[w]) & 0x80008000u, weights, lo, false);
        hi = __builtin_amdgcn_udot4((sums[4 + w] + comp[4 + w]) & 0x80008000u, weights, hi, false);
    }
    return (lo >> 7) | ((hi >> 7) << 8);
}

// Sums of the eight 16-bit entries of one 8-byte code (words w0, w1) for 16 queries from the tables at `l16`
// (entry (byte b, table j): two 16-byte halves of 8 queries at (b * 8 + j) * 2), two queries per word of a16.
// Every lane of a wave looks up other byte values, so the lanes walk the tables in a rotated order (lane l starts
// at table l & 7; lanes 8..15 of every 16 read the halves in the other order): the 16 lanes that the LDS serves
// together then read 16 different 16-byte bank groups whatever their bytes are.  Integer adds: any order, same sums.
typedef uint32_t lds_v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void sums16_rotated(const __attribute__((address_space(3))) lds_v4u *l16, uint32_t w0, uint32_t w1,
                                               int lane, uint32_t (&a16)[8]) {
    const uint64_t w = ((uint64_t)w1 << 32) | w0;
    const uint32_t rot = (uint32_t)lane & 7u, other = ((uint32_t)lane >> 3) & 1u;
    uint32_t fa[4] = {0, 0, 0, 0}, fb[4] = {0, 0, 0, 0};   // first and second half read by this lane
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t jj = ((uint32_t)j + rot) & 7u;
        const uint32_t byte = (uint32_t)(w >> (8u * jj)) & 255u;
        const uint32_t e = (byte * 8u + jj) * 2u;
        const lds_v4u x = l16[e + other], y = l16[e + (other ^ 1u)];
        fa[0] += x.x; fa[1] += x.y; fa[2] += x.z; fa[3] += x.w;
        fb[0] += y.x; fb[1] += y.y; fb[2] += y.z; fb[3] += y.w;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a16[i] = other ? fb[i] : fa[i];
        a16[4 + i] = other ? fa[i] : fb[i];
    }
}

// Insert path of the pruned float scan.  The scan loop works on 16-bit tables
//   L[j][b] = min(4095, floor((D[j][b] - min_b D[j][b]) * scale)),
// whose sums are lower bounds (in table units, above the sum of the minima) of the float
// distances: a code whose bound reaches the threshold derived from the query's current bound
// cannot be a candidate, and almost every code is dismissed that way without a float operation
// (the lower-bound pruning of PQ Fast Scan, Section 4.2, with tables that need no grouping).
// Here the parked codes get their exact distances: the lane re-reads its codes, repeats the
// integer test against the current thresholds, and for every (code, query) that still passes adds
// the eight float entries in table order -- the order of the plain definition, Eq. (adc1) -- tests the
// result against the float bound and appends it to the wave's list of the query.
template <class SM, int NT, int E, int QB = 8>
__device__ __noinline__ int scan_flush_pruned(LDS_PTR(SM) sm, uint64_t *wave_buf, int n) {
    constexpr int CPL = 16 / NT, CAP = 64 * E;
    constexpr bool Q8 = QB == 16;   // 8-bit entries, 16 queries per slot
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    LdsWaveState *ws = &sm->ws[wave];
    const int nvalid = sm->nvalid, skip = sm->skip, ncodes = sm->ncodes;
    const uint32_t row0 = (uint32_t)sm->code_begin;
    const uint8_t *chunk_ptr = sm->chunk_ptr;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const __attribute__((address_space(3))) char *lut_bytes = (const __attribute__((address_space(3))) char *)sm->lut;
    const int ql = lane & (QB - 1);
    int appended = 0;   // keys added to the wave's lists (returned)
    for (int base = 0; base < n; base += 64) {
        // room for 64 * CPL more keys in every list
        uint32_t full = (uint32_t)__ballot(ws->cnt[ql] > CAP - 64 * CPL) & ((1u << QB) - 1u);
        while (full != 0u) {
            const int q = __builtin_ctz(full);
            full &= full - 1u;
            const int cnt = scan_compact<SM, E, false>(sm, wave_buf + (size_t)q * CAP, ws->cnt[q], q);
            if (lane == 0) ws->cnt[q] = cnt;
        }
        const bool have = base + lane < n;
        const int pos = have ? (int)sm->ring[wave][base + lane] : 0;   // position of the 16 bytes' first code
        uint4 c = make_uint4(0, 0, 0, 0);
        if (have) {
            const uint8_t *p = chunk_ptr + (size_t)(pos / CPL) * 16;
            if (pos + CPL <= ncodes) {
                c = *reinterpret_cast<const uint4 *>(p);
            } else if (CPL == 2 && pos < ncodes) {   // last lane of a ragged chunk: only its first code exists
                const uint2 half = *reinterpret_cast<const uint2 *>(p);
                c.x = half.x; c.y = half.y;
            }
        }
        const LaneWalk<NT> lw((uint32_t)(pos / CPL) & 15u);
        uint32_t acc[CPL][4];
        code_values<NT, true>(c, lw, [&](uint32_t off) {
            const v4u v = *(const __attribute__((address_space(3))) v4u *)(lut_bytes + off);
            return make_uint4(v.x, v.y, v.z, v.w);
        }, acc);
        bool ok[CPL];
#pragma unroll
        for (int h = 0; h < CPL; ++h) ok[h] = have && pos + h >= skip && pos + h < ncodes;
        // lane q: float bound of query q (ordered bits) and the same bound in table units
        uint32_t eff_lane, thr_lane;
        {
            const uint32_t shared = sm->tau_blk[ql];
            const uint32_t loose = shared == 0xffffffffu ? shared : shared + 1u;
            const uint32_t own = ws->own_ord[ql];
            eff_lane = own < loose ? own : loose;
            const float sc = sm->prune_scale[ql];
            const float t = floorf((ord_to_f32(eff_lane) - sm->prune_off[ql]) * sc) + (float)(Q8 ? PRUNE_MARGIN_Q8 : PRUNE_MARGIN);
            thr_lane = sc >= 0.f ? (uint32_t)fmaxf(fminf(t, Q8 ? 127.f : 32767.f), 0.f) : 0u;
            if constexpr (Q8) sm->eff_tmp[wave][ql] = eff_lane;   // (16 lanes write the same 16 words four times over)
        }
        // bit h * QB + q of m: the lower bound of code h does not rule out query q
        uint32_t m = 0;
        if constexpr (Q8) {
            // all 16 queries of a code at once (bounds of empty slots are 0: never below)
            const uint32_t thr_valid = ql < nvalid ? thr_lane : 0u;
            uint32_t comp[4];
#pragma unroll
            for (int p = 0; p < 4; ++p)
                comp[p] = 0x80808080u - (__builtin_amdgcn_readlane(thr_valid, 4 * p) | (__builtin_amdgcn_readlane(thr_valid, 4 * p + 1) << 8) |
                                         (__builtin_amdgcn_readlane(thr_valid, 4 * p + 2) << 16) | (__builtin_amdgcn_readlane(thr_valid, 4 * p + 3) << 24));
#pragma unroll
            for (int h = 0; h < CPL; ++h)
                if (ok[h]) m |= (~fail_flags_8bit(acc[h], comp) & 0xffffu) << (h * QB);
        } else {
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                const uint32_t thr = __builtin_amdgcn_readlane(thr_lane, q);
#pragma unroll
                for (int h = 0; h < CPL; ++h) {
                    const uint32_t lb = (acc[h][q >> 1] >> (16 * (q & 1))) & 0xffffu;
                    if (ok[h] && q < nvalid && lb < thr) m |= 1u << (h * QB + q);
                }
            }
        }
        if constexpr (Q8) {
            // Second test, 16 queries per pass only: the 8-bit bounds are coarse (64 units, entries saturating
            // at 15), so most parked codes are no candidates.  The 16-bit tables of the same queries wait in
            // LDS; the lanes that still have a bit set add up their eight entries (two 16-byte halves of 8
            // queries each) and keep the bits whose 16-bit bound is below the 16-bit threshold.
            const float sc16 = sm->prune_scale16[ql];
            const float t16 = floorf((ord_to_f32(eff_lane) - sm->prune_off[ql]) * sc16) + (float)PRUNE_MARGIN;
            const uint32_t thr16_lane = sc16 > 0.f ? (uint32_t)fmaxf(fminf(t16, 32767.f), 0.f) : 32768u;   // no scale: every sum passes
            uint32_t comp16[8];   // 0x8000 - bound of queries 2w and 2w + 1
#pragma unroll
            for (int w = 0; w < 8; ++w)
                comp16[w] = 0x80008000u - (__builtin_amdgcn_readlane(thr16_lane, 2 * w) | (__builtin_amdgcn_readlane(thr16_lane, 2 * w + 1) << 16));
            if (m != 0u) {
                const __attribute__((address_space(3))) v4u *l16 = (const __attribute__((address_space(3))) v4u *)sm->lut16;
                uint32_t m2 = 0;
#pragma unroll
                for (int h = 0; h < CPL; ++h) {
                    if (((m >> (h * QB)) & 0xffffu) == 0u) continue;
                    const uint32_t w0 = h == 0 ? c.x : c.z, w1 = h == 0 ? c.y : c.w;
                    uint32_t a16[8];
                    sums16_rotated(l16, w0, w1, lane, a16);
                    m2 |= m & ((~fail_flags_16bit(a16, comp16) & 0xffffu) << (h * QB));
                }
                m = m2;
            }
        }
        // the float bounds as scalars (a lane read inside the divergent loop below would miss
        // the lanes that have already left it)
        uint32_t eff_q[Q8 ? 1 : QB];   // (with 16 queries the bounds wait in LDS instead)
        if constexpr (!Q8) {
#pragma unroll
            for (int q = 0; q < QB; ++q) eff_q[q] = __builtin_amdgcn_readlane(eff_lane, q);
        }
        uint32_t bits = m, inserted = 0;
        while (bits != 0u) {
            const int b = __builtin_ctz(bits);
            bits &= bits - 1u;
            const int q = b & (QB - 1), h = b / QB;
            const uint32_t w0 = h == 0 ? c.x : c.z, w1 = h == 0 ? c.y : c.w;
            const float *fl = (const float *)sm->slot_lut[q];   // the query's float tables [table][entry], in device memory
            float d = fl[w0 & 255u];
            d += fl[256 + ((w0 >> 8) & 255u)];
            d += fl[512 + ((w0 >> 16) & 255u)];
            d += fl[768 + (w0 >> 24)];
            d += fl[1024 + (w1 & 255u)];
            d += fl[1280 + ((w1 >> 8) & 255u)];
            d += fl[1536 + ((w1 >> 16) & 255u)];
            d += fl[1792 + (w1 >> 24)];
            if constexpr (NT == 16) {   // one 16-byte code per lane: tables 8..15 index with c.z, c.w
                d += fl[2048 + (c.z & 255u)];
                d += fl[2304 + ((c.z >> 8) & 255u)];
                d += fl[2560 + ((c.z >> 16) & 255u)];
                d += fl[2816 + (c.z >> 24)];
                d += fl[3072 + (c.w & 255u)];
                d += fl[3328 + ((c.w >> 8) & 255u)];
                d += fl[3584 + ((c.w >> 16) & 255u)];
                d += fl[3840 + (c.w >> 24)];
            }
            const uint32_t ord = f32_to_ord(d);
            uint32_t eff;
            if constexpr (Q8) {
                eff = sm->eff_tmp[wave][q];
            } else {
                eff = eff_q[0];
#pragma unroll
                for (int i = 1; i < QB; ++i) eff = q == i ? eff_q[i] : eff;
            }
            const uint64_t key = ((uint64_t)ord << 32) | (row0 + (uint32_t)(pos + h));
            if (ord < eff && key <= sm->tau_key_blk[q]) {
                inserted |= 1u << b;
                const int slot = __hip_atomic_fetch_add(&ws->cnt[q], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                key_store(wave_buf + (size_t)q * CAP + slot, key);
                const uint32_t ref = sm->tau_ref[q];
                if (ref != TAU_REF_UNSET && ord <= ref) {
                    const uint32_t below = (ref - ord) >> HIST_SHIFT;
                    const uint32_t bin = HIST_BINS - 1 - (below < HIST_BINS ? below : HIST_BINS - 1);
                    hist_count(sm, q, bin);
                }
            }
        }
        if (__ballot(inserted != 0u) == 0ull) continue;   // (the usual case with 8-bit bounds: nothing got through)
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            int added = __popcll(__ballot((inserted >> q) & 1u));
            if (CPL == 2) added += __popcll(__ballot((inserted >> (QB + q)) & 1u));
            appended += added;
            if (added != 0 && lane == 0)
                __hip_atomic_fetch_add(&sm->ncand_blk[q], (uint32_t)added, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    return appended;
}

// Insert path of the integer scan on 8-bit lower bounds (16 queries per pass, KIND_U4Q_M16): the exact
// pair-merged 16-bit tables of the 16 queries wait in LDS beside the 8-bit ones; a parked lane adds
// up the eight exact entries of each of its codes (two 16-byte halves of 8 queries per lookup) and
// appends the sums below a query's bound to the wave's list of that query.  Sums are exact integers.
template <class SM, int E>
__device__ __noinline__ int scan_flush_u4q(LDS_PTR(SM) sm, uint64_t *wave_buf, int n) {
    constexpr int QB = 16, CPL = 2, CAP = 64 * E;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    LdsWaveState *ws = &sm->ws[wave];
    const int nvalid = sm->nvalid, skip = sm->skip, ncodes = sm->ncodes;
    const uint32_t row0 = (uint32_t)sm->code_begin;
    const uint8_t *chunk_ptr = sm->chunk_ptr;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const __attribute__((address_space(3))) v4u *l16 = (const __attribute__((address_space(3))) v4u *)sm->lut16;
    const int ql = lane & (QB - 1);
    int appended = 0;   // keys added to the wave's lists (returned)
    for (int base = 0; base < n; base += 64) {
        // room for 64 * CPL more keys in every list
        uint32_t full = (uint32_t)__ballot(ws->cnt[ql] > CAP - 64 * CPL) & ((1u << QB) - 1u);
        while (full != 0u) {
            const int q = __builtin_ctz(full);
            full &= full - 1u;
            const int cnt = scan_compact<SM, E, true>(sm, wave_buf + (size_t)q * CAP, ws->cnt[q], q);
            if (lane == 0) ws->cnt[q] = cnt;
        }
        const bool have = base + lane < n;
        const int pos = have ? (int)sm->ring[wave][base + lane] : 0;   // position of the 16 bytes' first code
        uint4 c = make_uint4(0, 0, 0, 0);
        if (have) {
            const uint8_t *p = chunk_ptr + (size_t)(pos / CPL) * 16;
            if (pos + CPL <= ncodes) {
                c = *reinterpret_cast<const uint4 *>(p);
            } else if (pos < ncodes) {   // last lane of a ragged chunk: only its first code exists
                const uint2 half = *reinterpret_cast<const uint2 *>(p);
                c.x = half.x; c.y = half.y;
            }
        }
        // exact sums of the lane's two codes for the 16 queries, two per word
        uint32_t acc[CPL][8];
#pragma unroll
        for (int h = 0; h < CPL; ++h) {
            const uint32_t w0 = h == 0 ? c.x : c.z, w1 = h == 0 ? c.y : c.w;
            sums16_rotated(l16, w0, w1, lane, acc[h]);
        }
        bool ok[CPL];
#pragma unroll
        for (int h = 0; h < CPL; ++h) ok[h] = have && pos + h >= skip && pos + h < ncodes;
        // candidates satisfy sum < eff: the wave's own bound is strict, the block's is "<="
        uint32_t eff_lane;
        {
            const uint32_t shared = sm->tau_blk[ql];
            const uint32_t loose = shared == 0xffffffffu ? shared : shared + 1u;
            const uint32_t own = ws->own_ord[ql];
            eff_lane = own < loose ? own : loose;
        }
        // bit h * QB + q of m: code h of this lane qualifies for query q (all 16 queries of a code at once; the bounds
        // are at most 0x7fff, those of empty slots 0: never below)
        uint32_t m = 0;
        {
            const uint32_t eff_valid = ql < nvalid ? eff_lane : 0u;
            uint32_t comp16[8];
#pragma unroll
            for (int w = 0; w < 8; ++w)
                comp16[w] = 0x80008000u - (__builtin_amdgcn_readlane(eff_valid, 2 * w) | (__builtin_amdgcn_readlane(eff_valid, 2 * w + 1) << 16));
#pragma unroll
            for (int h = 0; h < CPL; ++h)
                if (ok[h]) m |= (~fail_flags_16bit(acc[h], comp16) & 0xffffu) << (h * QB);
        }
        if (__ballot(m != 0u) == 0ull) continue;
        uint32_t bits = m;
        while (bits != 0u) {
            const int b = __builtin_ctz(bits);
            bits &= bits - 1u;
            const int q = b & (QB - 1), h = b / QB, pp = q >> 1;
            uint32_t pk = h == 0 ? acc[0][0] : acc[1][0];
#pragma unroll
            for (int i = 1; i < 8; ++i) pk = pp == i ? (h == 0 ? acc[0][i] : acc[1][i]) : pk;
            const uint32_t ord = (pk >> (16 * (q & 1))) & 0xffffu;
            const uint64_t key = ((uint64_t)ord << 32) | (row0 + (uint32_t)(pos + h));
            if (key > sm->tau_key_blk[q]) { m &= ~(1u << b); continue; }   // ties with the k-th value beyond the k-th row
            const int slot = __hip_atomic_fetch_add(&ws->cnt[q], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            key_store(wave_buf + (size_t)q * CAP + slot, key);
            hist_count(sm, q, ord < HIST_BINS ? ord : HIST_BINS - 1);
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int added = __popcll(__ballot((m >> q) & 1u)) + __popcll(__ballot((m >> (QB + q)) & 1u));
            appended += added;
            if (added != 0 && lane == 0)
                __hip_atomic_fetch_add(&sm->ncand_blk[q], (uint32_t)added, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    return appended;
}

// Periodic path (one wave per query and period): pick up the best bound published for query q
// by any block and, if enough candidates arrived since the histogram was last evaluated and no
// other wave is already doing it, recompute the bound from the histogram.
constexpr uint32_t REFRESH_MIN_NEW = 16;

template <class SM, bool IS_U4>
__device__ __noinline__ void scan_refresh(LDS_PTR(SM) sm, int q) {
    // the four device words of the query are independent of one another: one round trip
    const unsigned long long gk = __hip_atomic_load(sm->tau_key_global[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t g = (uint32_t)(gk >> 32);
    // (the block's own count of new candidates goes into the device counter on this occasion)
    // The block's histogram window goes to device memory once it holds a worthwhile share of a result list (a
    // quarter, 16 .. 256 keys): moving it costs up to HWIN device-scope atomic adds on this wave's path.
    uint32_t n_v = 0, flush_v = 0;
    if (lane_id() == 0) {
        const uint32_t mine = __hip_atomic_exchange(&sm->ncand_blk[q], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        n_v = __hip_atomic_fetch_add(sm->ncand[q], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
        const uint32_t pending = __hip_atomic_fetch_add(&sm->hwin_pending[q], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) + mine;
        const uint32_t quarter = (uint32_t)sm->topk / 4u;
        if (pending >= (quarter < 16u ? 16u : quarter > 256u ? 256u : quarter)) {
            sm->hwin_pending[q] = 0u;
            flush_v = 1u;
        }
    }
    if (__builtin_amdgcn_readfirstlane(flush_v) != 0u) hist_window_flush(sm, q);
    const uint32_t mark_v = __hip_atomic_load(sm->refresh_mark[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t ref_v = IS_U4 ? 0u : __hip_atomic_load(sm->tau_ref_global[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane_id() == 0) {
        __hip_atomic_fetch_min(&sm->tau_blk[q], g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __hip_atomic_fetch_min(&sm->tau_key_blk[q], gk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    uint32_t ref = 0;
    if (!IS_U4) {
        ref = __builtin_amdgcn_readfirstlane(sm->tau_ref[q]);
        if (ref == TAU_REF_UNSET) {
            ref = __builtin_amdgcn_readfirstlane(ref_v);
            if (ref == TAU_REF_UNSET) return;
            if (lane_id() == 0) sm->tau_ref[q] = ref;
        }
    }
    const uint32_t n = __builtin_amdgcn_readfirstlane(n_v);
    const uint32_t mark = __builtin_amdgcn_readfirstlane(mark_v);
    if (n - mark < REFRESH_MIN_NEW) return;
    uint32_t won = 0;
    if (lane_id() == 0) {
        uint32_t expected = mark;
        won = __hip_atomic_compare_exchange_strong(sm->refresh_mark[q], &expected, n, __ATOMIC_RELAXED,
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ? 1u : 0u;
    }
    if (__builtin_amdgcn_readfirstlane(won) == 0u) return;
    const int bin = hist_threshold(sm->hist[q], sm->topk);
    if (bin < HIST_BINS) {
        // every value counted in bins <= bin is at or below this edge
        const uint32_t edge = IS_U4 ? (uint32_t)bin : ref - ((uint32_t)(HIST_BINS - 1 - bin) << HIST_SHIFT);
        if (lane_id() == 0) publish_bound(sm, q, edge);
    }
}

// End of item, per wave: leave at most k keys in the lists of the queries in qmask.
template <class SM, int QB, int E>
__device__ __noinline__ void scan_finish_wave(LDS_PTR(SM) sm, uint64_t *wave_buf, uint32_t qmask) {
    constexpr int CAP = 64 * E;
    LdsWaveState *ws = &sm->ws[threadIdx.x >> 6];
    for (int q = 0; q < QB; ++q) {
        int cnt = ws->cnt[q];
        if (((qmask >> q) & 1u) != 0u && cnt > sm->topk) {
            wave_compact<E>(wave_buf + (size_t)q * CAP, cnt, sm->topk);
            if (lane_id() == 0) ws->cnt[q] = cnt;
        }
    }
}

// End of item, per wave: the keys of the wave's lists that are within the block's bound of their
// query go straight to the item's result list of that query (position from a counter in LDS).
// Keys above the bound cannot be among the k smallest.  If more than KPAD keys arrive for a query
// the surplus is dropped here and the query is merged from the lists instead (scan_merge_item).
template <class SM, int QB, int E, int KPAD>
__device__ __noinline__ void scan_emit_wave(LDS_PTR(SM) sm, uint64_t *wave_buf) {
    constexpr int CAP = 64 * E;
    const int lane = lane_id();
    LdsWaveState *ws = &sm->ws[threadIdx.x >> 6];
    list_fence();
    // lane q: the bound of query q, the better of the block's and the device's current one
    const int ql = lane & (QB - 1);
    const unsigned long long dev_key = __hip_atomic_load(sm->tau_key_global[ql], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long blk_key = sm->tau_key_blk[ql];
    const unsigned long long key_lane = dev_key < blk_key ? dev_key : blk_key;
    const uint32_t blk_bound = sm->tau_blk[ql];
    const uint32_t bound_lane = (uint32_t)(key_lane >> 32) < blk_bound ? (uint32_t)(key_lane >> 32) : blk_bound;
    for (int q = 0; q < sm->nvalid && q < QB; ++q) {
        const int cnt = ws->cnt[q];
        if (cnt == 0) continue;
        const uint32_t bound = __builtin_amdgcn_readlane(bound_lane, q);
        const uint64_t key_bound = ((uint64_t)__builtin_amdgcn_readlane((uint32_t)(key_lane >> 32), q) << 32) |
                                   __builtin_amdgcn_readlane((uint32_t)key_lane, q);
        uint64_t *out = sm->slot_out[q];
        const uint64_t *buf = wave_buf + (size_t)q * CAP;
        for (int i0 = 0; i0 < cnt; i0 += 64) {
            const uint64_t key = i0 + lane < cnt ? key_load(buf + i0 + lane) : KEY_EMPTY;
            const bool pass = key != KEY_EMPTY && (uint32_t)(key >> 32) <= bound && key <= key_bound;
            const uint64_t mask = __ballot(pass);
            if (mask == 0ull) continue;
            int at = 0;
            if (lane == 0) at = __hip_atomic_fetch_add(&sm->out_cnt[q], __popcll(mask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            at = __builtin_amdgcn_readfirstlane(at) + (int)mask_prefix(mask);
            if (pass && at < KPAD) out[at] = key;
        }
    }
}

// End of item, whole block, for a query whose result list overflowed but whose keys within the
// bound fit into the memory of the tables (idle once every wave has left the scan; the next item
// stages them anew): gather them there, sort them with the whole block, write the KPAD smallest
// and share the k-th as a bound.  Every thread of the block must call it.
template <class SM, int QB, int E, int KPAD>
__device__ __noinline__ void scan_overflow_sort(LDS_PTR(SM) sm, uint64_t *wave_buf, int q) {
    constexpr int CAP = 64 * E;
    const int lane = lane_id();
    LdsWaveState *ws = &sm->ws[threadIdx.x >> 6];
    uint64_t *keys = (uint64_t *)&sm->lut[0];   // generic pointer into LDS (lut16 follows lut without a gap)
    if (threadIdx.x == 0) sm->out_cnt[q] = 0;
    __syncthreads();
    const unsigned long long dev_key = __hip_atomic_load(sm->tau_key_global[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long blk_key = sm->tau_key_blk[q];
    const uint64_t key_bound = dev_key < blk_key ? dev_key : blk_key;       // never above the bounds of the first pass
    const uint32_t blk_bound = sm->tau_blk[q];
    const uint32_t bound = (uint32_t)(key_bound >> 32) < blk_bound ? (uint32_t)(key_bound >> 32) : blk_bound;
    const int cnt = ws->cnt[q];
    const uint64_t *buf = wave_buf + (size_t)q * CAP;
    for (int i0 = 0; i0 < cnt; i0 += 64) {
        const uint64_t key = i0 + lane < cnt ? key_load(buf + i0 + lane) : KEY_EMPTY;
        const bool pass = key != KEY_EMPTY && (uint32_t)(key >> 32) <= bound && key <= key_bound;
        const uint64_t mask = __ballot(pass);
        if (mask == 0ull) continue;
        int at = 0;
        if (lane == 0) at = __hip_atomic_fetch_add(&sm->out_cnt[q], __popcll(mask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        at = __builtin_amdgcn_readfirstlane(at) + (int)mask_prefix(mask);
        if (pass) keys[at] = key;
    }
    __syncthreads();
    const int total = sm->out_cnt[q];
    int n2 = 64;
    while (n2 < total) n2 <<= 1;
    for (int i = total + threadIdx.x; i < n2; i += TUNED_THREADS) keys[i] = KEY_EMPTY;
    block_bitonic_sort(keys, n2);
    uint64_t *out = sm->slot_out[q];
    for (int i = threadIdx.x; i < KPAD; i += TUNED_THREADS) out[i] = i < n2 ? keys[i] : KEY_EMPTY;
    // the k-th smallest key of the item bounds the k-th smallest of the whole scan
    if (threadIdx.x == 0 && total >= sm->topk) publish_key_bound(sm, q, keys[sm->topk - 1]);
    __syncthreads();
}

// End of item, wave q < QB: fold the lists of all waves for query q into the list of wave 0
// and write KPAD keys (padded with KEY_EMPTY) to out.
template <class SM, int QB, int E, int KPAD>
__device__ __noinline__ void scan_merge_item(LDS_PTR(SM) sm, uint64_t *block_scratch, uint64_t *out) {
    constexpr int CAP = 64 * E;
    const int q = threadIdx.x >> 6, lane = lane_id();
    const int k = sm->topk;
    uint64_t *acc = block_scratch + (size_t)q * CAP;   // list of wave 0
    int cnt = sm->ws[0].cnt[q];
    uint64_t kth = KEY_EMPTY;
    for (int w = 1; w < TUNED_WAVES; ++w) {
        const uint64_t *src = block_scratch + (size_t)(w * QB + q) * CAP;
        const int cw = sm->ws[w].cnt[q];
        if (cw == 0) continue;
        for (int i = lane; i < cw; i += 64) key_store(acc + cnt + i, key_load(src + i));
        cnt += cw;
        if (cnt > k) kth = wave_compact<E>(acc, cnt, k);
    }
    if (kth != KEY_EMPTY && lane == 0) publish_key_bound(sm, q, kth);
    if (cnt > 0) list_fence();
    for (int i = lane; i < KPAD; i += 64) out[i] = i < cnt ? key_load(acc + i) : KEY_EMPTY;
}

// Optional instrumentation (-DPQ_SCAN_TIMING, measurement builds only): wall-clock cycles of every wave per
// phase, added up in stats[1 + phase] when the wave leaves the kernel.
#ifdef PQ_SCAN_TIMING
#define PQ_TICK(phase) do { const unsigned long long now__ = __builtin_amdgcn_s_memtime(); tick_acc[phase] += now__ - tick_last; tick_last = now__; } while (0)
#else
#define PQ_TICK(phase) do { } while (0)
#endif
enum { TICK_SETUP = 0, TICK_LOOP, TICK_FLUSH, TICK_REFRESH, TICK_EMIT, TICK_OVERFLOW, TICK_COUNT };

template <int KIND, int E, int KPAD, int DEPTH>
__global__ __launch_bounds__(TUNED_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4)))
void scan_tuned_kernel(TunedArgs a) {
    constexpr bool IS_U4 = KIND == KIND_U4_M16 || KIND == KIND_U4Q_M16;   // values are integer sums
    constexpr bool U4Q = KIND == KIND_U4Q_M16;            // integer sums, scan loop on 8-bit lower bounds, 16 queries
    constexpr bool Q8 = KIND == KIND_F32Q_M8 || U4Q;      // scan loop on 8-bit lower bounds, 16 queries per pass
    constexpr bool PRUNED = KIND == KIND_F32P_M8 || KIND == KIND_F32P_M16 || KIND == KIND_F32Q_M8;   // float values, scan loop on integer lower bounds
    constexpr bool PACKED = IS_U4 || PRUNED;              // scan loop adds packed entries (16-bit: 8 queries, 8-bit: 16)
    constexpr int QB = Q8 ? 16 : PACKED ? 8 : 4;
    constexpr int NT = KIND == KIND_F32_M16 || KIND == KIND_F32P_M16 ? 16 : 8;   // tables = lookups per code
    constexpr int CB = NT;                                // code bytes (8 or 16)
    constexpr int CPL = 16 / CB;                          // codes per lane per 16-byte load
    constexpr int SUB = 64 * CPL;                         // codes per wave sub-tile (one load per lane)
    // DEPTH = sub-tiles a wave has in registers or on their way: 2 when the codes are shared by many
    // blocks through L2 (flat scan of many query groups), 8 when every block streams its own codes
    // from HBM (few groups, inverted lists).  A wave works through groups of DEPTH sub-tiles.
    constexpr int CAP = 64 * E;
    typedef typename std::conditional<IS_U4, U32Val, F32Val>::type V;
    // ring: two tiles fit behind a ring that was not flushed
    typedef TunedSmemT<RING_FLUSH + 64 * DEPTH, Q8> SM;   // a group of sub-tiles fits behind a ring that was not flushed
    static_assert(TUNED_WAVES != 8 || sizeof(SM) <= 80 * 1024, "two blocks of 8 waves share the 160 KB of a CU");
    __shared__ SM sm;
    LDS_PTR(SM) smp = (LDS_PTR(SM))&sm;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keep it scalar
    const int lane = lane_id();
    const LaneWalk<NT> lw((uint32_t)lane & 15u);
    const char *lut_bytes = reinterpret_cast<const char *>(sm.lut);
    uint64_t *block_scratch = a.scratch + (size_t)blockIdx.x * TUNED_WAVES * QB * CAP;
    uint64_t *wave_buf = block_scratch + (size_t)wave * QB * CAP;

    const int nitems = a.item_tab ? (int)*a.nitems_dev : a.nitems;
    int gstep = 0;   // steps of this wave over all its items: paces the periodic bound refresh
    unsigned long long parked_total = 0;   // positions this wave has handed to the insert path (uniform; reported when profiling)
    if (threadIdx.x == 0) sm.stat_parked = 0ull;
#ifdef PQ_SCAN_TIMING
    unsigned long long tick_acc[TICK_COUNT] = {0, 0, 0, 0, 0, 0}, tick_last = __builtin_amdgcn_s_memtime();
#endif
    for (;;) {
        if (threadIdx.x == 0) sm.item = (int)atomicAdd(a.work_counter, 1u);
        __syncthreads();
        const int item = sm.item;
        if (item >= nitems) {
            if (a.stats != nullptr) {   // one device atomic per block: thousands of waves adding to one word would serialise
                if (lane == 0 && parked_total != 0ull)
                    __hip_atomic_fetch_add(&sm.stat_parked, parked_total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __syncthreads();
                if (threadIdx.x == 0 && sm.stat_parked != 0ull) atomicAdd(a.stats, sm.stat_parked);
            }
#ifdef PQ_SCAN_TIMING
            if (a.stats != nullptr && lane == 0)
                for (int i = 0; i < TICK_COUNT; ++i) atomicAdd(a.stats + 1 + i, tick_acc[i]);
#endif
            break;
        }

        // ---- describe the item: rows to scan, and for every slot the query whose tables it holds ----
        if (threadIdx.x < QB) {
            const int s = threadIdx.x;
            int qid = -1;                  // index of the query's threshold state, -1: empty slot
            const void *lut = nullptr;
            uint64_t *out = nullptr;
            if (a.item_tab) {
                const IvfItem it = a.item_tab[item];
                const int nslots = (it.skip_slots_chunk >> 8) & 0xff;
                if (s < nslots) {
                    const int pair = a.pairs_by_list[it.pair_pos + s];
                    qid = pair / a.nprobe;
                    lut = (const float *)a.luts + (size_t)pair * (NT * 256);
                    out = a.partial + ((size_t)a.pair_out[pair] + (it.skip_slots_chunk >> 16)) * KPAD;
                    if constexpr (PRUNED) {
                        sm.prune_off[s] = a.prune_off[pair];
                        sm.prune_scale[s] = a.prune_scale[pair];
                        const float4 *pm = reinterpret_cast<const float4 *>(a.pair_min + (size_t)pair * NT);
#pragma unroll
                        for (int i = 0; i < NT / 4; ++i) *reinterpret_cast<float4 *>(&sm.pmin[s][4 * i]) = pm[i];
                    }
                } else if constexpr (PRUNED) {
                    sm.prune_off[s] = 0.f; sm.prune_scale[s] = -1.f;
                }
                if (s == 0) {
                    sm.code_begin = it.code_begin;
                    sm.chunk_ptr = a.codes + (size_t)it.code_begin * CB;   // (64-bit: rows beyond 2^32 / CB bytes)
                    sm.ncodes = (int)it.ncodes;
                    sm.skip = it.skip_slots_chunk & 0xff;
                    sm.nvalid = nslots;
                }
            } else {
                const int group = item % a.ngroups, chunk = item / a.ngroups;
                const int gq = group * QB + s;
                if (gq < a.nq) {
                    qid = gq;
                    lut = IS_U4 ? (const void *)((const uint8_t *)a.luts + (size_t)gq * 256)
                                : (const void *)((const float *)a.luts + (size_t)gq * (NT * 256));
                    if constexpr (PRUNED) { sm.prune_off[s] = a.prune_off[gq]; sm.prune_scale[s] = a.prune_scale[gq]; }
                    if constexpr (Q8 && PRUNED) sm.prune_scale16[s] = a.prune_scale16[gq];
                } else if constexpr (PRUNED) {
                    sm.prune_off[s] = 0.f; sm.prune_scale[s] = 0.f;
                    if constexpr (Q8 && PRUNED) sm.prune_scale16[s] = 0.f;
                }
                out = a.partial + ((size_t)item * QB + s) * KPAD;
                if (s == 0) {
                    const bool head = chunk < a.head_chunks;
                    const int64_t cbeg = head ? (int64_t)chunk * a.head_codes
                                              : (int64_t)a.head_chunks * a.head_codes + (int64_t)(chunk - a.head_chunks) * a.chunk_codes;
                    const int64_t clen = head ? a.head_codes : a.chunk_codes;
                    const int64_t cend = cbeg + clen < a.n ? cbeg + clen : a.n;
                    sm.code_begin = cbeg;
                    sm.chunk_ptr = a.codes + cbeg * CB;
                    sm.ncodes = cend > cbeg ? (int)(cend - cbeg) : 0;
                    sm.skip = 0;
                    sm.group = group;
                    sm.nvalid = a.nq - group * QB < QB ? a.nq - group * QB : QB;
                }
            }
            const int sq = qid < 0 ? 0 : qid;
            sm.slot_lut[s] = lut;
            sm.slot_out[s] = out;
            sm.hist[s] = a.hist + (size_t)sq * HIST_BINS;
            sm.ncand[s] = a.ncand + sq;
            sm.refresh_mark[s] = a.refresh_mark + sq;
            sm.tau_key_global[s] = a.tau_key + sq;
            const unsigned long long start_key = qid < 0 ? 0ull : __hip_atomic_load(&a.tau_key[sq], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sm.tau_key_blk[s] = start_key;
            sm.tau_ref_global[s] = a.tau_ref + sq;
            sm.tau_blk[s] = (uint32_t)(start_key >> 32);
            sm.tau_ref[s] = __hip_atomic_load(&a.tau_ref[sq], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (s == 0) sm.topk = a.topk;
        }
        if (lane < QB) { sm.ws[wave].cnt[lane] = 0; sm.ws[wave].own_ord[lane] = V::ord_inf(); }
        if (threadIdx.x < 16) { sm.out_cnt[threadIdx.x] = 0; sm.ncand_blk[threadIdx.x] = 0; sm.hwin_pending[threadIdx.x] = 0; }
        if (threadIdx.x == 0) sm.next_group = 2 * TUNED_WAVES;
        __syncthreads();

        // ---- stage the tables of the slots' queries -----------------------------------------------
        if constexpr (PRUNED) {
            if (a.item_tab) {
                // inverted lists: every slot has the float tables of its own (query, list) pair; the
                // 16-bit entries min(ENTRY_MAX, floor((D - min of the table) * scale of the pair)) are
                // formed here (same arithmetic as prune_tables_kernel)
                constexpr float ENTRY_MAX = (float)(32767 / NT);
                for (int e = threadIdx.x; e < NT * 256; e += TUNED_THREADS) {
                    const int j = e >> 8, byte = e & 255;
                    uint32_t v[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const float *lut = (const float *)sm.slot_lut[q];
                        const float sc = sm.prune_scale[q];
                        v[q] = 0u;
                        if (lut != nullptr && sc > 0.f) v[q] = (uint32_t)fminf(floorf((lut[e] - sm.pmin[q][j]) * sc), ENTRY_MAX);
                    }
                    const uint4 pk = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
                    if (NT == 8) { sm.lut[byte * 16 + 2 * j] = pk; sm.lut[byte * 16 + 2 * j + 1] = pk; }
                    else sm.lut[byte * 16 + j] = pk;
                }
            } else {
                // 16-bit tables of the group, prepared in slot order: [group][byte][table] x 8 queries
                const uint4 *qt = a.qtabs + (size_t)sm.group * (256 * NT);
                for (int e = threadIdx.x; e < 256 * NT; e += TUNED_THREADS) {
                    const uint4 pk = qt[e];
                    if constexpr (NT == 8) {
                        sm.lut[(e >> 3) * 16 + 2 * (e & 7) + ((e >> 3) & 1)] = pk;   // (the first copies of two neighbouring byte values go to the even and to the odd slot of the
                                                                                       // table: the 16 lanes the LDS serves together write 16 different bank groups)
                        sm.lut[(e >> 3) * 16 + 2 * (e & 7) + 1 - ((e >> 3) & 1)] = pk;
                    } else {
                        sm.lut[e] = pk;   // (e >> 4) * 16 + (e & 15)
                    }
                }
                if constexpr (Q8) {   // the 16-bit tables of the second test, as prepared
                    const uint4 *qt16 = a.qtabs16 + (size_t)sm.group * 4096;
                    for (int e = threadIdx.x; e < 4096; e += TUNED_THREADS) sm.lut16[e] = qt16[e];
                }
            }
        } else if constexpr (U4Q) {
            // Integer scan on 8-bit lower bounds.  (1) the 16 queries' 8-bit tables of 16 entries; (2) the exact
            // pair-merged tables T[r][byte] = Q[2r][byte & 15] + Q[2r+1][byte >> 4] as 16-bit entries into
            // lut16; (3) their minima (from the 8-bit tables), the sum of the minima and, from the bound the item starts with, the
            // scale of the lower bounds; (4) L[r][byte] = min(15, floor((T - min_r) * scale)) into lut.
            for (int e = threadIdx.x; e < QB * 256; e += TUNED_THREADS) {
                const int q = e >> 8;
                const uint8_t *ql = (const uint8_t *)sm.slot_lut[q];
                sm.qstage[q][e & 255] = ql ? ql[e & 255] : 0;
            }
            __syncthreads();
            for (int e = threadIdx.x; e < 8 * 256; e += TUNED_THREADS) {
                const int r = e & 7, byte = e >> 3;   // (table fastest: a wave's LDS accesses spread over the bank groups)
                uint32_t t[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    t[q] = sm.slot_lut[q] ? (uint32_t)sm.qstage[q][(2 * r) * 16 + (byte & 15)] +
                                                (uint32_t)sm.qstage[q][(2 * r + 1) * 16 + (byte >> 4)]
                                          : 0x0fffu;
                }
                sm.lut16[(byte * 8 + r) * 2] = make_uint4(t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16));
                sm.lut16[(byte * 8 + r) * 2 + 1] = make_uint4(t[8] | (t[9] << 16), t[10] | (t[11] << 16), t[12] | (t[13] << 16), t[14] | (t[15] << 16));
            }
            if (threadIdx.x < 128) {   // minima of the merged tables: the two components of a byte vary independently
                const int q = threadIdx.x >> 3, r = threadIdx.x & 7;
                uint32_t lo = 255u, hi = 255u;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t x = sm.qstage[q][(2 * r) * 16 + i], y = sm.qstage[q][(2 * r + 1) * 16 + i];
                    lo = x < lo ? x : lo;
                    hi = y < hi ? y : hi;
                }
                sm.umin[q][r] = sm.slot_lut[q] ? lo + hi : 0x0fffu;
            }
            __syncthreads();
            if (threadIdx.x < 16) {
                const int q = threadIdx.x;
                uint32_t off = 0;
#pragma unroll
                for (int r = 0; r < 8; ++r) off += sm.umin[q][r];
                // sums at or below the bound the item starts with are what must get through
                const uint32_t bound = sm.tau_blk[q];
                float scale = 0.f;   // no bound yet: every entry 0, every sum passes
                if (sm.slot_lut[q] != nullptr && bound < 0x7fffu && bound >= off) scale = PRUNE_RANGE_U4Q / (float)(bound - off + 1u);
                sm.prune_off[q] = (float)off;
                sm.prune_scale[q] = scale;
            }
            __syncthreads();
            for (int e = threadIdx.x; e < 8 * 256; e += TUNED_THREADS) {
                const int r = e & 7, byte = e >> 3;   // (table fastest: a wave's LDS accesses spread over the bank groups)
                const uint4 lo = sm.lut16[(byte * 8 + r) * 2], hi = sm.lut16[(byte * 8 + r) * 2 + 1];
                const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                uint32_t l[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const uint32_t t = (w[q >> 1] >> (16 * (q & 1))) & 0xffffu;
                    const float x = (float)(t - sm.umin[q][r]) * sm.prune_scale[q];
                    l[q] = sm.slot_lut[q] ? (uint32_t)fminf(floorf(x), PRUNE_ENTRY_MAX_Q8) : (uint32_t)PRUNE_ENTRY_MAX_Q8;
                }
                const uint4 pk = make_uint4(l[0] | (l[1] << 8) | (l[2] << 16) | (l[3] << 24), l[4] | (l[5] << 8) | (l[6] << 16) | (l[7] << 24),
                                            l[8] | (l[9] << 8) | (l[10] << 16) | (l[11] << 24), l[12] | (l[13] << 8) | (l[14] << 16) | (l[15] << 24));
                sm.lut[byte * 16 + 2 * r + (byte & 1)] = pk;
                sm.lut[byte * 16 + 2 * r + 1 - (byte & 1)] = pk;
            }
        } else if constexpr (!IS_U4) {
            // (byte values fastest: the tables come from device memory, often for the only time, and the loads of a wave
            // are contiguous that way; the price is that its 64 lanes write the same LDS bank group)
            for (int e = threadIdx.x; e < NT * 256; e += TUNED_THREADS) {
                const int j = e >> 8, byte = e & 255;
                float v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float *lut = (const float *)sm.slot_lut[q];
                    v[q] = lut ? lut[e] : __builtin_inff();   // empty slots never qualify
                }
                const uint4 pk = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]),
                                            __float_as_uint(v[3]));
                if (NT == 8) { sm.lut[byte * 16 + 2 * j] = pk; sm.lut[byte * 16 + 2 * j + 1] = pk; }
                else sm.lut[byte * 16 + j] = pk;
            }
        } else {
            for (int e = threadIdx.x; e < QB * 256; e += TUNED_THREADS) {
                const int q = e >> 8;
                const uint8_t *ql = (const uint8_t *)sm.slot_lut[q];
                sm.qstage[q][e & 255] = ql ? ql[e & 255] : 0;
            }
            __syncthreads();
            // pair-merged tables: T[r][byte] = Q[2r][byte & 15] + Q[2r+1][byte >> 4]
            for (int e = threadIdx.x; e < 8 * 256; e += TUNED_THREADS) {
                const int r = e & 7, byte = e >> 3;   // (table fastest: a wave's LDS accesses spread over the bank groups)
                uint32_t s[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    s[q] = sm.slot_lut[q] ? (uint32_t)sm.qstage[q][(2 * r) * 16 + (byte & 15)] +
                                                (uint32_t)sm.qstage[q][(2 * r + 1) * 16 + (byte >> 4)]
                                          : 0x0fffu;   // empty slots never qualify
                }
                const uint4 pk = make_uint4(s[0] | (s[1] << 16), s[2] | (s[3] << 16), s[4] | (s[5] << 16),
                                            s[6] | (s[7] << 16));
                sm.lut[byte * 16 + 2 * r + (byte & 1)] = pk;
                sm.lut[byte * 16 + 2 * r + 1 - (byte & 1)] = pk;
            }
        }
        __syncthreads();
        // the staging memory now serves as the histogram windows of the slots' queries: HWIN bins up to the bin
        // of the bound the item starts with
        for (int i = threadIdx.x; i < QB * HWIN; i += TUNED_THREADS) hist_window(smp, 0)[i] = 0u;
        if (threadIdx.x < QB) {
            const uint32_t bound = sm.tau_blk[threadIdx.x];
            uint32_t top = HIST_BINS - 1;
            if constexpr (IS_U4) {
                top = bound < (uint32_t)HIST_BINS ? bound : HIST_BINS - 1;
            } else {
                const uint32_t ref = sm.tau_ref[threadIdx.x];
                if (ref != TAU_REF_UNSET && bound <= ref) {
                    const uint32_t below = (ref - bound) >> HIST_SHIFT;
                    top = HIST_BINS - 1 - (below < (uint32_t)HIST_BINS ? below : HIST_BINS - 1);
                }
            }
            sm.hwin_base[threadIdx.x] = top >= (uint32_t)(HWIN - 1) ? top - (HWIN - 1) : 0u;
        }
        __syncthreads();

        PQ_TICK(TICK_SETUP);
        const int nvalid_q = sm.nvalid;
        int ring_cnt = 0;                  // positions parked in this wave's ring (uniform)
        // Thresholds in registers: a code is a candidate for query q if value < tau[q].
        // Float: the four thresholds as float bits; integer: the eight as four packed pairs.
        uint32_t tau[4];
        auto reload_tau = [&]() {
            // lane q works out the bound of query q (own bound strict, the block's bound "<="),
            // lane reads hand the values to the whole wave as scalars
            const int ql = lane & (QB - 1);
            const uint32_t shared = sm.tau_blk[ql];
            const uint32_t loose = shared == 0xffffffffu ? shared : shared + 1u;
            const uint32_t own = sm.ws[wave].own_ord[ql];
            uint32_t eff = own < loose ? own : loose;
            if constexpr (U4Q) {
                // sums below eff qualify, i.e. sums of at most eff - 1: that bound in units of the 8-bit tables,
                // rounded down, plus the slack for the fp32 conversion
                const float t = floorf(((float)eff - 1.f - sm.prune_off[ql]) * sm.prune_scale[ql]) + (float)PRUNE_MARGIN_Q8;
                eff = ql < nvalid_q && eff != 0u ? (uint32_t)fmaxf(fminf(t, 127.f), 0.f) : 0u;
            } else if constexpr (IS_U4) {
                eff = ql < nvalid_q ? eff : 0u;
            } else if constexpr (PRUNED) {
                // the bound in table units, rounded down, plus the slack that covers the rounding of
                // the tables and of this conversion; no bound (or no scale) admits every sum
                const float sc = sm.prune_scale[ql];
                const float t = floorf((ord_to_f32(eff) - sm.prune_off[ql]) * sc) + (float)(Q8 ? PRUNE_MARGIN_Q8 : PRUNE_MARGIN);
                eff = ql < nvalid_q && sc >= 0.f ? (uint32_t)fmaxf(fminf(t, Q8 ? 127.f : 32767.f), 0.f) : 0u;
            } else {
                eff = __float_as_uint(ord_to_f32(eff));
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if constexpr (Q8)   // 0x80 minus the threshold in every byte (thresholds are at most 127): see the test
                    tau[p] = 0x80808080u - (__builtin_amdgcn_readlane(eff, 4 * p) | (__builtin_amdgcn_readlane(eff, 4 * p + 1) << 8) |
                                            (__builtin_amdgcn_readlane(eff, 4 * p + 2) << 16) | (__builtin_amdgcn_readlane(eff, 4 * p + 3) << 24));
                else if constexpr (PACKED)
                    tau[p] = __builtin_amdgcn_readlane(eff, 2 * p) | (__builtin_amdgcn_readlane(eff, 2 * p + 1) << 16);
                else
                    tau[p] = __builtin_amdgcn_readlane(eff, p);
            }
        };
        reload_tau();

        const int ncodes = sm.ncodes;                                      // rows of this item (below 2^31)
        const int nsub = (ncodes + SUB - 1) / SUB;                         // sub-tiles, the last may be ragged
        const int nfull = ncodes / SUB;                                    // sub-tiles with every code present
        const uint8_t *chunk_ptr = sm.chunk_ptr;

        // the 16 bytes of this lane in full sub-tile t
        // (the codes are in device memory: saying so lets the loads be global ones, which do not
        // share a completion counter with the LDS reads of the loop the way generic loads do)
        typedef uint32_t v4u __attribute__((ext_vector_type(4)));
        typedef const __attribute__((address_space(1))) v4u *global_v4u;
        auto load_full = [&](int t) -> uint4 {
            const v4u v = *(global_v4u)(chunk_ptr + (size_t)t * (SUB * CB) + lane * 16);
            return make_uint4(v.x, v.y, v.z, v.w);
        };
        // one sub-tile past the full tiles (zeros for codes past the end of the chunk)
        auto load_ragged = [&](int sidx) -> uint4 {
            uint4 c = make_uint4(0, 0, 0, 0);
            const uint8_t *p = chunk_ptr + (size_t)sidx * (SUB * CB) + lane * 16;
            const int rem = ncodes - sidx * SUB;   // codes from the start of this sub-tile to the end of the chunk
            if (lane * CPL + CPL <= rem) {
                c = *reinterpret_cast<const uint4 *>(p);
            } else if (CPL == 2 && lane * CPL < rem) {
                const uint2 h = *reinterpret_cast<const uint2 *>(p);
                c.x = h.x; c.y = h.y;
            }
            return c;
        };

        // One sub-tile: values of this lane's codes for all queries, threshold test, and the
        // positions of the lanes with a candidate parked in the ring.  No calls in here.
        auto scan_sub = [&](const uint4 cur, const int sidx) {
            uint32_t d[CPL][4];
            code_values<NT, PACKED, DEPTH == 2 ? 16 : 8>(cur, lw, [&](uint32_t off) { return *reinterpret_cast<const uint4 *>(lut_bytes + off); }, d);
            uint64_t hit = 0;
            if constexpr (Q8) {
                // 8-bit fields below 0x80 (sums and thresholds): sum + (0x80 - threshold) has bit 7 set iff the sum
                // is not below the threshold; every field stays within 1 .. 255, so none carries into its neighbour
                uint32_t keep = 0x80808080u;
#pragma unroll
                for (int h = 0; h < CPL; ++h)
#pragma unroll
                    for (int pp = 0; pp < 4; ++pp) keep &= d[h][pp] + tau[pp];
                hit = __ballot(keep != 0x80808080u);
            } else if constexpr (PACKED) {
                // 16-bit fields below 0x8000: the smaller of the lane's two sums minus the threshold
                // wraps (sets bit 15) iff one of them is below the threshold
                typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
                uint32_t below = 0;
#pragma unroll
                for (int pp = 0; pp < 4; ++pp) {
                    u16x2 v = __builtin_bit_cast(u16x2, d[0][pp]);
                    if (CPL == 2) v = __builtin_elementwise_min(v, __builtin_bit_cast(u16x2, d[CPL - 1][pp]));
                    below |= __builtin_bit_cast(uint32_t, (u16x2)(v - __builtin_bit_cast(u16x2, tau[pp])));
                }
                hit = __ballot((below & 0x80008000u) != 0u);
            } else {
#pragma unroll
                for (int h = 0; h < CPL; ++h)
#pragma unroll
                    for (int q = 0; q < QB; ++q) hit |= __ballot(__uint_as_float(d[h][q]) < __uint_as_float(tau[q]));
            }
            if (__builtin_expect(hit != 0ull, 0)) {
                if ((hit >> lane) & 1ull) sm.ring[wave][ring_cnt + mask_prefix(hit)] = (uint32_t)(sidx * SUB + lane * CPL);
                ring_cnt += __popcll(hit);
            }
        };

        // Everything that is not the scan itself happens between steps (a step = a pair of tiles in
        // the main loop, one sub-tile in the tail): parked positions become list inserts, one wave
        // per query re-evaluates the query's histogram now and then, thresholds are re-read.
        // Every wave takes its turn at refreshing one query from the device state: the 16 / QB waves
        // that share a query alternate, so that each query is looked at every 32 steps of the block
        // and no wave carries more of this work than another (with 16 queries per pass, one wave per
        // query, every 128 steps: a look costs a device round trip, and a wave whose bound is stale
        // finds keys and asks earlier, see `pressure`).
        const int my_q = wave % QB;
        const int my_phase = QB > 8 ? 1 + 8 * my_q : 1 + 4 * my_q + 32 * (wave / QB);
        constexpr int REFRESH_MASK = QB > 8 ? 127 : 32 * (TUNED_WAVES / QB) - 1;
        const bool refresher = my_q < nvalid_q;
        // Items that start without a useful bound: no bound at all, or (long result lists) the first
        // item of a block, which only has the loose bound the launch was seeded with.
        const bool cold_item = sm.tau_blk[my_q] >= V::ord_inf() || (KPAD > 128 && a.item_tab == nullptr && gstep == 0);
        int step = 0;
        int pressure = 0;   // positions this wave has flushed (8-bit bounds: keys it has added) since it last refreshed a bound
        auto flush_due = [&]() { return ring_cnt > RING_FLUSH || (ring_cnt > 0 && (step & (RING_PERIOD / 2 - 1)) == 0); };
        // in cold items: at steps 1, 2, 4 .. 32 as well
        auto refresh_due = [&]() {
            return refresher && ((gstep & REFRESH_MASK) == my_phase ||
                                 (wave < QB && cold_item && step <= 32 && (step & (step - 1)) == 0));
        };
        auto between_steps = [&]() {
            bool changed = false;
            PQ_TICK(TICK_LOOP);
            if (flush_due()) {
                // A full ring is drained in whole batches of 64 positions (every lane of the insert path busy); what
                // is left over moves to the front and waits for company.  The periodic drain takes everything.
                const int take = ring_cnt > RING_FLUSH ? (ring_cnt & ~63) : ring_cnt;
                parked_total += (unsigned long long)take;
                int appended;
                if constexpr (PRUNED) appended = scan_flush_pruned<SM, NT, E, QB>(smp, wave_buf, take);
                else if constexpr (U4Q) appended = scan_flush_u4q<SM, E>(smp, wave_buf, take);
                else appended = scan_flush<SM, KIND, E>(smp, wave_buf, take);
                // 8-bit bounds park many codes that turn out to be none: there only the keys count
                pressure += Q8 ? appended : take;
                const int left = ring_cnt - take;   // below 64
                if (left > 0) {
                    const uint32_t moved = lane < left ? sm.ring[wave][take + lane] : 0u;   // (take >= 64 > lane)
                    if (lane < left) sm.ring[wave][lane] = moved;
                }
                ring_cnt = left;
                changed = true;
                PQ_TICK(TICK_FLUSH);
            }
            // a wave that keeps finding candidates asks for a new bound without waiting for its turn
            if (refresh_due() || (refresher && pressure >= KPAD / 2)) {
                scan_refresh<SM, IS_U4>(smp, my_q);
                pressure = 0;
                PQ_TICK(TICK_REFRESH);
            }
            if (changed || step < 32 || (step & 3) == 0) reload_tau();
        };

        // Full sub-tiles go in groups of DEPTH, one register set per sub-tile of the group.  While
        // a group is scanned, the sub-tiles of the wave's next group are requested into the registers
        // just freed, so DEPTH - 1 loads are always on their way; a sub-tile is waited for right
        // before its use (the empty asm reads its last register, and loads complete in order), so
        // that wait never includes younger requests.  The loads are unconditional (past the last group
        // they re-read it and the data is dropped).  Groups are handed out through a counter in LDS,
        // two groups ahead, so that a wave held up by inserts or refreshes simply takes fewer groups
        // and the waves reach the end of the item together.  The inner loop holds no call.
        const int ngroups_t = nfull / DEPTH;
        int g = wave, g_next = wave + TUNED_WAVES;   // the first two groups of a wave are fixed, the counter starts behind them
        if (g < ngroups_t) {
            uint4 buf[DEPTH];
#pragma unroll
            for (int i = 0; i < DEPTH; ++i) buf[i] = load_full(g * DEPTH + i);
            for (;;) {
                bool more;
                do {
                    int after_v = 0;
                    if (lane == 0) after_v = __hip_atomic_fetch_add(&sm.next_group, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    const int gl = g_next < ngroups_t ? g_next : ngroups_t - 1;
#pragma unroll
                    for (int i = 0; i < DEPTH; ++i) {
                        asm volatile("" : "+v"(buf[i].w) : : "memory");
                        const uint4 cur = buf[i];
                        buf[i] = load_full(gl * DEPTH + i);
                        scan_sub(cur, g * DEPTH + i);
                    }
                    g = g_next;
                    g_next = __builtin_amdgcn_readfirstlane(after_v);
                    ++step;
                    ++gstep;
                    more = g < ngroups_t;
                    if (step < 32 || (step & 3) == 0) reload_tau();
                } while (__builtin_expect(more && !flush_due() && !refresh_due(), 1));
                between_steps();
                if (!more) break;
            }
        }
        // what is left after the groups: fewer than DEPTH full sub-tiles and possibly a ragged one,
        // dealt round-robin
        for (int sidx = ngroups_t * DEPTH + wave; sidx < nsub; sidx += TUNED_WAVES) {
            scan_sub(load_ragged(sidx), sidx);
            ++step;
            ++gstep;
            between_steps();
        }

        // ---- end of item: merge the wave lists of each query ------------------------------------
        PQ_TICK(TICK_LOOP);
        if (ring_cnt > 0) {
            parked_total += (unsigned long long)ring_cnt;
            if constexpr (PRUNED) scan_flush_pruned<SM, NT, E, QB>(smp, wave_buf, ring_cnt);
            else if constexpr (U4Q) scan_flush_u4q<SM, E>(smp, wave_buf, ring_cnt);
            else scan_flush<SM, KIND, E>(smp, wave_buf, ring_cnt);
        }
        PQ_TICK(TICK_FLUSH);
        scan_emit_wave<SM, QB, E, KPAD>(smp, wave_buf);
        __syncthreads();   // (orders the waves' scratch writes within the block as well)
        PQ_TICK(TICK_EMIT);
        if (wave < QB) hist_window_flush(smp, wave);   // (every insert of the item is done)
        if (wave == TUNED_WAVES - 1 && lane < QB && sm.ncand_blk[lane] != 0u)   // what the block has not reported yet
            __hip_atomic_fetch_add(sm.ncand[lane], sm.ncand_blk[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Queries whose result list overflowed (loose bounds, first items): if their keys within the
        // bound fit into the ring memory they are sorted there; otherwise every wave's list is cut to
        // its k smallest keys and the lists are merged.
        constexpr int SORT_KEYS = Q8 ? 16384 : 8192;   // the tables' 64 KB (128 KB with the second set) as 64-bit keys
        static_assert(offsetof(SM, lut16) == sizeof(sm.lut), "the second set of tables follows the first");
        uint32_t overflow = 0, sortable = 0;
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int got = sm.out_cnt[q];
            if (got > KPAD) {
                if (got <= SORT_KEYS) sortable |= 1u << q;
                else overflow |= 1u << q;
            }
        }
        __syncthreads();   // every wave has read the counters before any of them is reused
#ifdef PQ_SCAN_TIMING
        if (a.stats != nullptr && threadIdx.x == 0) {
            if (sortable) atomicAdd(a.stats + 7, (unsigned long long)__popc(sortable));
            if (overflow) atomicAdd(a.stats + 8, (unsigned long long)__popc(overflow));
            for (int q = 0; q < QB; ++q) if (sm.out_cnt[q] > KPAD) atomicAdd(a.stats + 9, (unsigned long long)sm.out_cnt[q]);
        }
#endif
        if (__builtin_expect(sortable != 0u, 0)) {
            for (int q = 0; q < QB; ++q)
                if ((sortable >> q) & 1u) scan_overflow_sort<SM, QB, E, KPAD>(smp, wave_buf, q);
        }
        if (__builtin_expect(overflow != 0u, 0)) {
            scan_finish_wave<SM, QB, E>(smp, wave_buf, overflow);
            __syncthreads();
        }
        if (wave < QB && sm.slot_out[wave] != nullptr) {
            if ((overflow >> wave) & 1u) {
                scan_merge_item<SM, QB, E, KPAD>(smp, block_scratch, sm.slot_out[wave]);
            } else if (!((sortable >> wave) & 1u)) {
                uint64_t *out = sm.slot_out[wave];
                for (int i = sm.out_cnt[wave] + lane; i < KPAD; i += 64) out[i] = KEY_EMPTY;
            }
        }
        __syncthreads();
        PQ_TICK(TICK_OVERFLOW);
    }
}

// tau0 (optional, [nq]): a bound already known per query (at least k codes are at or below it);
// times tau0_scale (1, or slightly more when the scan adds in another order than the bound was
// computed in) it seeds the shared bound and serves as the reference of the query's histogram.
__global__ void tuned_init_kernel(uint32_t *work_counter, unsigned long long *tau_key, uint32_t *ncand, uint32_t *mark,
                                  uint32_t *tau_ref, int ntau,
                                  uint32_t tau_value, uint32_t *hist, size_t nhist, const float *tau0, int nq,
                                  float tau0_scale, uint32_t *also_zero = nullptr, size_t also_zero_n = 0) {
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    if (i0 == 0) {
        *work_counter = 0;
        for (int i = 2; i < 32; ++i) work_counter[i] = 0;   // the 64-bit statistics words behind it
    }
    for (size_t i = i0; i < (size_t)ntau; i += stride) {
        const bool seeded = tau0 != nullptr && i < (size_t)nq && tau0[i] < __builtin_inff();
        // enlarged away from the value whatever its sign (tables handed in need not be distances)
        const float bound = seeded ? tau0[i] + fabsf(tau0[i]) * (tau0_scale - 1.f) : 0.f;
        tau_key[i] = ((unsigned long long)(seeded ? f32_to_ord(bound) : tau_value) << 32) | 0xffffffffull;   // (bounds on the value alone: last row)
        tau_ref[i] = seeded ? f32_to_ord(bound) : TAU_REF_UNSET;
        ncand[i] = 0;
        mark[i] = 0;
    }
    for (size_t i = i0; i < nhist; i += stride) hist[i] = 0;
    for (size_t i = i0; i < also_zero_n; i += stride) also_zero[i] = 0;   // (the bins of a first-bound pass that follows)
}

// First bound of the integer scan: one block per SEED_QPB queries adds up the 8-bit table entries of the
// first `cnt` codes (two 4-bit indexes per byte), finds per query the smallest sum T with at least kq
// codes at or below it, and stores it as the query's shared bound (the scan prunes with "<=" against it).
// What limits this kernel is fetching the codes once per block, hence several queries per block: the
// entries of the block's queries for one code byte (both of its components added) are one 8-byte LDS
// read, and their sums add up as four 16-bit fields of a 64-bit word.
constexpr int SEED_QPB = 4;
__global__ __launch_bounds__(1024) void u4_seed_kernel(const uint8_t *__restrict__ codes, int cnt,
                                                       const uint8_t *__restrict__ qluts, int kq, int nq, unsigned long long *tau_key) {
    static_assert(HIST_BINS == 4096, "sums of 16 bytes index the bins");
    __shared__ __align__(16) uint32_t hist[SEED_QPB][HIST_BINS];
    __shared__ uint8_t tab[SEED_QPB][256];
    __shared__ uint2 pair[8][256];
    __shared__ uint32_t cut_s[SEED_QPB];
    const int q0 = blockIdx.x * SEED_QPB, tid = threadIdx.x;
    const int myq = tid >> 8, sub = tid & 255;   // 256 threads per query where the queries are handled apart
    tab[myq][sub] = q0 + myq < nq ? qluts[(size_t)(q0 + myq) * 256 + sub] : (uint8_t)255;
    for (int i = tid; i < SEED_QPB * HIST_BINS; i += 1024) (&hist[0][0])[i] = 0;
    __syncthreads();
    for (int e = tid; e < 8 * 256; e += 1024) {
        const int r = e >> 8, byte = e & 255;
        uint32_t t[SEED_QPB];
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq)
            t[qq] = (uint32_t)tab[qq][(2 * r) * 16 + (byte & 15)] + (uint32_t)tab[qq][(2 * r + 1) * 16 + (byte >> 4)];
        pair[r][byte] = make_uint2(t[0] | (t[1] << 16), t[2] | (t[3] << 16));
    }
    // per query: smallest sum with at least kq counted codes at or below it (4096: fewer than kq counted)
    auto kth_sums = [&]() {   // (the first wave of the query's 256 threads)
        __syncthreads();
        if (sub < 64) {
            const int b = hist_threshold(hist[myq], kq);
            if (sub == 0) cut_s[myq] = (uint32_t)b;
        }
        __syncthreads();
    };
    auto load_code = [&](int i) { return *reinterpret_cast<const uint2 *>(codes + (size_t)i * 8); };
    auto code_sums = [&](const uint2 c) -> uint64_t {   // four sums of at most 16 * 255 < 4096
        uint64_t acc = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint2 v = pair[r][((r < 4 ? c.x : c.y) >> (8 * (r & 3))) & 255u];
            acc += ((uint64_t)v.y << 32) | v.x;
        }
        return acc;
    };
    // The first 4096 codes are all counted; their kq-th sum bounds that of any superset, so of the other
    // codes only the sums up to it need counting.
    const int head = cnt < 4096 ? cnt : 4096;
    __syncthreads();
    // four codes of a thread on their way at a time (the loops are otherwise chains of load latencies)
    auto for_codes = [&](int begin, int end, auto &&f) {
        int i = begin + tid;
        for (; i + 3 * 1024 < end; i += 4 * 1024) {
            const uint2 c0 = load_code(i), c1 = load_code(i + 1024), c2 = load_code(i + 2048), c3 = load_code(i + 3072);
            f(i, code_sums(c0)); f(i + 1024, code_sums(c1)); f(i + 2048, code_sums(c2)); f(i + 3072, code_sums(c3));
        }
        for (; i < end; i += 1024) f(i, code_sums(load_code(i)));
    };
    for_codes(0, head, [&](int, uint64_t acc) {
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq) atomicAdd(&hist[qq][(uint32_t)(acc >> (16 * qq)) & 0xffffu], 1u);
    });
    if (cnt > head) {
        kth_sums();
        uint32_t cut[SEED_QPB];
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq) cut[qq] = cut_s[qq] > 4095u ? 4095u : cut_s[qq];
        for_codes(head, cnt, [&](int, uint64_t acc) {
#pragma unroll
            for (int qq = 0; qq < SEED_QPB; ++qq) {
                const uint32_t sum = (uint32_t)(acc >> (16 * qq)) & 0xffffu;
                if (sum <= cut[qq]) atomicAdd(&hist[qq][sum], 1u);
            }
        });
    }
    kth_sums();
    if (sub == 0 && q0 + myq < nq && cut_s[myq] < 4096u) tau_key[q0 + myq] = ((unsigned long long)cut_s[myq] << 32) | 0xffffffffull;
    // Integer sums tie: far more than kq codes can share the sum T found above (8-bit tables are coarse where the
    // codes crowd), and a bound on the sum alone lets all of them through.  Rows decide among ties, so the bound is
    // handed on as a whole key as well: with r = kq - count(sum < T), the row at the end of the bucket of 1024 sample
    // rows in which the r-th code with sum T falls.  At least kq codes of the sample have a key at or below (T, that row).
    constexpr int TIE_BUCKETS = 256;
    __shared__ uint32_t tie_cnt[SEED_QPB][TIE_BUCKETS];
    __shared__ uint32_t need_s[SEED_QPB];   // r per query, 0: no key bound wanted
    __shared__ int any_s;
    if (tid == 0) any_s = 0;
    for (int i = tid; i < SEED_QPB * TIE_BUCKETS; i += 1024) (&tie_cnt[0][0])[i] = 0;
    __syncthreads();
    if (sub < 64) {   // the first wave of the query's threads: codes below the cut, codes at the cut
        const uint32_t cut = cut_s[myq];
        uint32_t below = 0;
        if (cut < 4096u) for (uint32_t b = sub; b < cut; b += 64) below += hist[myq][b];
        for (int o = 32; o > 0; o >>= 1) below += __shfl_xor(below, o);
        if (sub == 0) {
            uint32_t r = 0;
            // (worth a pass over the sample only if many codes tie at the cut)
            if (q0 + myq < nq && cut < 4096u && below < (uint32_t)kq && below + hist[myq][cut] > (uint32_t)kq + 256u &&
                (cnt + 1023) / 1024 <= TIE_BUCKETS)
                r = (uint32_t)kq - below;
            need_s[myq] = r;
            if (r != 0u) any_s = 1;
        }
    }
    __syncthreads();
    if (any_s == 0) return;
    {
        uint32_t cut[SEED_QPB];
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq) cut[qq] = need_s[qq] != 0u ? cut_s[qq] : 0xffffffffu;
        for_codes(0, cnt, [&](int i, uint64_t acc) {
#pragma unroll
            for (int qq = 0; qq < SEED_QPB; ++qq)
                if (((uint32_t)(acc >> (16 * qq)) & 0xffffu) == cut[qq]) atomicAdd(&tie_cnt[qq][i >> 10], 1u);
        });
    }
    __syncthreads();
    if (sub == 0 && need_s[myq] != 0u) {
        uint32_t cum = 0;
        int b = 0;
        const int nb = (cnt + 1023) / 1024;
        while (b < nb && cum + tie_cnt[myq][b] < need_s[myq]) cum += tie_cnt[myq][b++];
        if (b < nb) {
            const uint32_t last_row = (uint32_t)((b + 1) * 1024 < cnt ? (b + 1) * 1024 : cnt) - 1u;
            tau_key[q0 + myq] = ((unsigned long long)cut_s[myq] << 32) | last_row;
        }
    }
}

// The same over more codes than one block can look at (few query groups, large database):
// block (s, q) counts the sums of slice s of the first `cnt` codes into the query's bins in device
// memory, u4_seed_pick_kernel reads the bound off the counts.
__global__ __launch_bounds__(1024) void u4_seed_hist_kernel(const uint8_t *__restrict__ codes, int64_t cnt,
                                                            const uint8_t *__restrict__ qluts, uint32_t *seed_hist) {
    __shared__ uint32_t hist[4096];
    __shared__ uint8_t tab[256];
    const int q = blockIdx.y, tid = threadIdx.x;
    if (tid < 256) tab[tid] = qluts[(size_t)q * 256 + tid];
    for (int i = tid; i < 4096; i += 1024) hist[i] = 0;
    __syncthreads();
    const int64_t begin = (int64_t)blockIdx.x * (1 << 16);
    const int64_t end = begin + (1 << 16) < cnt ? begin + (1 << 16) : cnt;
    for (int64_t i0 = begin + tid; i0 < end; i0 += 4 * 1024) {
        uint2 c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + u * 1024;
            c[u] = i < end ? *reinterpret_cast<const uint2 *>(codes + (size_t)i * 8) : make_uint2(0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + u * 1024 >= end) break;
            uint32_t sum = 0;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint32_t byte = ((r < 4 ? c[u].x : c[u].y) >> (8 * (r & 3))) & 255u;
                sum += (uint32_t)tab[(2 * r) * 16 + (byte & 15u)] + (uint32_t)tab[(2 * r + 1) * 16 + (byte >> 4)];
            }
            atomicAdd(&hist[sum], 1u);   // sum <= 16 * 255 < 4096
        }
    }
    __syncthreads();
    for (int i = tid; i < 4096; i += 1024)
        if (hist[i] != 0u) atomicAdd(&seed_hist[(size_t)q * 4096 + i], hist[i]);
}

__global__ __launch_bounds__(64) void u4_seed_pick_kernel(const uint32_t *__restrict__ seed_hist, int kq, unsigned long long *tau_key) {
    const int q = blockIdx.x;
    const int b = hist_threshold(seed_hist + (size_t)q * 4096, kq);   // one wave; smallest sum with kq counted codes at or below it
    if (threadIdx.x == 0 && b < HIST_BINS) tau_key[q] = ((unsigned long long)b << 32) | 0xffffffffull;
}

// Better first bound (every candidate the first bound lets through costs far more than a code the
// integer test dismisses): one block per four queries looks at the first `cnt` codes, counts the float distances at or
// below the bound known so far (tau0 as handed in, or with self_ref the greatest distance of the first k codes)
// in the bins the scan's histogram uses, and lowers tau0 to the smallest bin edge with at least k
// distances at or below it, enlarged by 4e-6 of itself: the distances are summed from the lane's own first table on,
// not in table order as in the scans (the tables' layout in LDS, see below).
template <int M>
__global__ __launch_bounds__(1024) void f32_seed_refine_kernel(const uint8_t *__restrict__ codes, int cnt,
                                                               const float *__restrict__ luts, int k, bool self_ref, int nq,
                                                               float *tau0) {
    // SEED_QPB queries per block (the kernel is limited by fetching the codes once per block): entry e of table j
    // for the block's queries is one 16-byte LDS read
    static_assert(SEED_QPB == 4, "four queries share a float4");
    __shared__ float4 tab[M * 256];
    __shared__ __align__(16) uint32_t hist[SEED_QPB][HIST_BINS];
    __shared__ uint32_t ref_s[SEED_QPB];
    const int q0 = blockIdx.x * SEED_QPB, tid = threadIdx.x;
    const int myq = tid >> 8, sub = tid & 255;   // 256 threads per query where the queries are handled apart
    // entry b of table j at slot b * M + j: a lane walks the tables from its own first one (lane % M), so the 16 lanes that the
    // LDS serves together read at least 8 different bank groups whatever their bytes are (all in one table: 16 random ones)
    for (int e = tid; e < M * 256; e += 1024) {
        float v[SEED_QPB];
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq) v[qq] = q0 + qq < nq ? luts[(size_t)(q0 + qq) * (M * 256) + e] : __builtin_inff();
        tab[(e & 255) * M + (e >> 8)] = make_float4(v[0], v[1], v[2], v[3]);
    }
    const uint32_t rot = (uint32_t)tid & (M - 1);
    for (int i = tid; i < SEED_QPB * HIST_BINS; i += 1024) (&hist[0][0])[i] = 0;
    if (sub == 0) ref_s[myq] = self_ref || q0 + myq >= nq ? 0u : f32_to_ord(tau0[q0 + myq]);
    __syncthreads();
    struct Code { uint32_t w[M / 4]; };
    auto load_code = [&](int i) {
        Code c;
        if (M == 8) {
            const uint2 v = *reinterpret_cast<const uint2 *>(codes + (size_t)i * 8);
            c.w[0] = v.x; c.w[1] = v.y;
        } else {
            const uint4 v = *reinterpret_cast<const uint4 *>(codes + (size_t)i * 16);
            c.w[0] = v.x; c.w[1] = v.y; c.w[M / 4 - 2] = v.z; c.w[M / 4 - 1] = v.w;
        }
        return c;
    };
    auto dist_ords = [&](Code c, uint32_t (&ord)[SEED_QPB]) {
        uint32_t (&w)[M / 4] = c.w;
        if constexpr (M == 8) rot8(w[0], w[1], (rot & 4u) != 0u, rot & 3u);
        else rot16(w, rot);
        float4 d = tab[(w[0] & 255u) * M + rot];   // (step s: byte s of the rotated code, table (rot + s) % M)
#pragma unroll
        for (int st = 1; st < M; ++st) {
            const float4 t = tab[((w[st >> 2] >> (8 * (st & 3))) & 255u) * M + ((rot + st) & (M - 1))];
            d.x += t.x; d.y += t.y; d.z += t.z; d.w += t.w;
        }
        ord[0] = f32_to_ord(d.x); ord[1] = f32_to_ord(d.y); ord[2] = f32_to_ord(d.z); ord[3] = f32_to_ord(d.w);
    };
    if (self_ref) {   // no bound yet: the greatest distance among the first k codes is one
        for (int i = tid; i < k && i < cnt; i += 1024) {
            uint32_t ord[SEED_QPB];
            dist_ords(load_code(i), ord);
#pragma unroll
            for (int qq = 0; qq < SEED_QPB; ++qq) atomicMax(&ref_s[qq], ord[qq]);
        }
        __syncthreads();
    }
    uint32_t ref[SEED_QPB];
#pragma unroll
    for (int qq = 0; qq < SEED_QPB; ++qq) ref[qq] = ref_s[qq];
    __shared__ int bin_s[SEED_QPB];
    // per query: the smallest bin with at least k counted distances in the bins up to it (HIST_BINS: fewer than k)
    auto kth_bins = [&]() {   // (the first wave of the query's 256 threads)
        __syncthreads();
        if (sub < 64) {
            const int b = hist_threshold(hist[myq], k);
            if (sub == 0) bin_s[myq] = b;
        }
        __syncthreads();
    };
    // every distance counted in bins <= b is at or below this edge, every other one above it
    auto edge_of = [&](uint32_t rq, int b) { return rq - ((uint32_t)(HIST_BINS - 1 - b) << HIST_SHIFT); };
    auto count = [&](const Code &c, const uint32_t (&limit)[SEED_QPB]) {
        uint32_t ord[SEED_QPB];
        dist_ords(c, ord);
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq) {
            if (ord[qq] <= limit[qq]) {
                const uint32_t below = (ref[qq] - ord[qq]) >> HIST_SHIFT;
                atomicAdd(&hist[qq][HIST_BINS - 1 - (below < HIST_BINS ? below : HIST_BINS - 1)], 1u);
            }
        }
    };
    // The first 4096 codes are counted against the reference; the bin edge they give bounds the answer over any
    // superset, so of the other codes only the distances up to that edge need counting (counting them all is
    // what this kernel would spend most of its time on).
    const int head = cnt < 4096 ? cnt : 4096;
    // four codes of a thread on their way at a time (the loop is otherwise a chain of load latencies)
    auto count_range = [&](int begin, int end, const uint32_t (&limit)[SEED_QPB]) {
        int i = begin + tid;
        for (; i + 3 * 1024 < end; i += 4 * 1024) {
            const Code c0 = load_code(i), c1 = load_code(i + 1024), c2 = load_code(i + 2048), c3 = load_code(i + 3072);
            count(c0, limit); count(c1, limit); count(c2, limit); count(c3, limit);
        }
        for (; i < end; i += 1024) count(load_code(i), limit);
    };
    count_range(0, head, ref);
    if (cnt > head) {
        kth_bins();
        uint32_t limit[SEED_QPB];
#pragma unroll
        for (int qq = 0; qq < SEED_QPB; ++qq) limit[qq] = bin_s[qq] < HIST_BINS ? edge_of(ref[qq], bin_s[qq]) : ref[qq];
        count_range(head, cnt, limit);
    }
    kth_bins();
    if (sub == 0 && q0 + myq < nq) {
        const int q = q0 + myq;
        // (enlarged by a few units of fp32 rounding: the scans add a code's entries in table order, this kernel from
        // the lane's own first table on)
        auto enlarged = [](float x) { return x + fabsf(x) * 4e-6f; };
        if (bin_s[myq] < HIST_BINS) tau0[q] = enlarged(ord_to_f32(edge_of(ref_s[myq], bin_s[myq])));
        else if (self_ref) tau0[q] = cnt >= k ? enlarged(ord_to_f32(ref_s[myq])) : __builtin_inff();
    }
}

// The same refinement over more codes than one block can look at (flat scans of few
// query groups over large databases, where every candidate the first bound lets through costs more
// than a code it dismisses): block (s, q) counts the distances of slice s at or below the query's
// bound in the bins of the scan's histogram and adds its counts to the query's bins in device memory;
// f32_seed_pick_kernel then lowers the bound to the smallest bin edge with at least k distances.
constexpr int SEED_SLICE = 1 << 16;
__global__ __launch_bounds__(1024) void f32_seed_hist_kernel(const uint8_t *__restrict__ codes, int64_t cnt,
                                                             const float *__restrict__ luts, const float *__restrict__ tau0,
                                                             uint32_t *seed_hist) {
    __shared__ float tab[8 * 256];
    __shared__ uint32_t hist[HIST_BINS];
    const int q = blockIdx.y, tid = threadIdx.x;
    for (int i = tid; i < 2048; i += 1024) tab[i] = luts[(size_t)q * 2048 + i];
    for (int i = tid; i < HIST_BINS; i += 1024) hist[i] = 0;
    __syncthreads();
    const uint32_t ref = f32_to_ord(tau0[q]);
    const int64_t begin = (int64_t)blockIdx.x * SEED_SLICE;
    const int64_t end = begin + SEED_SLICE < cnt ? begin + SEED_SLICE : cnt;
    for (int64_t i0 = begin + tid; i0 < end; i0 += 4 * 1024) {
        uint2 c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + u * 1024;
            c[u] = i < end ? *reinterpret_cast<const uint2 *>(codes + (size_t)i * 8) : make_uint2(0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + u * 1024 >= end) break;
            float d = tab[c[u].x & 255u];
            d += tab[256 + ((c[u].x >> 8) & 255u)];
            d += tab[512 + ((c[u].x >> 16) & 255u)];
            d += tab[768 + (c[u].x >> 24)];
            d += tab[1024 + (c[u].y & 255u)];
            d += tab[1280 + ((c[u].y >> 8) & 255u)];
            d += tab[1536 + ((c[u].y >> 16) & 255u)];
            d += tab[1792 + (c[u].y >> 24)];
            const uint32_t ord = f32_to_ord(d);
            if (ord <= ref) {
                const uint32_t below = (ref - ord) >> HIST_SHIFT;
                atomicAdd(&hist[HIST_BINS - 1 - (below < HIST_BINS ? below : HIST_BINS - 1)], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < HIST_BINS; i += 1024)
        if (hist[i] != 0u) atomicAdd(&seed_hist[(size_t)q * HIST_BINS + i], hist[i]);
}

// The same sample without a pass before it: the bins hang below ref0 = the sum of the tables' greatest entries (no
// distance exceeds it; 4096 bins of 0.2 % reach down to 1/4000 of it), which every block works out for itself from
// the tables it stages anyway.  A block counts its first 4096 codes in full; the k-th smallest of those bounds the
// k-th smallest of the whole sample, so of its other codes only the ones at or below that bin edge are counted.
// Blocks of `slice` codes (many short blocks when few queries share the launch: the pass is a chain of load latencies,
// not bandwidth).
constexpr int SEED2_SLICE = 1 << 14;
__global__ __launch_bounds__(1024) void f32_seed_hist2_kernel(const uint8_t *__restrict__ codes, int64_t cnt, int slice,
                                                              const float *__restrict__ luts, int k, uint32_t *seed_hist,
                                                              float *seed_ref) {
    __shared__ float tab[8 * 256];
    __shared__ __align__(16) uint32_t hist[HIST_BINS];
    __shared__ float smax[8];
    __shared__ int bin_s;
    const int q = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 2048; i += 1024) tab[i] = luts[(size_t)q * 2048 + i];
    for (int i = tid; i < HIST_BINS; i += 1024) hist[i] = 0;
    __syncthreads();
    if (wave < 8) {
        float v = fmaxf(fmaxf(tab[wave * 256 + lane], tab[wave * 256 + lane + 64]), fmaxf(tab[wave * 256 + lane + 128], tab[wave * 256 + lane + 192]));
        for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
        if (lane == 0) smax[wave] = v;
    }
    __syncthreads();
    float ref0 = smax[0];
    for (int j = 1; j < 8; ++j) ref0 += smax[j];
    if (blockIdx.x == 0 && tid == 0) seed_ref[q] = ref0;
    const uint32_t ref = f32_to_ord(ref0);
    const int64_t begin = (int64_t)blockIdx.x * slice;
    const int64_t end = begin + slice < cnt ? begin + slice : cnt;
    auto count_range = [&](int64_t from, int64_t to, uint32_t limit) {
        for (int64_t i0 = from + tid; i0 < to; i0 += 4 * 1024) {
            uint2 c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t i = i0 + u * 1024;
                c[u] = i < to ? *reinterpret_cast<const uint2 *>(codes + (size_t)i * 8) : make_uint2(0, 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (i0 + u * 1024 >= to) break;
                float d = tab[c[u].x & 255u];
                d += tab[256 + ((c[u].x >> 8) & 255u)];
                d += tab[512 + ((c[u].x >> 16) & 255u)];
                d += tab[768 + (c[u].x >> 24)];
                d += tab[1024 + (c[u].y & 255u)];
                d += tab[1280 + ((c[u].y >> 8) & 255u)];
                d += tab[1536 + ((c[u].y >> 16) & 255u)];
                d += tab[1792 + (c[u].y >> 24)];
                const uint32_t ord = f32_to_ord(d);
                if (ord <= limit) {
                    const uint32_t below = (ref - ord) >> HIST_SHIFT;
                    atomicAdd(&hist[HIST_BINS - 1 - (below < HIST_BINS ? below : HIST_BINS - 1)], 1u);
                }
            }
        }
    };
    const int64_t head_end = begin + 4096 < end ? begin + 4096 : end;
    count_range(begin, head_end, ref);
    if (head_end < end) {
        __syncthreads();
        if (wave == 0) {
            const int b = hist_threshold(hist, k);
            if (lane == 0) bin_s = b;
        }
        __syncthreads();
        const uint32_t limit = bin_s < HIST_BINS ? ref - ((uint32_t)(HIST_BINS - 1 - bin_s) << HIST_SHIFT) : ref;
        count_range(head_end, end, limit);
    }
    __syncthreads();
    for (int i = tid; i < HIST_BINS; i += 1024)
        if (hist[i] != 0u) atomicAdd(&seed_hist[(size_t)q * HIST_BINS + i], hist[i]);
}

__global__ __launch_bounds__(64) void f32_seed_pick_kernel(const uint32_t *__restrict__ seed_hist, int k, float *tau0) {
    const int q = blockIdx.x;
    const int b = hist_threshold(seed_hist + (size_t)q * HIST_BINS, k);   // one wave
    if (threadIdx.x == 0 && b < HIST_BINS) {
        const uint32_t ref = f32_to_ord(tau0[q]);
        tau0[q] = ord_to_f32(ref - ((uint32_t)(HIST_BINS - 1 - b) << HIST_SHIFT));
    }
}

__global__ void zero_u32_kernel(uint32_t *p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// 16-bit tables of the pruned float scan.  Blocks (group, y) of 256 threads: every block of a group works out the
// minima and scales of the group's queries, block y writes the tables y, y + gridDim.y, ...
// Per query: off = sum over the tables of their minimum entry, scale = PRUNE_RANGE / (tau0 - off)
// (0, which disables the pruning of that query, if tau0 leaves no usable range), and for every table
// L[j][b] = min(32767 / M, floor((D[j][b] - min_j) * scale)) for the M = 8 or 16 tables.  Output in
// the slot order of the scan kernel: qtabs[group][b][j] holds entry b of table j for the 8 queries
// of the group.
// With seed_hist given, the kernel first reads every query's first bound off the bins of the sampling pass
// (f32_seed_hist2_kernel; bins below seed_ref) and stores it as tau0, as the query's shared bound and as the reference
// of its scan histogram: one launch instead of three.
template <int M, int G = 8>   // G: queries per group (8 with 16-bit entries, 16 with 8-bit entries)
__global__ __launch_bounds__(256) void prune_tables_kernel(const float *__restrict__ luts, float *tau0,
                                                           int nq, uint4 *qtabs, float *off_out, float *scale_out, float range_q8,
                                                           uint4 *qtabs16, float *scale16_out, const uint32_t *seed_hist = nullptr,
                                                           const float *seed_ref = nullptr, int seed_k = 0,
                                                           unsigned long long *tau_key_out = nullptr, uint32_t *tau_ref_out = nullptr) {
    constexpr bool Q8 = G == 16;
    constexpr float ENTRY_MAX = Q8 ? PRUNE_ENTRY_MAX_Q8 : (float)(32767 / M);   // M entries must add up to less than 2^15 (2^7)
    const float RANGE = Q8 ? range_q8 : PRUNE_RANGE;
    static_assert(!Q8 || M == 8, "8-bit entries: eight tables");
    __shared__ float smin[G][M];
    __shared__ float sscale[G];
    __shared__ float sscale16[G];   // 8-bit entries: the scale of the 16-bit tables written beside them
    const int group = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (seed_hist != nullptr) {
        for (int q = wave; q < G; q += 4) {
            const int gq = group * G + q;
            if (gq >= nq) continue;
            const int b = hist_threshold(seed_hist + (size_t)gq * HIST_BINS, seed_k);
            if (lane == 0) {
                const uint32_t ref = f32_to_ord(seed_ref[gq]);
                const uint32_t edge = b < HIST_BINS ? ref - ((uint32_t)(HIST_BINS - 1 - b) << HIST_SHIFT) : ref;
                tau0[gq] = ord_to_f32(edge);   // (every block of the group stores the same value)
                if (blockIdx.y == 0) {
                    tau_key_out[gq] = ((unsigned long long)edge << 32) | 0xffffffffull;
                    tau_ref_out[gq] = edge;
                }
            }
        }
        __syncthreads();
    }
    for (int r = wave * (G * M / 4); r < (wave + 1) * (G * M / 4); ++r) {
        const int q = r / M, j = r % M, gq = group * G + q;
        float v = __builtin_inff();
        if (gq < nq) {
            const float *t = luts + ((size_t)gq * M + j) * 256;
            v = fminf(fminf(t[lane], t[lane + 64]), fminf(t[lane + 128], t[lane + 192]));
        }
        for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
        if (lane == 0) smin[q][j] = v;
    }
    __syncthreads();
    if (tid < G) {
        const int gq = group * G + tid;
        float scale = 0.f;
        if (gq < nq) {
            float off = 0.f;
            for (int j = 0; j < M; ++j) off += smin[tid][j];
            // RANGE units between the sum of the minima and the first bound, but never so many per unit of distance that
            // the threshold conversion loses a fraction of a table unit in fp32 (bound * scale stays below 10^6).  A bound
            // that leaves no range at all (k codes and more attain the minima: exact duplicates) takes that finest scale:
            // any entry above its table's minimum then counts several units and only the duplicates pass.
            const float bound = tau0[gq], range = bound - off;
            const float finest = bound > 0.f && bound < 3.0e38f ? 0.99e6f / bound : 0.f;
            auto scale_for = [&](float units) {
                float sc = range > 0.f ? units / range : finest;
                if (!(sc < finest)) sc = finest;
                return sc > 0.f && sc < 3.0e38f ? sc : 0.f;
            };
            scale = scale_for(RANGE);
            if (blockIdx.y == 0) { off_out[gq] = off; scale_out[gq] = scale; }
            if constexpr (Q8) {
                const float scale16 = scale_for(PRUNE_RANGE);
                if (blockIdx.y == 0) scale16_out[gq] = scale16;
                sscale16[tid] = scale16;
            }
        } else if (Q8) {
            sscale16[tid] = 0.f;
        }
        sscale[tid] = scale;
    }
    __syncthreads();
    const int b = tid;
    for (int j = blockIdx.y; j < M; j += gridDim.y) {
        uint32_t e[G];
#pragma unroll
        for (int q = 0; q < G; ++q) {
            const int gq = group * G + q;
            e[q] = (uint32_t)ENTRY_MAX;   // no query in this slot: sums that never qualify
            if (gq < nq) {
                const float x = (luts[((size_t)gq * M + j) * 256 + b] - smin[q][j]) * sscale[q];
                e[q] = (uint32_t)fminf(floorf(x), ENTRY_MAX);
            }
        }
        uint4 pk;
        if constexpr (Q8) {
            pk = make_uint4(e[0] | (e[1] << 8) | (e[2] << 16) | (e[3] << 24), e[4] | (e[5] << 8) | (e[6] << 16) | (e[7] << 24),
                            e[8] | (e[9] << 8) | (e[10] << 16) | (e[11] << 24), e[12] | (e[13] << 8) | (e[14] << 16) | (e[15] << 24));
        } else {
            pk = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
        }
        qtabs[(size_t)group * (256 * M) + b * M + j] = pk;
        if constexpr (Q8) {   // 16-bit entries of the same 16 queries, two halves of 8
            uint32_t w[G];
#pragma unroll
            for (int q = 0; q < G; ++q) {
                const int gq = group * G + q;
                w[q] = 4095u;
                if (gq < nq) {
                    const float x = (luts[((size_t)gq * M + j) * 256 + b] - smin[q][j]) * sscale16[q];
                    w[q] = (uint32_t)fminf(floorf(x), 4095.f);
                }
            }
            uint4 *dst = qtabs16 + (size_t)group * 4096 + (size_t)(b * 8 + j) * 2;
            dst[0] = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
            dst[1] = make_uint4(w[8] | (w[9] << 16), w[10] | (w[11] << 16), w[12] | (w[13] << 16), w[14] | (w[15] << 16));
        }
    }
}

template <int KIND, int E, int KPAD, int DEPTH>
static int launch_kind(pq_ctx *ctx, const TunedArgs &a, int nblocks) {
    scan_tuned_kernel<KIND, E, KPAD, DEPTH><<<nblocks, TUNED_THREADS, 0, ctx->stream>>>(a);
    PQ_HIP(ctx, hipGetLastError());
    return PQ_OK;
}

struct StateLayout {
    size_t off_key, off_ncand, off_mark, off_ref, off_hist, off_scratch, total;
    size_t nhist;
};

static StateLayout state_layout(int qb, int ntau, int cap, int nblocks) {
    StateLayout L;
    L.off_key = 256;
    L.off_ncand = L.off_key + align_up((size_t)ntau * 8, 256);
    L.off_mark = L.off_ncand + align_up((size_t)ntau * 4, 256);
    L.off_ref = L.off_mark + align_up((size_t)ntau * 4, 256);
    L.off_hist = L.off_ref + align_up((size_t)ntau * 4, 256);
    L.nhist = (size_t)ntau * HIST_BINS;
    L.off_scratch = L.off_hist + align_up(L.nhist * 4, 256);
    L.total = L.off_scratch + (size_t)nblocks * TUNED_WAVES * qb * cap * 8;
    return L;
}

static void bind_state(TunedArgs &a, uint8_t *ws, const StateLayout &L) {
    a.work_counter = (uint32_t *)ws;
    a.stats = nullptr;
    a.tau_key = (unsigned long long *)(ws + L.off_key);
    a.ncand = (uint32_t *)(ws + L.off_ncand);
    a.refresh_mark = (uint32_t *)(ws + L.off_mark);
    a.tau_ref = (uint32_t *)(ws + L.off_ref);
    a.hist = (uint32_t *)(ws + L.off_hist);
    a.scratch = (uint64_t *)(ws + L.off_scratch);
}

// DEPTH (sub-tiles per group, see the kernel): two when the same codes serve many query groups at
// about the same time and so come from the caches; eight when they stream from HBM (inverted
// lists, scans for few queries), which takes more bytes on their way per wave.
template <int KIND>
static int launch_kind_sized(pq_ctx *ctx, bool small, bool stream, const TunedArgs &a, int nblocks) {
#if PQ_TUNED_ITEMS_ONLY
    // work items of inverted lists: groups of four sub-tiles keep the rings small enough for two
    // blocks per CU
    (void)small; (void)stream;
    return launch_kind<KIND, E_SMALL, 128, 4>(ctx, a, nblocks);
#else
    if (stream) {
        if constexpr (KIND == KIND_F32Q_M8 || KIND == KIND_U4Q_M16) return fail(ctx, PQ_EINVAL, "scan: the 16-query kinds serve many query groups only");
        else return small ? launch_kind<KIND, E_SMALL, 128, 8>(ctx, a, nblocks) : launch_kind<KIND, E_LARGE, 1024, 8>(ctx, a, nblocks);
    }
    return small ? launch_kind<KIND, E_SMALL, 128, 2>(ctx, a, nblocks) : launch_kind<KIND, E_LARGE, 1024, 2>(ctx, a, nblocks);
#endif
}

static int launch_by_kind(pq_ctx *ctx, int kind, bool small, bool stream, const TunedArgs &a, int nblocks) {
    switch (kind) {
        case KIND_F32_M8: return launch_kind_sized<KIND_F32_M8>(ctx, small, stream, a, nblocks);
        case KIND_F32_M16: return launch_kind_sized<KIND_F32_M16>(ctx, small, stream, a, nblocks);
        case KIND_F32P_M8: return launch_kind_sized<KIND_F32P_M8>(ctx, small, stream, a, nblocks);
        case KIND_F32P_M16: return launch_kind_sized<KIND_F32P_M16>(ctx, small, stream, a, nblocks);
#if !PQ_TUNED_ITEMS_ONLY
        case KIND_F32Q_M8: return launch_kind_sized<KIND_F32Q_M8>(ctx, small, stream, a, nblocks);
        case KIND_U4Q_M16: return launch_kind_sized<KIND_U4Q_M16>(ctx, small, stream, a, nblocks);
#endif
#if PQ_TUNED_ITEMS_ONLY
        default: return fail(ctx, PQ_EUNSUPPORTED, "scan_items: kind %d", kind);
#else
        default: return launch_kind_sized<KIND_U4_M16>(ctx, small, stream, a, nblocks);
#endif
    }
}

// measurement aid: what the scan about to be launched is, and where its counters live
static void note_scan(pq_ctx *ctx, int kind, int qb, int passes, const unsigned long long *parked, const uint32_t *ncand, int ncand_len) {
    static const char *const names[] = {"F32_M8 (8x8 float, plain float adds, 4 queries per pass)", "F32_M16 (16x8 float, plain float adds, 4 queries per pass)",
                                        "U4_M16 (16x4 integer, exact 16-bit sums, 8 queries per pass)",
                                        "F32P_M8 (8x8 float on 16-bit lower bounds, 8 queries per pass)", "F32P_M16 (16x8 float on 16-bit lower bounds, 8 queries per pass)",
                                        "F32Q_M8 (8x8 float on 8-bit lower bounds, 16 queries per pass)", "U4Q_M16 (16x4 integer on 8-bit lower bounds, 16 queries per pass)"};
    snprintf(ctx->last_scan_name, sizeof(ctx->last_scan_name), "scan_tuned_kernel<%s>, blocks of %d waves", kind >= 0 && kind < 7 ? names[kind] : "?", TUNED_WAVES);
    ctx->last_scan_qpp = qb;
    ctx->last_scan_passes = passes;
    ctx->stat_parked = parked;
    ctx->stat_ncand = ncand;
    ctx->stat_ncand_len = ncand_len;
}

static int qb_of_kind(int kind) {
    return kind == KIND_F32Q_M8 || kind == KIND_U4Q_M16 ? 16 : (kind == KIND_U4_M16 || kind == KIND_F32P_M8 || kind == KIND_F32P_M16 ? 8 : 4);
}

// blocks that share a CU: one of 16 waves, two of 8
constexpr int BLOCKS_PER_CU = 16 / TUNED_WAVES;

size_t tuned_state_bytes(int kind, int nq, int topk, int num_cu) {
    const int qb = qb_of_kind(kind);
    const int cap = 64 * (topk <= 128 ? E_SMALL : E_LARGE);
    return state_layout(qb, nq, cap, num_cu * BLOCKS_PER_CU).total;
}

int launch_scan_items(pq_ctx *ctx, int kind, const float *pair_min, const float *pair_off, const float *pair_scale,
                      const uint8_t *codes, const float *luts, int nq, int nprobe, int topk,
                      const IvfItem *items, const uint32_t *nitems_dev, const int32_t *pairs_by_list,
                      const uint32_t *pair_out, uint64_t *partial, uint8_t *state, size_t state_bytes,
                      const float *tau0, unsigned long long **tau_key_out) {
    const int qb = qb_of_kind(kind);
    if ((kind == KIND_F32P_M8 || kind == KIND_F32P_M16) && (!pair_min || !pair_off || !pair_scale))
        return fail(ctx, PQ_EINVAL, "scan_items: the pruned scan needs the pairs' minima, offsets and scales");
    const bool small = topk <= 128;
    const int cap = 64 * (small ? E_SMALL : E_LARGE);
    const int nblocks = ctx->num_cu * BLOCKS_PER_CU;
    if (!small) return fail(ctx, PQ_EUNSUPPORTED, "scan_items: topk above 128");
    const StateLayout L = state_layout(qb, nq, cap, nblocks);
    if (L.total > state_bytes) return fail(ctx, PQ_EINVAL, "scan_items: state region too small");
    TunedArgs a;
    a.codes = codes; a.n = 0; a.chunk_codes = 0; a.head_codes = 0; a.head_chunks = 0; a.nchunks = 0; a.ngroups = 1; a.nitems = 0;
    a.luts = luts; a.nq = nq; a.topk = topk;
    bind_state(a, state, L);
    a.partial = partial;
    a.item_tab = items; a.nitems_dev = nitems_dev; a.pairs_by_list = pairs_by_list; a.pair_out = pair_out;
    a.nprobe = nprobe;
    a.qtabs = nullptr; a.prune_off = pair_off; a.prune_scale = pair_scale; a.pair_min = pair_min;
    a.qtabs16 = nullptr; a.prune_scale16 = nullptr;
    tuned_init_kernel<<<1024, 256, 0, ctx->stream>>>(a.work_counter, a.tau_key, a.ncand, a.refresh_mark, a.tau_ref, nq,
                                                     0xff800000u, a.hist, L.nhist, tau0, nq, 1.f);
    PQ_HIP(ctx, hipGetLastError());
    if (ctx->profiling) {
        a.stats = (unsigned long long *)(state + 8);
        note_scan(ctx, kind, qb, 0, a.stats, a.ncand, nq);
        PQ_HIP(ctx, hipEventRecord(ctx->ev_begin, ctx->stream));
    }
    int rc = launch_by_kind(ctx, kind, small, true, a, nblocks);
    if (rc) return rc;
    if (ctx->profiling) {
        PQ_HIP(ctx, hipEventRecord(ctx->ev_end, ctx->stream));
        ctx->ev_valid = 1;
    }
    *tau_key_out = a.tau_key;
    return PQ_OK;
}

#if !PQ_TUNED_ITEMS_ONLY
int launch_scan_tuned(pq_ctx *ctx, int kind, const uint8_t *codes, int64_t n, const void *luts, int nq, int topk,
                      void *out_val, int64_t *out_ids) {
    int rc;
    const bool is_u4 = kind == KIND_U4_M16;
    // The 8 x 256 float scan prunes with 16-bit lower bounds when the database is large enough to
    // pay for the preparation (a bound per query from the first PRUNE_INIT codes, then the tables).
    const bool prune = (kind == KIND_F32_M8 || kind == KIND_F32_M16) && n >= PRUNE_MIN_N && opt_int(ctx, PQ_OPT_SCAN_PRUNE, 1) != 0;
    const int tables = kind == KIND_F32_M16 ? 16 : 8;
    // eight tables and too many queries for the streaming shape (32 groups of 8 and more, i.e. 249 queries): 8-bit
    // lower bounds, 16 queries per pass (PQ_SCAN_Q8=0: 16-bit lower bounds, 8 queries per pass).  Measured on 25 M
    // codes: 256 queries 1.69 -> 1.28 ms, 384 queries 2.28 -> 1.51 ms; 128 queries in the streaming shape 0.62 ms
    // against 1.21 ms with this loop.
    const bool many16 = (nq + 7) / 8 >= STREAM_GROUPS && opt_int(ctx, PQ_OPT_SCAN_Q8, 1) != 0;
    const bool q8 = prune && tables == 8 && many16;
    if (prune) kind = q8 ? KIND_F32Q_M8 : (tables == 16 ? KIND_F32P_M16 : KIND_F32P_M8);
    // the integer scan likewise: with a first bound and enough queries, its loop runs on 8-bit lower bounds of
    // the integer sums, 16 queries per pass
    const bool u4q = is_u4 && n >= PRUNE_MIN_N && many16;
    if (u4q) kind = KIND_U4Q_M16;
    const int qb = q8 || u4q ? 16 : (is_u4 || prune ? 8 : 4);
    const int cb = kind == KIND_F32_M16 || kind == KIND_F32P_M16 ? 16 : 8;
    const int depth = !(q8 || u4q) && (nq + qb - 1) / qb < STREAM_GROUPS ? 8 : 2;
    const int tile = 64 * (16 / cb) * depth;   // codes per wave group (DEPTH sub-tiles)
    const bool small = topk <= 128;
    const int kpad = small ? 128 : 1024;
    const int cap = 64 * (small ? E_SMALL : E_LARGE);
    const int ngroups = (nq + qb - 1) / qb;
    const int64_t block_tile = (int64_t)tile * TUNED_WAVES;
    // persistent blocks: one per CU (64 KB of tables and 16 waves of 128 registers fill a CU)
    int nblocks_max = opt_int(ctx, PQ_OPT_SCAN_BLOCKS, ctx->num_cu);
    if (nblocks_max < 1) nblocks_max = 1;

    // several items per block for balance, chunks of at least 8 block tiles
    // (six for the 16-query loops: 2 .. 4 % faster than four on 25 M codes, more than eight slower again)
    // Long result lists on the 16-query loops start with a round of short items, one per block (PQ_SCAN_HEAD block
    // tiles per chunk, 4 by default, if that is a small part of the database): every block's first long item then
    // starts on bounds from a sample of several of them instead of on the first bound.  Measured on 25 M codes,
    // top-1000: 256 queries 2.44 -> 1.97 ms per step, 1000 queries 4.31 -> 4.27 ms; top-100 loses 1 .. 2 %.
    int head_chunks = 0;
    int64_t head_codes = 0;
    if ((q8 || u4q) && topk > 128) {
        const int64_t hc = (int64_t)opt_int(ctx, PQ_OPT_SCAN_HEAD, 4) * block_tile;
        const int64_t c0 = (nblocks_max + ngroups - 1) / ngroups;
        if (hc > 0 && c0 * hc * 16 <= n) { head_chunks = (int)c0; head_codes = hc; }
    }
    const int64_t n_head = (int64_t)head_chunks * head_codes, n_main = n - n_head;
    // Up to 8 query groups over a large database (streaming shape): one item per block.  All items are equally long there,
    // so nothing is gained by handing out several, and every item pays its set-up (tables, bounds, first codes) and
    // leaves a result list for the merge (10^8 codes, one query: scan 0.21 -> 0.19 ms, call 0.39 -> 0.34 ms).
    const int ipb_default = q8 || u4q ? 6 : (ngroups <= 8 && (nq + qb - 1) / qb < STREAM_GROUPS && n >= ((int64_t)1 << 22) ? 1 : 4);
    const int ipb = opt_int(ctx, PQ_OPT_SCAN_ITEMS_PER_BLOCK, ipb_default);
    int64_t nchunks = ipb == 1 ? (nblocks_max >= ngroups ? nblocks_max / ngroups : 1)   // (never more items than blocks)
                               : ((int64_t)ipb * nblocks_max + ngroups - 1) / ngroups;
    const int64_t max_by_n = (n_main + 8 * block_tile - 1) / (8 * block_tile);
    if (nchunks > max_by_n) nchunks = max_by_n;
    const int64_t min_chunks = (n_main + ((int64_t)1 << 30) - 1) >> 30;   // a chunk's rows are counted in 32 bits
    if (nchunks < min_chunks) nchunks = min_chunks;
    if (nchunks < 1) nchunks = 1;
    int64_t chunk_codes = (n_main + nchunks - 1) / nchunks;
    chunk_codes = (chunk_codes + block_tile - 1) / block_tile * block_tile;
    if (chunk_codes < block_tile) chunk_codes = block_tile;
    nchunks = (n_main > 0 ? (n_main + chunk_codes - 1) / chunk_codes : 1) + head_chunks;   // (all chunks, the short ones first)
    const int64_t nitems = nchunks * ngroups;
    if (nitems > 0x3fffffff) return fail(ctx, PQ_EUNSUPPORTED, "scan: too many work items (%lld)", (long long)nitems);
    const int nblocks = (int)(nitems < nblocks_max ? nitems : nblocks_max);

    const int ntau = ngroups * qb;
    const StateLayout L = state_layout(qb, ntau, cap, nblocks);
    const size_t off_partial = align_up(L.total, 256);
    const size_t off_tau0 = off_partial + align_up((size_t)nitems * qb * kpad * 8, 256);
    const size_t off_poff = off_tau0 + align_up((size_t)ntau * 4, 256);
    const size_t off_pscale = off_poff + align_up((size_t)ntau * 4, 256);
    const size_t off_qtabs = off_pscale + align_up((size_t)ntau * 4, 256);
    // the plain float loops get a first bound as well (enlarged by a few units of fp32 rounding: they
    // add the table entries in a rotated order, the bound is computed in table order)
    const bool seed_plain = !is_u4 && !prune && n >= PRUNE_INIT;
    // Few query groups over a large database: the first bound comes from a larger part of the codes.
    // Measured optimum (10^7 .. 10^9 codes, 1 .. 200 queries): about 64 M code evaluations over all
    // queries of the call, at most a thirty-second of the database per query.
    const bool few_groups = !(q8 || u4q) && ngroups < STREAM_GROUPS;   // (the 16-query loops start at 16 groups)
    int64_t seed_codes_f32 = SEED_CODES_STREAM;   // (integer scans use the same count)
    if (few_groups) {
        int64_t want = ((int64_t)64 << 20) / (nq > 0 ? nq : 1);
        if (want > n / 32) want = n / 32;
        if (want > seed_codes_f32) seed_codes_f32 = want;
    }
    const bool wide_ok = opt_int(ctx, PQ_OPT_SCAN_WIDE_SEED, 1) != 0;
    const bool wide_seed = wide_ok && prune && few_groups && tables == 8 && seed_codes_f32 > SEED_SLICE;
    const bool wide_seed_u4 = wide_ok && is_u4 && few_groups && n >= PRUNE_MIN_N && seed_codes_f32 > SEED_SLICE;
    const size_t off_seedhist = prune ? off_qtabs + align_up((size_t)ngroups * 256 * tables * sizeof(uint4), 256) : off_tau0;
    // 16 queries per pass: the 16-bit tables of the second test (64 KB per group) and their scales
    const size_t off_seedref = off_seedhist + align_up(wide_seed ? (size_t)nq * HIST_BINS * 4 : 0, 256);   // (wide first bound: reference of the bins per query)
    const size_t off_qtabs16 = off_seedref + align_up(wide_seed ? (size_t)ntau * 4 : 0, 256);
    const size_t off_pscale16 = off_qtabs16 + (q8 ? (size_t)ngroups * 4096 * sizeof(uint4) : 0);
    const size_t total = prune ? off_pscale16 + (q8 ? align_up((size_t)ntau * 4, 256) : 0)
                               : (wide_seed_u4 ? off_seedhist + (size_t)nq * 4096 * 4 : (seed_plain ? off_poff : off_tau0));
    rc = ws_reserve(ctx, total);
    if (rc) return rc;
    uint8_t *ws = (uint8_t *)ctx->ws;

    TunedArgs a;
    a.codes = codes; a.n = n; a.chunk_codes = chunk_codes; a.head_codes = head_codes; a.head_chunks = head_chunks;
    a.nchunks = (int)nchunks; a.ngroups = ngroups;
    a.nitems = (int)nitems; a.luts = luts; a.nq = nq; a.topk = topk;
    bind_state(a, ws, L);
    a.partial = (uint64_t *)(ws + off_partial);
    a.item_tab = nullptr; a.nitems_dev = nullptr; a.pairs_by_list = nullptr; a.pair_out = nullptr; a.nprobe = 0;

    a.qtabs = nullptr; a.prune_off = nullptr; a.prune_scale = nullptr; a.pair_min = nullptr;
    a.qtabs16 = nullptr; a.prune_scale16 = nullptr;
    float *tau0 = nullptr;
    if (prune) {
        tau0 = (float *)(ws + off_tau0);
        float *poff = (float *)(ws + off_poff), *pscale = (float *)(ws + off_pscale);
        uint4 *qtabs = (uint4 *)(ws + off_qtabs);
        uint4 *qtabs16 = q8 ? (uint4 *)(ws + off_qtabs16) : nullptr;
        float *pscale16 = q8 ? (float *)(ws + off_pscale16) : nullptr;
        if (wide_seed) {
            // Few query groups over a large database: state cleared first, then one sampling pass whose bins every block
            // bounds for itself, then bound, shared state and tables of every group in one launch (three launches before the
            // scan; a pass over the first 4096 codes for the bins' reference, a launch to clear the bins, one to pick the
            // bounds and one to seed the state came on top before: 10^8 codes x 1 query 0.32 -> 0.27 ms per call)
            uint32_t *seed_hist = (uint32_t *)(ws + off_seedhist);
            float *seed_ref = (float *)(ws + off_seedref);
            tuned_init_kernel<<<1024, 256, 0, ctx->stream>>>(a.work_counter, a.tau_key, a.ncand, a.refresh_mark, a.tau_ref, ntau,
                                                             0xff800000u, a.hist, L.nhist, nullptr, nq, 1.f, seed_hist, (size_t)nq * HIST_BINS);
            // (short slices while the launch stays under 2048 blocks, else the slices of the older pass)
            const int slice = (seed_codes_f32 + SEED2_SLICE - 1) / SEED2_SLICE * nq <= 2048 ? SEED2_SLICE : SEED_SLICE;
            const dim3 sgrid((unsigned)((seed_codes_f32 + slice - 1) / slice), (unsigned)nq);
            f32_seed_hist2_kernel<<<sgrid, 1024, 0, ctx->stream>>>(codes, seed_codes_f32, slice, (const float *)luts, topk, seed_hist, seed_ref);
            prune_tables_kernel<8><<<dim3(ngroups, 8), 256, 0, ctx->stream>>>((const float *)luts, tau0, nq, qtabs, poff, pscale, 0.f, nullptr, nullptr,
                                                                             seed_hist, seed_ref, topk, a.tau_key, a.tau_ref);
            PQ_HIP(ctx, hipGetLastError());
        } else {
            // the first bound: smallest histogram edge with k distances among the first codes
            // (batched: 256 codes per result wanted, between 32 768 and 131 072: top-1000 4.60 -> 4.30 ms per step)
            int batch_codes = topk * 256 > SEED_CODES_BATCH ? topk * 256 : SEED_CODES_BATCH;
            if (batch_codes > 4 * SEED_CODES_BATCH) batch_codes = 4 * SEED_CODES_BATCH;
            // fewer queries: more chunks of a query start at once with this bound, and the seed kernel has blocks to spare
            // (2^26 code evaluations per call, at most 262 144 codes: 256 queries 1.39 -> 1.30 ms per step)
            const int by_queries = (1 << 26) / (nq > 0 ? nq : 1) < (1 << 18) ? (1 << 26) / (nq > 0 ? nq : 1) : (1 << 18);
            if (batch_codes < by_queries && (int64_t)by_queries <= n / 16) batch_codes = by_queries;   // (a small part of the database only)
            if ((int64_t)batch_codes > n) batch_codes = (int)n;
            const int first_codes = few_groups ? SEED_CODES_STREAM : batch_codes;
            if (tables == 8) f32_seed_refine_kernel<8><<<(nq + SEED_QPB - 1) / SEED_QPB, 1024, 0, ctx->stream>>>(codes, first_codes, (const float *)luts, topk, true, nq, tau0);
            else f32_seed_refine_kernel<16><<<(nq + SEED_QPB - 1) / SEED_QPB, 1024, 0, ctx->stream>>>(codes, first_codes, (const float *)luts, topk, true, nq, tau0);
            PQ_HIP(ctx, hipGetLastError());
            if (q8) prune_tables_kernel<8, 16><<<dim3(ngroups, 8), 256, 0, ctx->stream>>>((const float *)luts, tau0, nq, qtabs, poff, pscale, PRUNE_RANGE_Q8, qtabs16, pscale16);
            else if (tables == 8) prune_tables_kernel<8><<<dim3(ngroups, 8), 256, 0, ctx->stream>>>((const float *)luts, tau0, nq, qtabs, poff, pscale, 0.f, nullptr, nullptr);
            else prune_tables_kernel<16><<<dim3(ngroups, 8), 256, 0, ctx->stream>>>((const float *)luts, tau0, nq, qtabs, poff, pscale, 0.f, nullptr, nullptr);
            PQ_HIP(ctx, hipGetLastError());
        }
        a.qtabs = qtabs; a.prune_off = poff; a.prune_scale = pscale; a.qtabs16 = qtabs16; a.prune_scale16 = pscale16;
    } else if (seed_plain) {
        tau0 = (float *)(ws + off_tau0);
        rc = launch_qmax_prescan(ctx, codes, n, PQ_CODES_U8, (const float *)luts, nq, cb, 256, PRUNE_INIT, topk, tau0);
        if (rc) return rc;
    }
    if (!wide_seed) {   // (the wide first bound has cleared and seeded the state already)
        uint32_t *seed_hist_u4 = wide_seed_u4 ? (uint32_t *)(ws + off_seedhist) : nullptr;
        tuned_init_kernel<<<1024, 256, 0, ctx->stream>>>(a.work_counter, a.tau_key, a.ncand, a.refresh_mark, a.tau_ref, ntau,
                                                         is_u4 ? 0x7fffu : 0xff800000u, a.hist, L.nhist, tau0, nq,
                                                         seed_plain ? 1.f + 4e-6f : 1.f, seed_hist_u4, wide_seed_u4 ? (size_t)nq * 4096 : 0);
        PQ_HIP(ctx, hipGetLastError());
    }
    if (is_u4 && n >= PRUNE_MIN_N) {
        if (wide_seed_u4) {
            uint32_t *seed_hist = (uint32_t *)(ws + off_seedhist);
            const dim3 sgrid((unsigned)((seed_codes_f32 + SEED_SLICE - 1) / SEED_SLICE), (unsigned)nq);
            u4_seed_hist_kernel<<<sgrid, 1024, 0, ctx->stream>>>(codes, seed_codes_f32, (const uint8_t *)luts, seed_hist);
            u4_seed_pick_kernel<<<nq, 64, 0, ctx->stream>>>(seed_hist, topk, a.tau_key);
        } else {
            // 256 codes per result wanted, between PRUNE_INIT and 262 144 (top-1000: 4.11 -> 3.94 ms per step; twice as many
            // cost the seed kernel more than they save the scan)
            int seed_codes = topk * 256 > PRUNE_INIT ? topk * 256 : PRUNE_INIT;
            if (few_groups) seed_codes = SEED_CODES_STREAM;
            else if (seed_codes > 4 * SEED_CODES_STREAM) seed_codes = 4 * SEED_CODES_STREAM;
            if (!few_groups) {   // (fewer queries: larger sample, as for the float scan)
                const int by_queries = (1 << 26) / (nq > 0 ? nq : 1) < (1 << 18) ? (1 << 26) / (nq > 0 ? nq : 1) : (1 << 18);
                if (seed_codes < by_queries && (int64_t)by_queries <= n / 16) seed_codes = by_queries;
            }
            if ((int64_t)seed_codes > n) seed_codes = (int)n;
            u4_seed_kernel<<<(nq + SEED_QPB - 1) / SEED_QPB, 1024, 0, ctx->stream>>>(codes, seed_codes, (const uint8_t *)luts, topk, nq, a.tau_key);
        }
        PQ_HIP(ctx, hipGetLastError());
    }
    if (ctx->profiling) {
        a.stats = (unsigned long long *)(ws + 8);
        note_scan(ctx, kind, qb, ngroups, a.stats, a.ncand, ntau);
        PQ_HIP(ctx, hipEventRecord(ctx->ev_begin, ctx->stream));
    }
    rc = launch_by_kind(ctx, kind, small, few_groups, a, nblocks);
    if (rc) return rc;
    if (ctx->profiling) {
        PQ_HIP(ctx, hipEventRecord(ctx->ev_end, ctx->stream));
        ctx->ev_valid = 1;
    }
    return launch_merge_filtered(ctx, a.partial, nullptr, (int)nchunks, ngroups, qb, a.tau_key, kpad, nq, topk, nullptr, is_u4,
                                 out_val, out_ids);
}

#endif   // !PQ_TUNED_ITEMS_ONLY

}  // namespace PQ_TUNED_NS
}  // namespace pq
