// Declarations shared by the scan kernels: value traits, per-wave selection state, launch
// arguments of the tuned kernels and the host-side launchers.
#pragma once
#include <stdlib.h>

#include "pq_internal.h"
#include "topk_device.h"

namespace pq {

// The tuned scan kernels are built twice (scan_tuned.hip, scan_items_w8.hip): blocks of 16 waves, one
// per CU, for flat scans, and blocks of 8 waves, two per CU, for the short work items of inverted
// lists, where one block's item set-up runs while the other block scans.  Each build lives in its
// own namespace (w16, w8).
#ifndef PQ_TUNED_WAVES
#define PQ_TUNED_WAVES 16
#endif
constexpr int TUNED_WAVES = PQ_TUNED_WAVES;
constexpr int TUNED_THREADS = TUNED_WAVES * 64;
constexpr int HIST_BITS = 12;
constexpr int HIST_BINS = 1 << HIST_BITS;
constexpr int HIST_SHIFT = 14;             // float path: bin width in units of the ordered value
constexpr uint32_t TAU_REF_UNSET = 0xffffffffu;

// One work item of the IVF search: a chunk of one inverted list for up to QB of the queries
// that probe the list.
struct IvfItem {
    uint32_t code_begin;   // first row of the chunk, rounded down to a 16-byte boundary
    uint32_t ncodes;       // rows from code_begin to the end of the chunk
    uint32_t pair_pos;     // position in pairs_by_list of the item's first (query, list) pair
    uint32_t skip_slots_chunk;   // bits 0-7: rows at the front that belong to the previous list,
                                 // bits 8-15: number of pairs (slots), bits 16-31: chunk index in the list
};

// IVF search with Quick ADC (ivf_quick_kernels.hip): the query-wide qmax, the 8-bit tables of every pair, the integer
// scan of the work items to the kprime candidates of every (pair, chunk) and their float rerank into the pair's
// first result list; tau_key [nq] receives a bound of each query's result for the merge that follows.
int launch_ivf_quick(pq_ctx *ctx, const uint8_t *codes, const int64_t *list_offsets, const int32_t *probes,
                     const float *luts, int nq, int nprobe, int init, int kprime, int topk, float *qmax_pair,
                     uint8_t *qluts, const IvfItem *items, const uint32_t *nitems_dev, const int32_t *pairs_by_list,
                     const uint32_t *pair_out, const uint32_t *nc_arr, uint64_t *partial, unsigned long long *tau_key,
                     uint32_t *saved_rows, int64_t max_item_rows);
// bytes of `saved_rows` (rows that the counting pass of a work item hands to its collecting pass, per wave) when no
// work item has more than max_item_rows rows
size_t ivf_quick_saved_bytes(const pq_ctx *ctx, int64_t max_item_rows);

// One work item of the scan of short inverted lists (ivf_short_kernels.hip): a whole list for up to
// IVF_SHORT_QS of the (query, list) pairs that probe it.  32 bytes.
constexpr int IVF_SHORT_QS = 4;
struct __align__(16) IvfShortItem {
    uint32_t code_begin;          // first row, rounded down to a 16-byte boundary
    uint32_t ncodes_skip_slots;   // bits 0-23: rows from code_begin to the end of the list, 24-27: rows at the front that
                                  // belong to the previous list, 28-31: pairs in use (0: no item)
    int32_t pair[IVF_SHORT_QS];   // pair = query * nprobe + rank
    uint32_t pad[2];
};
int launch_ivf_short_scan(pq_ctx *ctx, const uint8_t *codes, const float *luts, const IvfShortItem *items,
                          const uint32_t *nitems_dev, const uint32_t *pair_out, int nprobe, int topk,
                          unsigned long long *tau_key, uint64_t *partial);

struct TunedArgs {
    const uint8_t *codes;
    int64_t n;
    int64_t chunk_codes;     // multiple of the block tile
    int64_t head_codes;      // flat scans: the first head_chunks chunks are this short (a first round of items that
    int head_chunks;         // leaves good bounds behind); the other chunks follow them and have chunk_codes codes each
    int nchunks;
    int ngroups;
    int nitems;              // nchunks * ngroups, item = chunk * ngroups + group
    const void *luts;        // [nq][m][k] f32 or u8
    int nq;
    int topk;
    uint32_t *work_counter;  // next item to hand out
    unsigned long long *stats;   // measurement aid (nullptr unless profiling is on): [0] lanes parked for the insert path
    unsigned long long *tau_key;   // [ngroups*QB] best bound known per query, a whole key (ordered value << 32 | row): at least k
                                   // keys are at or below it.  A bound on the value alone is stored with the last row
                                   // (0xffffffff).  Values cannot separate codes that tie at the k-th value; their rows can.
    uint32_t *ncand;         // [ngroups*QB] number of insert events per query
    uint32_t *refresh_mark;  // [ngroups*QB] value of ncand when the histogram was last evaluated
    uint32_t *tau_ref;       // [ngroups*QB] reference value of the histogram bins (float path), UNSET at first
    uint32_t *hist;          // [ngroups*QB][HIST_BINS] values of the candidates inserted
    uint64_t *scratch;       // [nblocks][TUNED_WAVES][QB][CAP]
    uint64_t *partial;       // [nitems][QB][KPAD]; IVF: [number of (pair, chunk) lists][KPAD]
    // IVF mode (item_tab != nullptr): items come from a table, every slot has its own tables
    const IvfItem *item_tab;
    const uint32_t *nitems_dev;      // number of items, computed on the device
    const int32_t *pairs_by_list;    // pair = query * nprobe + rank, grouped by list
    const uint32_t *pair_out;        // [npairs] index of the pair's first output list
    int nprobe;
    // pruned float scan: 16-bit tables in slot order [group][entry][table] (8 queries x u16 each),
    // and per query the sum of the table minima and the scale of the 16-bit tables
    const uint4 *qtabs;
    const float *prune_off;
    const float *prune_scale;
    // pruned float scan of inverted lists: offsets and scales per (query, list) pair (prune_off and
    // prune_scale are indexed by pair; a negative scale marks a pair no code of which can enter the
    // result), and the minima of the pair's tables, from which the 16-bit entries are formed while
    // the item's tables are staged
    const float *pair_min;       // [npairs][tables]
    // 16 queries per pass (8-bit tables in qtabs): the 16-bit tables of the same queries, [group][entry][table][2]
    // (two 16-byte halves of 8 queries each), for the second test of the insert path, and their scale per query
    const uint4 *qtabs16;
    const float *prune_scale16;
};

int launch_merge_topk(pq_ctx *ctx, const uint64_t *partial, int nchunks, int ngroups, int qb, int kpad, int nq,
                      int topk, bool val_u32, void *out_val, int64_t *out_ids);
// merge of the per-query result lists of a scan that leaves a final bound per query in tau_key
// (see merge_filtered_kernel); any number of lists
int launch_merge_filtered(pq_ctx *ctx, const uint64_t *partial, const uint32_t *qlist_off, int nchunks, int ngroups, int qb,
                          const unsigned long long *tau_key, int kpad, int nq, int topk, const int64_t *ids, bool val_u32,
                          void *out_val, int64_t *out_ids);
// IVF: run the persistent scan kernel over a table of work items (see IvfItem).  `state` is a
// caller-provided device region of tuned_state_bytes() bytes holding the per-query bounds,
// histograms and the per-block candidate scratch; tau0 (optional, [nq]) seeds the per-query bounds
// (+inf: none); *tau_key_out receives the per-query bounds.
namespace w16 {
size_t tuned_state_bytes(int kind, int nq, int topk, int num_cu);
int launch_scan_items(pq_ctx *ctx, int kind, const float *pair_min, const float *pair_off, const float *pair_scale,
                      const uint8_t *codes, const float *luts, int nq, int nprobe, int topk,
                      const IvfItem *items, const uint32_t *nitems_dev, const int32_t *pairs_by_list,
                      const uint32_t *pair_out, uint64_t *partial, uint8_t *state, size_t state_bytes,
                      const float *tau0, unsigned long long **tau_key_out);
int launch_scan_tuned(pq_ctx *ctx, int kind, const uint8_t *codes, int64_t n, const void *luts, int nq, int topk,
                      void *out_val, int64_t *out_ids);
}  // namespace w16
namespace w8 {   // work items only, results of up to 128
size_t tuned_state_bytes(int kind, int nq, int topk, int num_cu);
int launch_scan_items(pq_ctx *ctx, int kind, const float *pair_min, const float *pair_off, const float *pair_scale,
                      const uint8_t *codes, const float *luts, int nq, int nprobe, int topk,
                      const IvfItem *items, const uint32_t *nitems_dev, const int32_t *pairs_by_list,
                      const uint32_t *pair_out, uint64_t *partial, uint8_t *state, size_t state_bytes,
                      const float *tau0, unsigned long long **tau_key_out);
}  // namespace w8

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

// smallest histogram bin b with count(bins <= b) >= k, or HIST_BINS if fewer than k counted; for one wave
// (all 64 lanes); `hist` (HIST_BINS words, 16-byte aligned) in device memory or LDS
__device__ __forceinline__ int hist_threshold(const uint32_t *hist, int k) {
    const int lane = lane_id();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    const uint4 *h4 = reinterpret_cast<const uint4 *>(hist) + lane * (HIST_BINS / 64 / 4);
    uint32_t tot = 0;
#pragma unroll 4
    for (int i = 0; i < HIST_BINS / 64 / 4; ++i) {
        const uint4 v = h4[i];
        tot += v.x + v.y + v.z + v.w;
    }
    uint32_t incl = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    const uint64_t reach = __ballot(incl >= (uint32_t)k);
    if (reach == 0ull) return HIST_BINS;
    const int first = __builtin_ctzll(reach);
    // every lane locates the crossing inside its own 64 bins; only lane `first` has a meaningful need
    const uint32_t need = (uint32_t)k - (incl - tot);
    uint32_t cum = 0;
    int bin = HIST_BINS;
#pragma unroll 2
    for (int i = 0; i < HIST_BINS / 64 / 4; ++i) {
        const uint4 v = h4[i];
        const uint32_t e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            cum += e[t];
            if (bin == HIST_BINS && cum >= need) bin = lane * (HIST_BINS / 64) + i * 4 + t;
        }
    }
    return __shfl(bin, first);
}


}  // namespace pq
