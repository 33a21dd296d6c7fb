// Scan step of the IVFADC search (Section 2.3.3, Step 3; Alg. 1 `scan`/`adc` on the codes of one inverted
// list) for SHORT lists.
//
// Most inverted lists of a large index are short (with 2^16 cells over 10^9 vectors and skewed cell sizes
// half of them hold under 3000 codes), and the thesis notes that switching cells has a visible cost of its
// own at about 1000 codes per cell (Section 5.3).  On this machine the cost of a short list is a chain of
// dependent memory round trips (which item, which (query, list) pairs, their tables, the first codes),
// not the additions.  The large persistent scan kernel spends 15 us per work item on it with two blocks
// of 8 waves per compute unit.  This kernel is the same scan for lists of at most a few thousand codes,
// shaped for that chain instead of for streaming:
//   - blocks of 4 waves that need under 40 KB of LDS, four to a compute unit: four chains in flight;
//   - one work item = one list x up to 4 of the (query, list) pairs that probe it, described by one
//     32-byte record; items are dealt to blocks in a fixed stride (no work counter), and the record of the
//     item after next and the bounds and result places of the next item are requested while the current
//     one is scanned;
//   - the four pairs' float tables are staged once (entry (byte b, table j) of all four pairs = one 16-byte
//     LDS slot, slots of a byte value side by side); every lane walks the tables in an order rotated by its
//     lane number, so the 16 lanes the LDS serves together read 8 different tables, and lanes that share a
//     table collide only if their bytes have equal parity;
//   - candidates (keys (distance, row) at or below the query's bound) go to a small LDS list per pair; at
//     the end of the item the list is written to the pair's result list, sorted first if it is long enough
//     to yield a bound (k keys) or exceeds the result list.  If more candidates arrive than the list holds
//     (loose or missing bound), the k-th smallest of those held becomes the pair's bound and the list is
//     scanned again: every pass shrinks the candidate set, the last one fits.
// Results have the format of the large kernel (lists of KPAD keys, packed, padded with KEY_EMPTY) and are
// merged with its results by merge_filtered_kernel.  Float sums add the 8 entries in the lane's rotated
// order (within (m - 1) * 2^-24 relative of any other order).
#include "pq_internal.h"
#include "scan_common.h"
#include "topk_device.h"
#include "lds_walk.h"

namespace pq {

constexpr int SH_THREADS = 256;
constexpr int SH_QS = IVF_SHORT_QS;     // (query, list) pairs per item
constexpr int SH_CAP = 160;             // candidate keys held per pair (more than k = 128 of them, see the rescan)
constexpr int SH_SORT = 256;            // SH_CAP padded to a power of two
constexpr int SH_KPAD = 128;
constexpr int SH_BATCH = 4;             // codes of a thread on their way at a time

struct __align__(16) ShortSmem {
    float4 lut[256 * 8];                    // slot (b, j) at b * 8 + j: entry b of table j for the 4 pairs
    unsigned long long cand[SH_QS][SH_CAP];
    unsigned long long sortbuf[SH_SORT];
    unsigned long long bkey[SH_QS];         // candidates satisfy key <= bkey
    IvfShortItem rec;                       // the item being scanned
    uint32_t out_idx[SH_QS];                // result list of each pair
    int cnt[SH_QS];
};
static_assert(sizeof(ShortSmem) <= 40 * 1024, "four blocks share the 160 KB of a compute unit");

// In-LDS bitonic sort of SH_SORT keys by the block's 256 threads (ascending).
__device__ __forceinline__ void short_sort(unsigned long long *s) {
    for (int size = 2; size <= SH_SORT; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            const int i = threadIdx.x;
            if (i < SH_SORT / 2) {
                const int lo = 2 * i - (i & (stride - 1)), hi = lo + stride;
                const bool asc = (lo & size) == 0;
                const unsigned long long a = s[lo], b = s[hi];
                if ((a > b) == asc) { s[lo] = b; s[hi] = a; }
            }
        }
    __syncthreads();
}

#ifdef PQ_SCAN_TIMING
__device__ unsigned long long g_short_ticks[8];
#define SH_TICK(phase) do { const unsigned long long now__ = __builtin_amdgcn_s_memtime(); tick_acc[phase] += now__ - tick_last; tick_last = now__; } while (0)
#else
#define SH_TICK(phase) do { } while (0)
#endif

__global__ __launch_bounds__(SH_THREADS, 4) void ivf_short_scan_kernel(const uint8_t *__restrict__ codes,
                                                                    const float *__restrict__ luts,
                                                                    const IvfShortItem *__restrict__ items,
                                                                    const uint32_t *__restrict__ nitems_dev,
                                                                    const uint32_t *__restrict__ pair_out, int nprobe,
                                                                    int topk, unsigned long long *tau_key,
                                                                    uint64_t *partial) {
    __shared__ ShortSmem sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int nitems = (int)*nitems_dev;
    const int stride = (int)gridDim.x;

    // Records and per-pair state travel in the registers of threads 0 .. SH_QS-1 (thread s: pair slot s):
    //   rec2: record of the item after next; rec1 + out1/key1: next item, complete when its turn comes.
    IvfShortItem rec1, rec2;
    uint32_t out1 = 0;
    unsigned long long key1 = 0ull;
    auto load_rec = [&](int item, IvfShortItem &r) {
        if (item < nitems) r = items[item];
        else r.ncodes_skip_slots = 0u;   // (nslots = 0 marks "no item")
    };
    auto load_pair_state = [&](const IvfShortItem &r, uint32_t &out, unsigned long long &key) {
        const int nslots = (int)(r.ncodes_skip_slots >> 28);
        if (tid < nslots) {
            const int pair = tid == 0 ? r.pair[0] : tid == 1 ? r.pair[1] : tid == 2 ? r.pair[2] : r.pair[3];
            out = pair_out[pair];
            key = __hip_atomic_load(&tau_key[pair / nprobe], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    int item = (int)blockIdx.x;
    if (tid < SH_QS) {
        load_rec(item, rec1);
        load_rec(item + stride, rec2);
        load_pair_state(rec1, out1, key1);
    }

#ifdef PQ_SCAN_TIMING
    unsigned long long tick_acc[5] = {0, 0, 0, 0, 0}, tick_last = __builtin_amdgcn_s_memtime();
#endif
    for (; item < nitems; item += stride) {
        // ---- the item: record and per-pair words come from the prefetching threads
        if (tid < SH_QS) {
            if (tid == 0) sm.rec = rec1;
            sm.out_idx[tid] = out1;
            sm.bkey[tid] = tid < (int)(rec1.ncodes_skip_slots >> 28) ? key1 : 0ull;   // empty slots: nothing qualifies
            sm.cnt[tid] = 0;
            // shift the pipeline: the next item's pair state and the record after it are requested now and have the
            // whole item to arrive
            rec1 = rec2;
            load_pair_state(rec1, out1, key1);
            load_rec(item + 2 * stride, rec2);
        }
        __syncthreads();
        const IvfShortItem rec = sm.rec;
        const int nslots = (int)(rec.ncodes_skip_slots >> 28);
        const int skip = (int)((rec.ncodes_skip_slots >> 24) & 15u);
        const int ncodes = (int)(rec.ncodes_skip_slots & 0xffffffu);
        SH_TICK(0);
        // the first codes are requested before the tables (both depend on the record only)
        const uint8_t *base = codes + (size_t)rec.code_begin * 8;
        const uint32_t row0 = rec.code_begin;
        auto load_batch = [&](int i0, uint2 (&c)[SH_BATCH]) {
#pragma unroll
            for (int u = 0; u < SH_BATCH; ++u) {
                const int i = i0 + u * SH_THREADS;
                c[u] = i < ncodes ? *reinterpret_cast<const uint2 *>(base + (size_t)i * 8) : make_uint2(0, 0);
            }
        };
        uint2 cur[SH_BATCH], nxt[SH_BATCH];
        load_batch(skip + tid, cur);
        // ---- stage the tables of the item's pairs: thread e takes entries e, e + 256, ... of every pair
        {
            const float *lp[SH_QS];
#pragma unroll
            for (int s = 0; s < SH_QS; ++s) lp[s] = s < nslots ? luts + (size_t)rec.pair[s] * 2048 : nullptr;
            float v[8][SH_QS];
#pragma unroll
            for (int r = 0; r < 8; ++r)
#pragma unroll
                for (int s = 0; s < SH_QS; ++s) v[r][s] = lp[s] ? lp[s][r * 256 + tid] : __builtin_inff();
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                // entry e = r * 256 + tid is entry b = tid of table j = r
                sm.lut[tid * 8 + r] = make_float4(v[r][0], v[r][1], v[r][2], v[r][3]);
            }
        }
        __syncthreads();
        SH_TICK(1);

        // the lane's walk: at step st it reads table (rot + st) & 7; its code is rotated by rot bytes so that the byte for
        // step st sits at position st
        const uint32_t rot = (uint32_t)lane & 7u;
        uint32_t tbase[8];
#pragma unroll
        for (int st = 0; st < 8; ++st) tbase[st] = ((rot + (uint32_t)st) & 7u) << 4;
        const char *lut_bytes = reinterpret_cast<const char *>(sm.lut);
        for (int pass = 0;; ++pass) {   // (one pass; more only if a candidate list overflowed)
            float bval[SH_QS];
#pragma unroll
            for (int s = 0; s < SH_QS; ++s) bval[s] = ord_to_f32((uint32_t)(sm.bkey[s] >> 32));
            if (pass > 0) load_batch(skip + tid, cur);
            // batches of SH_BATCH codes per thread: the next batch is requested before the current one is added up
            for (int i0 = skip + tid; i0 < ncodes; i0 += SH_BATCH * SH_THREADS) {
                load_batch(i0 + SH_BATCH * SH_THREADS, nxt);
#pragma unroll
                for (int u = 0; u < SH_BATCH; ++u) {
                    const int i = i0 + u * SH_THREADS;
                    if (i >= ncodes) break;
                    uint32_t lo = cur[u].x, hi = cur[u].y;
                    rot8(lo, hi, (rot & 4u) != 0u, rot & 3u);
                    float4 e[8];
#pragma unroll
                    for (int st = 0; st < 8; ++st) {
                        const uint32_t b = ((st < 4 ? lo : hi) >> (8 * (st & 3))) & 255u;
                        e[st] = *reinterpret_cast<const float4 *>(lut_bytes + ((b << 7) + tbase[st]));   // slot (b, table) at b * 128 + table * 16
                    }
                    float d[SH_QS] = {e[0].x, e[0].y, e[0].z, e[0].w};
#pragma unroll
                    for (int st = 1; st < 8; ++st) { d[0] += e[st].x; d[1] += e[st].y; d[2] += e[st].z; d[3] += e[st].w; }
                    // (never true for empty slots: their bound is the smallest key)
                    if ((d[0] <= bval[0]) | (d[1] <= bval[1]) | (d[2] <= bval[2]) | (d[3] <= bval[3])) {
#pragma unroll
                        for (int s = 0; s < SH_QS; ++s) {
                            if (d[s] <= bval[s]) {
                                const unsigned long long key = ((unsigned long long)f32_to_ord(d[s]) << 32) | (row0 + (uint32_t)i);
                                if (key <= sm.bkey[s]) {
                                    const int at = atomicAdd(&sm.cnt[s], 1);
                                    if (at < SH_CAP) sm.cand[s][at] = key;
                                }
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < SH_BATCH; ++u) cur[u] = nxt[u];
            }
            __syncthreads();
            SH_TICK(2);
            // a list that overflowed: the k-th smallest of the keys held bounds the k-th smallest of the item; scan again
            bool again = false;
            for (int s = 0; s < nslots; ++s) {
                if (sm.cnt[s] <= SH_CAP) continue;   // (uniform: LDS value read after the barrier)
                again = true;
                sm.sortbuf[tid] = tid < SH_CAP ? sm.cand[s][tid] : KEY_EMPTY;
                short_sort(sm.sortbuf);
                if (tid == 0) {
                    const unsigned long long kth = sm.sortbuf[topk - 1];
                    sm.bkey[s] = kth;   // (below the old bound: every key held was at or below it)
                    atomicMin(&tau_key[sm.rec.pair[s] / nprobe], kth);
                }
                __syncthreads();   // (the sorted keys have been read before the next pair's are written over them)
            }
            if (!again) break;
            __syncthreads();
            if (tid < SH_QS) sm.cnt[tid] = 0;
            __syncthreads();
        }

        SH_TICK(3);
        // ---- results: the pair's keys to its result list (sorted if that yields a bound or the list is too long)
        for (int s = 0; s < nslots; ++s) {
            const int c = sm.cnt[s];
            uint64_t *out = partial + (size_t)sm.out_idx[s] * SH_KPAD;
            if (c >= topk || c > SH_KPAD) {
                sm.sortbuf[tid] = tid < c ? sm.cand[s][tid] : KEY_EMPTY;
                short_sort(sm.sortbuf);
                if (tid < SH_KPAD) out[tid] = sm.sortbuf[tid];
                if (tid == 0 && c >= topk) atomicMin(&tau_key[sm.rec.pair[s] / nprobe], sm.sortbuf[topk - 1]);
                __syncthreads();
            } else if (tid < SH_KPAD) {
                out[tid] = tid < c ? sm.cand[s][tid] : KEY_EMPTY;
            }
        }
        __syncthreads();   // the lists and tables are free for the next item
        SH_TICK(4);
    }
#ifdef PQ_SCAN_TIMING
    if (lane == 0) for (int i = 0; i < 5; ++i) atomicAdd(&g_short_ticks[i], tick_acc[i]);
#endif
}

int launch_ivf_short_scan(pq_ctx *ctx, const uint8_t *codes, const float *luts, const IvfShortItem *items,
                          const uint32_t *nitems_dev, const uint32_t *pair_out, int nprobe, int topk,
                          unsigned long long *tau_key, uint64_t *partial) {
    if (topk > SH_KPAD) return fail(ctx, PQ_EUNSUPPORTED, "ivf short scan: topk above %d", SH_KPAD);
    // four blocks per compute unit; items are dealt in a stride of the grid, longest lists first
    ivf_short_scan_kernel<<<ctx->num_cu * 4, SH_THREADS, 0, ctx->stream>>>(codes, luts, items, nitems_dev, pair_out, nprobe,
                                                                          topk, tau_key, partial);
    PQ_HIP(ctx, hipGetLastError());
#ifdef PQ_SCAN_TIMING
    {
        unsigned long long t[8] = {0};
        PQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
        PQ_HIP(ctx, hipMemcpyFromSymbol(t, HIP_SYMBOL(g_short_ticks), sizeof(t)));
        fprintf(stderr, "short lists (wave cycles x 1e6): top %.1f stage %.1f scan %.1f rescan %.1f output %.1f\n", t[0] / 1e6, t[1] / 1e6,
                t[2] / 1e6, t[3] / 1e6, t[4] / 1e6);
        unsigned long long z[8] = {0};
        PQ_HIP(ctx, hipMemcpyToSymbol(HIP_SYMBOL(g_short_ticks), z, sizeof(z)));
    }
#endif
    return PQ_OK;
}

}  // namespace pq
