// Device-side building blocks of the top-k selection used by the scan kernels.
//
// A candidate is one 64-bit key: (ordered value << 32) | id.  Unsigned comparison of keys
// is the total order (value, id) of Alg. 1's heap, so "the k smallest keys" is exactly the
// content of that heap after the scan.  For float values the upper word is the usual
// order-preserving map of IEEE-754 bits to unsigned integers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pq {

constexpr uint64_t KEY_EMPTY = ~0ull;

__device__ __forceinline__ uint32_t f32_to_ord(float f) {
    uint32_t b = __float_as_uint(f);
    return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ __forceinline__ float ord_to_f32(uint32_t o) {
    uint32_t b = o ^ ((o >> 31) ? 0x80000000u : 0xffffffffu);
    return __uint_as_float(b);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }

// number of set bits of `mask` below this lane
__device__ __forceinline__ int mask_prefix(uint64_t mask) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Candidate lists in device scratch are written and read back by different lanes of a wave and,
// when a block merges its lists, by different waves of the same block: never by another block.
// Work-group scope is therefore enough, which keeps the lists in the caches of the block's own CU
// and XCD (device scope would send every access, and every fence, past the L2 to memory).
__device__ __forceinline__ void key_store(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ uint64_t key_load(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// orders the list accesses of the block's waves (stores before, loads after)
__device__ __forceinline__ void list_fence() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); }

// k-th smallest (1-based) of the wave's 64*E keys, by bitwise bisection on the key value:
// the smallest v with count(key <= v) >= k.  Every lane must call it; the result is uniform.
// If fewer than k non-empty keys exist the result is KEY_EMPTY.
template <int E>
__device__ __forceinline__ uint64_t wave_select_kth(const uint64_t (&key)[E], int k) {
    uint64_t v = 0;
    for (int bit = 63; bit >= 0; --bit) {
        const uint64_t trial = v | ((1ull << bit) - 1ull);
        int c = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) c += __popcll(__ballot(key[e] <= trial));
        if (c < k) v |= (1ull << bit);
    }
    return v;
}

// Keep the k smallest of buf[0..cnt) (cnt <= 64*E) in buf[0..min(cnt,k)), in no particular
// order.  Returns a key t with exactly min(cnt,k) keys <= t, at least the k-th smallest key
// (KEY_EMPTY if cnt < k), and updates cnt.  Lists of up to 512 keys are held in registers;
// longer ones are re-read from memory in every bisection step (rare path, few registers).
template <int E>
__device__ __forceinline__ uint64_t wave_compact(uint64_t *buf, int &cnt, int k) {
    const int lane = lane_id();
    list_fence();  // the appends of every lane are visible to the other lanes
    if constexpr (E <= 8) {
        uint64_t key[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int idx = e * 64 + lane;
            key[e] = idx < cnt ? key_load(buf + idx) : KEY_EMPTY;
        }
        const uint64_t kth = wave_select_kth<E>(key, k);
        int base = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const bool keep = key[e] <= kth && key[e] != KEY_EMPTY;
            const uint64_t mask = __ballot(keep);
            if (keep) key_store(buf + base + mask_prefix(mask), key[e]);
            base += __popcll(mask);
        }
        cnt = base;
        return kth;
    } else {
        uint64_t v = 0;
        for (int bit = 63; bit >= 0; --bit) {
            const uint64_t trial = v | ((1ull << bit) - 1ull);
            int c = 0;
#pragma unroll 8
            for (int e = 0; e < E; ++e) {
                const int idx = e * 64 + lane;
                const uint64_t key = idx < cnt ? key_load(buf + idx) : KEY_EMPTY;
                c += __popcll(__ballot(key <= trial));
            }
            if (c == k) { v = trial; break; }   // exactly k keys at or below the trial: good enough
            if (c < k) v |= (1ull << bit);
        }
        // in-place compaction, 64 keys per round: the write position never passes the read position
        int base = 0;
#pragma unroll 4
        for (int e = 0; e < E; ++e) {
            const int idx = e * 64 + lane;
            const uint64_t key = idx < cnt ? key_load(buf + idx) : KEY_EMPTY;
            const bool keep = key <= v && key != KEY_EMPTY;
            const uint64_t mask = __ballot(keep);
            if (keep) key_store(buf + base + mask_prefix(mask), key);
            base += __popcll(mask);
        }
        cnt = base;
        return v;
    }
}

// Append the lanes with `pass` set to buf at position cnt (uniform).  Returns the new count.
__device__ __forceinline__ int wave_append(uint64_t *buf, int cnt, bool pass, uint64_t key) {
    const uint64_t mask = __ballot(pass);
    if (pass) key_store(buf + cnt + mask_prefix(mask), key);
    return cnt + __popcll(mask);
}

// The k-th smallest (k = 1 .. n) of n 32-bit values in LDS, by the whole block (at least 256 threads), by radix
// selection, most significant byte first: four rounds of a 256-bin count over the values that share the bytes
// fixed so far.  `bins`: 256 LDS words, `state`: 2 LDS words.  Every thread gets the value; a few barriers in all.
__device__ inline uint32_t block_kth_smallest_u32(const uint32_t *vals, int n, uint32_t k, uint32_t *bins, uint32_t *state) {
    const int tid = threadIdx.x;
    if (tid == 0) { state[0] = 0u; state[1] = k; }
    for (int pass = 3; pass >= 0; --pass) {
        if (tid < 256) bins[tid] = 0u;
        __syncthreads();
        const int shift = 8 * pass;
        const uint32_t fixed = pass == 3 ? 0u : 0xffffffffu << (shift + 8);   // bytes decided in earlier rounds
        const uint32_t prefix = state[0], want = state[1];
        for (int i = tid; i < n; i += blockDim.x) {
            const uint32_t v = vals[i];
            if ((v & fixed) == prefix) atomicAdd(&bins[(v >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {   // one wave: the byte value whose bin holds the `want`-th value
            const uint32_t h[4] = {bins[4 * tid], bins[4 * tid + 1], bins[4 * tid + 2], bins[4 * tid + 3]};
            const uint32_t tot = h[0] + h[1] + h[2] + h[3];
            uint32_t incl = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t up = __shfl_up(incl, o);
                if (tid >= o) incl += up;
            }
            const uint64_t reach = __ballot(incl >= want);   // never empty: want <= values that share the prefix
            if (reach != 0ull && tid == __builtin_ctzll(reach)) {
                uint32_t cum = incl - tot;
                int b = 4 * tid;
                for (int t = 0; t < 3 && cum + h[t] < want; ++t) { cum += h[t]; ++b; }
                state[0] = prefix | ((uint32_t)b << shift);
                state[1] = want - cum;
            }
        }
        __syncthreads();
    }
    return state[0];
}

// In-LDS bitonic sort (ascending) of n2 keys, n2 a power of two, by the whole block.
__device__ inline void block_bitonic_sort(uint64_t *s, int n2) {
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int i = threadIdx.x; i < (n2 >> 1); i += blockDim.x) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool asc = (lo & size) == 0;
                const uint64_t a = s[lo], b = s[hi];
                if ((a > b) == asc) { s[lo] = b; s[hi] = a; }
            }
        }
    }
    __syncthreads();
}

}  // namespace pq
