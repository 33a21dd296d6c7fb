// Byte shuffles shared by the scan kernels that keep their tables in LDS rows of 256 bytes
// (one row per code-byte value, 16 slots of 16 bytes): every lane walks the slots in an order
// rotated by its lane number, so the 16 lanes that the LDS serves together always read 16
// different slots, and rotates the bytes of its code to match.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pq {

// rotate the bytes of a 64-bit code right by r bytes (r in 0..7): byte s of the result is
// byte (s + r) & 7 of the input
__device__ __forceinline__ void rot8(uint32_t &lo, uint32_t &hi, bool swap, uint32_t sh) {
    const uint32_t a = swap ? hi : lo, b = swap ? lo : hi;
    lo = __builtin_amdgcn_alignbyte(b, a, sh);
    hi = __builtin_amdgcn_alignbyte(a, b, sh);
}

// rotate the bytes of a 128-bit code right by r bytes (r in 0..15)
__device__ __forceinline__ void rot16(uint32_t (&w)[4], uint32_t r) {
    if (r & 8u) { uint32_t t = w[0]; w[0] = w[2]; w[2] = t; t = w[1]; w[1] = w[3]; w[3] = t; }
    if (r & 4u) { const uint32_t t = w[0]; w[0] = w[1]; w[1] = w[2]; w[2] = w[3]; w[3] = t; }
    const uint32_t sh = r & 3u;
    const uint32_t a = w[0], b = w[1], c = w[2], d = w[3];
    w[0] = __builtin_amdgcn_alignbyte(b, a, sh);
    w[1] = __builtin_amdgcn_alignbyte(c, b, sh);
    w[2] = __builtin_amdgcn_alignbyte(d, c, sh);
    w[3] = __builtin_amdgcn_alignbyte(a, d, sh);
}

// LDS byte offset of the lookup for byte `pos` of `word`: (code byte << 8) | slot offset.
// `bases` holds the slot offsets (slot * 16, below 256) of four consecutive steps.
template <int POS>
__device__ __forceinline__ uint32_t lut_offset(uint32_t word, uint32_t bases) {
    // result byte 0 <- bases byte POS, byte 1 <- word byte POS, bytes 2 and 3 <- 0
    constexpr uint32_t sel = 0x0c0c0000u | ((4u + POS) << 8) | (uint32_t)POS;
    return __builtin_amdgcn_perm(word, bases, sel);
}

}  // namespace pq
