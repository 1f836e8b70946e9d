// Shared device-side definitions of libe0m4: the packed code layout and the
// in-register dequantisation of E0M4 codes (paper: section "E0M4 FP4
// quantization", dequantization formula).  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace e0m4 {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---- packed code layout -----------------------------------------------------
// Rows are taken in blocks of 64 (one row per lane of a wavefront), K in chunks
// of 32 codes = 16 bytes = one dwordx4 load per lane.  Chunk (rb, q) of row r
// (r = n % 64, rb = n / 64, q = k / 32) lives at byte offset
//     ((rb * (K/32) + q) * 64 + r) * 16,
// so the 64 lanes of a wavefront read 1 KiB contiguous, and all chunks of one
// row block are contiguous along K.  Inside a chunk, 32-bit word w holds the
// codes of k = 32q + 8w .. +7; inside a word the nibbles are interleaved so
// that nibble i (bits 4i..4i+3) is code k0+2i and nibble 4+i is code k0+2i+1:
// a shift by 6-4i and one mask then leave two codes sitting in the four
// highest fraction bits of the two fp16 halves of a register.
constexpr int kRowsPerBlock = 64;
constexpr int kCodesPerChunk = 32;
constexpr int kChunkBytes = 16;

__host__ __device__ inline int64_t padded_rows(int64_t N) { return (N + kRowsPerBlock - 1) / kRowsPerBlock * kRowsPerBlock; }

// bit position of code j (0..7) inside its 32-bit word
__host__ __device__ inline int nibble_shift(int j) { return 4 * ((j >> 1) + ((j & 1) << 2)); }

constexpr uint32_t kFracMask2 = 0x03C003C0u;   // four highest fraction bits of both halves
constexpr uint32_t kExpBits2 = 0x40004000u;    // sign 0, exponent of the binade [2,4), both halves

// The paper's two bitwise operations, applied to two codes at once: pair i of
// a word (codes k0+2i, k0+2i+1) becomes two fp16 values 2 + code/8.  `mask`
// must hold kFracMask2; callers keep it in a vector register (see
// frac_mask_vgpr) so that the mask and the OR fuse into one v_and_or_b32
// (gfx950 allows only one scalar/constant operand per VOP3 instruction).
template <int I>
__device__ inline uint32_t w1_pair_bits(uint32_t word, uint32_t mask)
{
    static_assert(I >= 0 && I < 4, "pair index");
    uint32_t s;
    if (I == 0) s = word << 6;
    else if (I == 1) s = word << 2;
    else if (I == 2) s = word >> 2;
    else s = word >> 6;
    return (s & mask) | kExpBits2;
}

template <int I>
__device__ inline half2_t w1_pair(uint32_t word, uint32_t mask)
{
    return __builtin_bit_cast(half2_t, w1_pair_bits<I>(word, mask));
}

// kFracMask2 in a vector register the optimiser cannot fold back into a literal.
__device__ inline uint32_t frac_mask_vgpr()
{
    uint32_t m = kFracMask2;
    asm volatile("" : "+v"(m));
    return m;
}

}  // namespace e0m4
