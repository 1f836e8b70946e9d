// Shared device-side definitions of libe0m4: the packed weight layout and the
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

// ---- packed weight layout -----------------------------------------------------
// The weight matrix is cut into blocks of 16 rows x 128 k.  One block is what
// one wavefront reads with a single dwordx4 load per lane: lane = q*16 + r owns
// the 16-byte chunk with the 32 codes of row r (of the block), k = 32q .. 32q+31
// (of the block), so a block's codes are 1 KiB contiguous and 1 KiB aligned.
// A row block (16 rows, all of K) is stored as one contiguous run: first the
// codes of its k blocks in order, then the group parameters of its k blocks in
// order, one 32-bit word (scale in the low half, bias in the high half, both
// fp16) per (sub-group, row): 128/G sub-groups x 16 rows per k block.  So
// everything a workgroup that owns 16 output rows needs is one stream, and it
// never shares a cache line with another workgroup.
//
// Inside a chunk, 32-bit word w holds the codes of k = 8w .. 8w+7 (of the
// chunk); inside a word the nibbles are interleaved so that nibble i (bits
// 4i..4i+3) is code 2i and nibble 4+i is code 2i+1: a shift by 6-4i and one
// mask-or then leave two codes sitting in the four highest fraction bits of the
// two fp16 halves of a register.
//
// Rows beyond N and k beyond K inside the last blocks are stored as zero codes
// with zero parameters (they dequantise to 0).
constexpr int kBlockRows = 16;
constexpr int kBlockK = 128;
constexpr int kCodesPerChunk = 32;
constexpr int kBlockCodeBytes = kBlockRows * kBlockK / 2;      // 1024

__host__ __device__ constexpr int block_param_words(int G) { return (kBlockK / G) * kBlockRows; }
__host__ __device__ constexpr int block_bytes(int G) { return kBlockCodeBytes + 4 * block_param_words(G); }
__host__ __device__ inline int64_t row_blocks(int64_t N) { return (N + kBlockRows - 1) / kBlockRows; }
__host__ __device__ inline int64_t k_blocks(int64_t K) { return (K + kBlockK - 1) / kBlockK; }

// Addressing inside the packed buffer, in units of 16 bytes (codes) and 4 bytes (parameter words).
template <int G>
struct PackedLayout {
    static constexpr int kCodePieces = kBlockCodeBytes / 16;                // 64 uint4 per k block
    static constexpr int kParamWords = block_param_words(G);                // per k block
    int64_t nkb;
    __host__ __device__ explicit PackedLayout(int64_t K) : nkb(k_blocks(K)) {}
    // uint4 index of the first chunk of block (rb, kb)
    __host__ __device__ int64_t code_index(int64_t rb, int64_t kb) const
    {
        return rb * nkb * (block_bytes(G) / 16) + kb * kCodePieces;
    }
    // 32-bit word index of the first parameter word of block (rb, kb)
    __host__ __device__ int64_t param_index(int64_t rb, int64_t kb) const
    {
        return rb * nkb * (block_bytes(G) / 4) + nkb * (kBlockCodeBytes / 4) + kb * kParamWords;
    }
    // parameter word of (chunk q, row r) inside a block's parameter words
    __host__ __device__ static constexpr int param_slot(int q, int r) { return (q * kCodesPerChunk / G) * kBlockRows + r; }
};

// bit position of code j (0..7) inside its 32-bit word
__host__ __device__ inline int nibble_shift(int j) { return 4 * ((j >> 1) + ((j & 1) << 2)); }

constexpr uint32_t kFracMask2 = 0x03C003C0u;   // four highest fraction bits of both halves
constexpr uint32_t kExpBits2 = 0x40004000u;    // sign 0, exponent of the binade [2,4), both halves

// The paper's two bitwise operations, applied to two codes at once: pair i of
// a word (codes 2i, 2i+1) becomes two fp16 values 2 + code/8.  `mask` must hold
// kFracMask2; callers keep it in a vector register (see frac_mask_vgpr) so that
// the mask and the OR fuse into one v_and_or_b32 (gfx950 allows only one
// scalar/constant operand per VOP3 instruction).
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

__device__ inline half_t param_scale(uint32_t word) { return __builtin_bit_cast(half_t, (uint16_t)(word & 0xFFFFu)); }
__device__ inline half_t param_bias(uint32_t word) { return __builtin_bit_cast(half_t, (uint16_t)(word >> 16)); }

}  // namespace e0m4
