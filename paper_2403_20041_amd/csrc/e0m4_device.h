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
// chunk) as four pairs (2i, 2i+1).  The two codes of a pair sit 16 bits apart,
// so that after at most one shift or rotate they occupy fraction bits of the
// two fp16 halves of a register.  Bit position of the low bit of each code:
//     pair 0: 6 and 22    pair 1: 2 and 18    pair 2: 10 and 26
//     pair 3: 14 and 30 (the second code wraps around: bits 30, 31, 0, 1)
// Pair 0 already lies in the four highest fraction bits (9..6 and 25..22);
// pair 1 lies in fraction bits 5..2.  Rotating the word right by 8 brings
// pair 3 to 9..6 and pair 2 to 5..2.  A code in bits 9..6 of a half with the
// exponent of [2,4) reads 2 + code/8; in bits 5..2 it reads 2 + code/128.
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

// bit position of the low bit of code j (0..7) inside its 32-bit word; code 7 wraps (see above)
__host__ __device__ inline int nibble_shift(int j)
{
    const int pair_pos[4] = {6, 2, 10, 14};
    return pair_pos[j >> 1] + ((j & 1) << 4);
}
__host__ __device__ inline uint32_t rotl32(uint32_t v, int n) { return n ? (v << n) | (v >> (32 - n)) : v; }
__host__ __device__ inline uint32_t rotr32(uint32_t v, int n) { return n ? (v >> n) | (v << (32 - n)) : v; }
// a word with code c at position j, and the code at position j of a word
__host__ __device__ inline uint32_t place_code(uint32_t c, int j) { return rotl32(c & 15u, nibble_shift(j)); }
__host__ __device__ inline uint32_t extract_code(uint32_t word, int j) { return rotr32(word, nibble_shift(j)) & 15u; }

constexpr uint32_t kFracMask2 = 0x03C003C0u;   // four highest fraction bits of both halves
constexpr uint32_t kFracMaskLow2 = 0x003C003Cu;    // fraction bits 5..2 of both halves
constexpr uint32_t kFrac8Mask2 = 0x03FC03FCu;  // eight highest fraction bits of both halves (8-bit format)
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
    if (I == 0) s = word;
    else if (I == 1) s = word << 4;
    else if (I == 2) s = word >> 4;
    else s = __builtin_amdgcn_alignbit(word, word, 8);      // rotate right by 8
    return (s & mask) | kExpBits2;
}

template <int I>
__device__ inline half2_t w1_pair(uint32_t word, uint32_t mask)
{
    return __builtin_bit_cast(half2_t, w1_pair_bits<I>(word, mask));
}

// All four pairs of a word with one rotate: p[0] and p[3] read 2 + code/8, p[1] and p[2] read
// 2 + code/128 (see the layout above).  mask_hi holds kFracMask2, mask_lo kFracMaskLow2, both in
// vector registers.  For dot products: sum x*(2 + c/8) over the codes of pairs 1 and 2 equals
// 16 * sum x*(2 + c/128) - 30 * sum x.
__device__ inline void w1_pairs_mixed(uint32_t word, uint32_t mask_hi, uint32_t mask_lo, half2_t (&p)[4])
{
    const uint32_t t = __builtin_amdgcn_alignbit(word, word, 8);
    p[0] = __builtin_bit_cast(half2_t, (word & mask_hi) | kExpBits2);
    p[1] = __builtin_bit_cast(half2_t, (word & mask_lo) | kExpBits2);
    p[2] = __builtin_bit_cast(half2_t, (t & mask_lo) | kExpBits2);
    p[3] = __builtin_bit_cast(half2_t, (t & mask_hi) | kExpBits2);
}

// kFracMask2 in a vector register the optimiser cannot fold back into a literal.
__device__ inline uint32_t frac_mask_vgpr()
{
    uint32_t m = kFracMask2;
    asm volatile("" : "+v"(m));
    return m;
}

__device__ inline uint32_t frac_mask_low_vgpr()
{
    uint32_t m = kFracMaskLow2;
    asm volatile("" : "+v"(m));
    return m;
}

// Buffer resource over [p, p + 2 GiB): raw (stride 0), 32-bit data format word of gfx9-class targets.
// p must be wavefront-uniform; passing its halves through readfirstlane pins the resource to scalar
// registers (otherwise every buffer load is wrapped in a per-lane "waterfall" loop).
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p)
{
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    void* q = reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
    return __builtin_amdgcn_make_buffer_rsrc(q, 0, 0x7fffffff, 0x00020000);
}

// Operators folded into the decode kernels (e0m4_matmul_fused; paper: section "Operator and lagging
// optimizations", fusion of rms-norm and of element-wise operators into their neighbours):
//   gamma    : the rows of X are rms-normalised while they are staged (x * rsqrt(mean x^2 + eps) * gamma,
//              rounded to fp16 as the stand-alone operator's output would be);
//   swiglu   : weight row j (gate) is paired with row N/2 + j (up) and Y[m, j] = silu(gate) * up; a
//              workgroup then owns pairs of row blocks, slot 2p the gate block and slot 2p + 1 the up block
//              of pair p, `half_bytes` apart in the packed buffer;
//   residual : added to the result before its one rounding.
struct GemvFusion {
    const half_t* gamma;
    const half_t* residual;
    float eps;
    int swiglu;
    uint32_t half_bytes;
    int64_t n_out;                                      // row length of Y and of the residual
    // Small-batch matrix-core kernel only: more rows than one launch's 16 are dealt to the y dimension of the grid in
    // chunks of the kernel's M argument; m_total is then the number of rows of X (0: a single chunk).
    int m_total;
};

// Bytes between a gate row block and its up row block; the kernels add it to offsets inside a 2 GiB
// buffer resource, so it may not exceed 1 GiB.
constexpr int64_t kMaxHalfBytes = (int64_t)1 << 30;
inline int64_t gated_half_bytes(int64_t N, int64_t K, int group)
{
    return (N / 2 / kBlockRows) * k_blocks(K) * (int64_t)block_bytes(group);
}

__device__ inline float silu_f32(float g) { return g / (1.f + __expf(-g)); }

__device__ inline half_t param_scale(uint32_t word) { return __builtin_bit_cast(half_t, (uint16_t)(word & 0xFFFFu)); }
__device__ inline half_t param_bias(uint32_t word) { return __builtin_bit_cast(half_t, (uint16_t)(word >> 16)); }

}  // namespace e0m4
