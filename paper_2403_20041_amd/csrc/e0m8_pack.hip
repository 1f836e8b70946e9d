// E0M8, the 8-bit member of the paper's format family (section "E0M4 FP4 quantization", closing remark:
// the approach carries over to other bit widths): the code is the eight highest fraction bits of the
// mapped fp16 value plus the next one for rounding, saturated at 255, and
//     w1 = as_half(0x4000 | code << 2),   w = (w1 - bias) * scale,
// with the bias keeping its eight highest fraction bits.  Offline side: fit + encode + pack, dequantise,
// unpack.  Compiled with -ffp-contract=off like the E0M4 quantiser (every fp32 step one IEEE operation).
//
// Packed layout.  The buffer is the E0M4 layout of a [N, 2K] matrix of 4-bit codes with groups of 128
// codes: a block is 16 rows x 64 weights (1 KiB of codes, then one (scale, bias) word per row), lane
// q*16 + r of a wavefront owns the 16 weights k = 16q..16q+15 of row r as four 32-bit words, and word w
// holds weights 4w..4w+3 as
//     rotl32(c0 | c2 << 8 | c1 << 16 | c3 << 24, 2):
// c0 and c1 lie in fraction bits 9..2 of the two fp16 halves, so (word & 0x03FC03FC) | 0x40004000 is the
// pair (w1_0, w1_1) -- the paper's two bit operations, for two weights at once -- and the same after a
// rotation by 8 bits is (w1_2, w1_3).  In terms of the 4-bit layout the high nibble of a code sits in a
// slot that reads at 1/8 scale and its low nibble in the adjacent slot that reads at 1/128 scale.
// A group of 128 weights spans two blocks; both carry its parameters.
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr float kLo = 2.0f;
constexpr float kHi = 3.998046875f;     // 4 - one fp16 ulp of the binade
constexpr float kSpan = 1.998046875f;
constexpr float kMinScale = 6.103515625e-05f;
constexpr float kMaxScale = 65504.0f;
constexpr int kThreads = 256;
constexpr int kBlockK8 = 64;            // weights per block

__device__ inline uint16_t half_bits(half_t h) { return __builtin_bit_cast(uint16_t, h); }
__device__ inline half_t bits_half(uint16_t b) { return __builtin_bit_cast(half_t, b); }

__device__ inline uint32_t encode8(float w0, float sf, float bf)
{
    float q = w0 / sf;
    float t = q + bf;
    t = t < kLo ? kLo : t;
    t = t > kHi ? kHi : t;
    const uint32_t bits = half_bits((half_t)t);
    const uint32_t c = ((bits >> 2) & 255u) + ((bits >> 1) & 1u);
    return c > 255u ? 255u : c;
}

__host__ __device__ inline uint32_t pack4(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3)
{
    return rotl32(c0 | (c2 << 8) | (c1 << 16) | (c3 << 24), 2);
}
// code i (0..3) of a packed word
__host__ __device__ inline uint32_t code_of(uint32_t word, int i)
{
    const int pos[4] = {0, 16, 8, 24};
    return (rotr32(word, 2) >> pos[i]) & 255u;
}

// One workgroup: 64 rows (4 row blocks) x 128 weights (2 blocks).  Thread t owns the 8 weights
// k = 8 * (t % 16) .. of row t / 16 of row block i (i = 0..3): two packed words.  A group of G weights is
// G/8 adjacent lanes.
template <int G>
__global__ __launch_bounds__(kThreads) void quantize8_kernel(const half_t* __restrict__ W, int64_t N, int64_t K,
                                                             uint4* __restrict__ packed,
                                                             half_t* __restrict__ scales_out,
                                                             half_t* __restrict__ bias_out)
{
    constexpr int BW = block_bytes(128) / 4;            // 32-bit words per block (codes + 16 parameter words)
    constexpr int PPB = block_bytes(128) / 16;
    __shared__ __attribute__((aligned(16))) uint32_t stage[8 * BW];     // [row block i][block half h]
    const int t = threadIdx.x;
    const int64_t rb64 = blockIdx.x;
    const int64_t kb2 = blockIdx.y;                     // pair of blocks
    const int piece = t & 15, r = t >> 4;
    const int h = piece >> 3, p8 = piece & 7;           // block of the pair, piece inside the block
    const int q = p8 >> 1, w0 = (p8 & 1) * 2;           // chunk, first of the two words
    const int64_t k = kb2 * 128 + piece * 8;
    const bool k_ok = k < K;
    const int64_t ng = K / G, g = k / G;

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t n = rb64 * 64 + 16 * i + r;
        const bool ok = k_ok && n < N;
        half8_t v8 = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ok) v8 = *reinterpret_cast<const half8_t*>(W + n * K + k);
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (float)v8[j];
        float mn = 0.0f, mx = 0.0f;                     // the range always contains 0
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            mn = fminf(mn, v[j]);
            mx = fmaxf(mx, v[j]);
        }
#pragma unroll
        for (int d = G / 16; d >= 1; d >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, d));
            mx = fmaxf(mx, __shfl_xor(mx, d));
        }
        float s = (mx - mn) / kSpan;
        s = s < kMinScale ? kMinScale : s;
        s = s > kMaxScale ? kMaxScale : s;
        const half_t sh = (half_t)s;
        const float sf = (float)sh;                     // encode with the stored scale
        float b = kLo - mn / sf;                        // image of zero in the binade
        b = b < kLo ? kLo : b;
        b = b > kHi ? kHi : b;
        const half_t bh = bits_half(half_bits((half_t)b) & 0xFFFCu);    // keep the eight highest fraction bits
        const float bf = (float)bh;
        if (ok && (piece % (G / 8)) == 0) {
            scales_out[n * ng + g] = sh;
            bias_out[n * ng + g] = bh;
        }
        uint32_t word0 = 0, word1 = 0;
        if (ok) {
            word0 = pack4(encode8(v[0], sf, bf), encode8(v[1], sf, bf), encode8(v[2], sf, bf), encode8(v[3], sf, bf));
            word1 = pack4(encode8(v[4], sf, bf), encode8(v[5], sf, bf), encode8(v[6], sf, bf), encode8(v[7], sf, bf));
        }
        uint32_t* blk = &stage[(i * 2 + h) * BW];
        blk[(q * kBlockRows + r) * 4 + w0] = word0;
        blk[(q * kBlockRows + r) * 4 + w0 + 1] = word1;
        if (p8 == 0) blk[kBlockCodeBytes / 4 + r] = ok ? ((uint32_t)half_bits(sh) | ((uint32_t)half_bits(bh) << 16)) : 0u;
    }
    __syncthreads();
    const int64_t nrb = row_blocks(N);
    const PackedLayout<128> lay(2 * K);
    constexpr int CP = PackedLayout<128>::kCodePieces;
    for (int pi = t; pi < 8 * PPB; pi += kThreads) {
        const int blk = pi / PPB, off = pi % PPB;
        const int64_t rb = rb64 * 4 + (blk >> 1), kb8 = kb2 * 2 + (blk & 1);
        if (rb < nrb && kb8 < lay.nkb) {
            const int64_t dst = off < CP ? lay.code_index(rb, kb8) + off : lay.param_index(rb, kb8) / 4 + (off - CP);
            packed[dst] = *reinterpret_cast<const uint4*>(&stage[blk * BW + off * 4]);
        }
    }
}

// One thread per packed word (four weights).  BYTES: write the codes (uint8) instead of the weights.
template <bool BYTES>
__global__ __launch_bounds__(kThreads) void dequant8_kernel(const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                            half_t* __restrict__ W_out, uint8_t* __restrict__ codes_out)
{
    const PackedLayout<128> lay(2 * K);
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t words_per_rb = lay.nkb * 256;         // 64 lanes x 4 words per block
    const int64_t rb = idx / words_per_rb;
    if (rb >= row_blocks(N)) return;
    const int64_t rem = idx - rb * words_per_rb;
    const int64_t kb8 = rem >> 8;
    const int lane = (int)(rem >> 2) & 63, w = (int)rem & 3;
    const int q = lane >> 4, r = lane & 15;
    const int64_t n = rb * kBlockRows + r, k = kb8 * kBlockK8 + q * 16 + w * 4;
    if (n >= N || k >= K) return;
    const uint32_t word = reinterpret_cast<const uint32_t*>(packed + lay.code_index(rb, kb8) + lane)[w];
    if (BYTES) {
#pragma unroll
        for (int i = 0; i < 4; ++i) codes_out[n * K + k + i] = (uint8_t)code_of(word, i);
        return;
    }
    const uint32_t pw = reinterpret_cast<const uint32_t*>(packed)[lay.param_index(rb, kb8) + r];
    const half_t sc = param_scale(pw), bi = param_bias(pw);
    const half2_t s2 = {sc, sc}, b2 = {bi, bi};
    const half2_t w01 = __builtin_bit_cast(half2_t, (word & kFrac8Mask2) | kExpBits2);
    const half2_t w23 = __builtin_bit_cast(half2_t, (rotr32(word, 8) & kFrac8Mask2) | kExpBits2);
    const half2_t o01 = (w01 - b2) * s2, o23 = (w23 - b2) * s2;     // difference exact, product rounded once
    const half4_t o = {o01[0], o01[1], o23[0], o23[1]};
    *reinterpret_cast<half4_t*>(W_out + n * K + k) = o;
}

}  // namespace

int launch_quantize8(const void* W, int64_t N, int64_t K, int group, void* packed, void* scales, void* bias,
                     hipStream_t stream)
{
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((K + 127) / 128)), block(kThreads);
    const half_t* w = static_cast<const half_t*>(W);
    uint4* c = static_cast<uint4*>(packed);
    half_t* so = static_cast<half_t*>(scales);
    half_t* bo = static_cast<half_t*>(bias);
    if (group == 64) hipLaunchKernelGGL(quantize8_kernel<64>, grid, block, 0, stream, w, N, K, c, so, bo);
    else if (group == 128) hipLaunchKernelGGL(quantize8_kernel<128>, grid, block, 0, stream, w, N, K, c, so, bo);
    else return E0M4_ERR_GROUP;
    return check_launch();
}

int launch_dequant8(const void* packed, int64_t N, int64_t K, void* W_out, void* codes_out, hipStream_t stream)
{
    const int64_t words = row_blocks(N) * k_blocks(2 * K) * 256;
    const int64_t blocks = (words + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return E0M4_ERR_SHAPE;
    const uint4* c = static_cast<const uint4*>(packed);
    if (codes_out)
        hipLaunchKernelGGL(dequant8_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, c, N, K,
                           (half_t*)nullptr, static_cast<uint8_t*>(codes_out));
    else
        hipLaunchKernelGGL(dequant8_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, c, N, K,
                           static_cast<half_t*>(W_out), (uint8_t*)nullptr);
    return check_launch();
}

}  // namespace e0m4
