// Offline side of libe0m4: fit + encode + pack (e0m4_quantize, e0m4_encode) and
// the two ways to look inside the packed buffer (e0m4_dequant,
// e0m4_unpack_codes).  Paper: section "E0M4 FP4 quantization".
//
// Compiled with -ffp-contract=off: every fp32 step of the quantiser is one
// IEEE operation (divide, add, compare, convert), which is what makes the
// codes reproducible bit for bit on another machine.
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr float kLo = 2.0f;             // 2^n with n = 1
constexpr float kHi = 3.998046875f;     // 2^(n+1) - eps, eps = one fp16 ulp of the binade (bits 0x43FF)
constexpr float kSpan = 1.998046875f;   // kHi - kLo, exact
constexpr float kMinScale = 6.103515625e-05f;   // smallest normal fp16
constexpr float kMaxScale = 65504.0f;           // largest finite fp16

constexpr int kThreads = 256;
constexpr int kTileRows = 64;           // one workgroup handles 4 row blocks x 1 k block

__device__ inline uint16_t half_bits(half_t h) { return __builtin_bit_cast(uint16_t, h); }
__device__ inline half_t bits_half(uint16_t b) { return __builtin_bit_cast(half_t, b); }

// code = min(y1 + y2, 15): y1 = four highest fraction bits of the mapped fp16
// value, y2 = the bit below them (paper: quantization paragraph).
__device__ inline uint32_t encode_value(float w0, float sf, float bf)
{
    float q = w0 / sf;
    float t = q + bf;
    t = t < kLo ? kLo : t;
    t = t > kHi ? kHi : t;
    uint32_t bits = half_bits((half_t)t);
    uint32_t y1 = (bits >> 6) & 15u;
    uint32_t y2 = (bits >> 5) & 1u;
    uint32_t c = y1 + y2;
    return c > 15u ? 15u : c;
}

// INT4 comparison format (paper: section "Evaluation of FP4 quantization"): q = clamp(rne(w / scale)
// + zero, 0, 15) with an integer zero point kept as an fp16 number.
__device__ inline uint32_t encode_value_int4(float w0, float sf, float zf)
{
    float q = w0 / sf;
    float t = rintf(q) + zf;
    t = t < 0.0f ? 0.0f : t;
    t = t > 15.0f ? 15.0f : t;
    return (uint32_t)t;
}

// kE0M3: the 3-bit member of the family (the E0M4 definition with three code bits: code = min(fraction bits
// 9..7 + bit 6, 7), bias truncated to three fraction bits); a code c is stored in a 4-bit slot as 2c, which
// is the E0M4 code with the same value 2 + c/4, so every kernel that reads E0M4 codes reads these unchanged.
// kBf16: the same construction on bfloat16 (7 fraction bits: code = min(bits 6..3 + bit 2, 15), top of the
// binade 4 - 2^-6, bias truncated to bits 6..3; weights, scale and bias are bfloat16 bit patterns).
enum Format { kE0M4 = 0, kInt4 = 1, kE0M3 = 2, kBf16 = 3 };

constexpr float kHiBf16 = 3.984375f;            // 4 - 2^-6, bits 0x407F
constexpr float kSpanBf16 = 1.984375f;
constexpr float kMinScaleBf16 = 1.17549435e-38f;            // 2^-126, smallest normal bfloat16
constexpr float kMaxScaleBf16 = 3.3895313892515355e38f;     // largest finite bfloat16, bits 0x7F7F

__device__ inline float bf16_bits_to_float(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
// round to nearest even; the argument is finite here
__device__ inline uint16_t float_to_bf16_bits(float f)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// The general form of encode_value: CODE_SHIFT = fraction bits below the code, TOP = largest code.
template <int FMT>
__device__ inline uint32_t encode_value_fmt(float w0, float sf, float bf)
{
    constexpr bool BF = FMT == kBf16;
    constexpr int SHIFT = BF ? 3 : (FMT == kE0M3 ? 7 : 6);
    constexpr uint32_t TOP = FMT == kE0M3 ? 7u : 15u;
    const float hi = BF ? kHiBf16 : kHi;
    float q = w0 / sf;
    float t = q + bf;
    t = t < kLo ? kLo : t;
    t = t > hi ? hi : t;
    const uint32_t bits = BF ? (uint32_t)float_to_bf16_bits(t) : (uint32_t)half_bits((half_t)t);
    const uint32_t y1 = (bits >> SHIFT) & TOP;
    const uint32_t y2 = (bits >> (SHIFT - 1)) & 1u;
    const uint32_t c = y1 + y2;
    return c > TOP ? TOP : c;
}

// Thread t owns the 8-weight piece t%16 of row (t/16) of row block i, i = 0..3,
// so 16 consecutive lanes read 256 contiguous bytes of one row and a group of G
// weights is G/8 adjacent lanes.  The four finished blocks are staged in LDS and
// written out in 16-byte pieces.
template <int G, bool FIT, int FMT = kE0M4>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const half_t* __restrict__ W, int64_t N, int64_t K,
                                                            uint4* __restrict__ packed,
                                                            half_t* __restrict__ scales_out,
                                                            half_t* __restrict__ bias_out,
                                                            const half_t* __restrict__ scales_in,
                                                            const half_t* __restrict__ bias_in)
{
    constexpr int BW = block_bytes(G) / 4;              // 32-bit words per block
    constexpr int PPB = block_bytes(G) / 16;            // 16-byte pieces per block
    __shared__ __attribute__((aligned(16))) uint32_t stage[4 * BW];
    const int t = threadIdx.x;
    const int64_t rb64 = blockIdx.x;
    const int64_t kb = blockIdx.y;
    const int piece = t & 15;
    const int r = t >> 4;
    const int64_t k = kb * kBlockK + piece * 8;
    const bool k_ok = k < K;
    const int64_t ng = K / G;
    const int64_t g = k / G;

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t n = rb64 * kTileRows + 16 * i + r;
        const bool ok = k_ok && n < N;
        half8_t v8 = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ok) v8 = *reinterpret_cast<const half8_t*>(W + n * K + k);
        constexpr bool BF = FMT == kBf16;               // bfloat16 bit patterns in W, scales and bias
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = BF ? bf16_bits_to_float(half_bits(v8[j])) : (float)v8[j];

        float sf, bf;
        half_t sh, bh;                                  // 16-bit patterns of the group's parameters (fp16, or bfloat16)
        if (FIT) {
            float mn = 0.0f, mx = 0.0f;                 // the range always contains 0
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                mn = fminf(mn, v[j]);
                mx = fmaxf(mx, v[j]);
            }
#pragma unroll
            for (int d = G / 16; d >= 1; d >>= 1) {     // G/8 adjacent lanes form the group
                mn = fminf(mn, __shfl_xor(mn, d));
                mx = fmaxf(mx, __shfl_xor(mx, d));
            }
            float range = mx - mn;
            float s = range / (FMT == kInt4 ? 15.0f : (BF ? kSpanBf16 : kSpan));
            s = s < (BF ? kMinScaleBf16 : kMinScale) ? (BF ? kMinScaleBf16 : kMinScale) : s;
            s = s > (BF ? kMaxScaleBf16 : kMaxScale) ? (BF ? kMaxScaleBf16 : kMaxScale) : s;
            sh = BF ? bits_half(float_to_bf16_bits(s)) : (half_t)s;
            sf = BF ? bf16_bits_to_float(half_bits(sh)) : (float)sh;     // encode with the stored scale
            float q = mn / sf;
            if (BF) {
                float b = kLo - q;
                b = b < kLo ? kLo : b;
                b = b > kHiBf16 ? kHiBf16 : b;
                bh = bits_half(float_to_bf16_bits(b) & 0xFFF8u);          // keep fraction bits 6..3
            } else if (FMT == kInt4) {
                float z = rintf(-q);                    // integer zero point, round half to even
                z = z < 0.0f ? 0.0f : z;
                z = z > 15.0f ? 15.0f : z;
                bh = (half_t)z;                         // exact
            } else {
                float b = kLo - q;                      // image of zero in the binade
                b = b < kLo ? kLo : b;
                b = b > kHi ? kHi : b;
                // keep the four (three) highest fraction bits
                bh = bits_half(half_bits((half_t)b) & (FMT == kE0M3 ? 0xFF80u : 0xFFC0u));
            }
            bf = BF ? bf16_bits_to_float(half_bits(bh)) : (float)bh;
            if (ok && (piece % (G / 8)) == 0) {
                scales_out[n * ng + g] = sh;
                bias_out[n * ng + g] = bh;
            }
        } else {
            sh = BF ? bits_half(0x3F80u) : (half_t)1.0f;
            bh = bits_half(0x4000u);                    // 2.0 in both formats
            if (ok) {
                sh = scales_in[n * ng + g];
                bh = bias_in[n * ng + g];
            }
            sf = BF ? bf16_bits_to_float(half_bits(sh)) : (float)sh;
            bf = BF ? bf16_bits_to_float(half_bits(bh)) : (float)bh;
        }

        uint32_t word = 0;
        if (ok) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t c;
                if (FMT == kInt4) c = encode_value_int4(v[j], sf, bf);
                else if (FMT == kE0M4) c = encode_value(v[j], sf, bf);
                else if (FMT == kE0M3) c = encode_value_fmt<kE0M3>(v[j], sf, bf) << 1;      // the E0M4 code of the same value
                else c = encode_value_fmt<kBf16>(v[j], sf, bf);
                word |= place_code(c, j);
            }
        }
        stage[i * BW + ((piece >> 2) * kBlockRows + r) * 4 + (piece & 3)] = word;
        if ((piece % (G / 8)) == 0) {
            const uint32_t pw = ok ? ((uint32_t)half_bits(sh) | ((uint32_t)half_bits(bh) << 16)) : 0u;
            stage[i * BW + kBlockCodeBytes / 4 + (piece * 8 / G) * kBlockRows + r] = pw;
        }
    }
    __syncthreads();
    const int64_t nrb = row_blocks(N);
    const PackedLayout<G> lay(K);
    constexpr int CP = PackedLayout<G>::kCodePieces;    // the first CP pieces of a staged block are codes
    for (int pi = t; pi < 4 * PPB; pi += kThreads) {
        const int i = pi / PPB, off = pi % PPB;
        const int64_t rb = rb64 * 4 + i;
        if (rb < nrb) {
            const int64_t dst = off < CP ? lay.code_index(rb, kb) + off : lay.param_index(rb, kb) / 4 + (off - CP);
            packed[dst] = *reinterpret_cast<const uint4*>(&stage[i * BW + off * 4]);
        }
    }
}

// Wavefront i of the workgroup reads block (4*rb64 + i, kb): codes and the
// block's parameter words; the 64 x 128 tile goes through LDS so that rows are
// written out in 256-byte runs.
template <int G, int FMT = kE0M4>
__global__ __launch_bounds__(kThreads) void dequant_kernel(const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                           half_t* __restrict__ W_out)
{
    constexpr int kStride = kBlockK + 8;                // halves; +16 bytes keeps ds_write_b128 conflict-free
    __shared__ __attribute__((aligned(16))) half_t tile[kTileRows * kStride];
    const int t = threadIdx.x;
    const int64_t rb64 = blockIdx.x;
    const int64_t kb = blockIdx.y;
    const int64_t nrb = row_blocks(N);
    const PackedLayout<G> lay(K);
    {
        const int i = t >> 6, lane = t & 63;
        const int q = lane >> 4, r = lane & 15;
        const int64_t rb = rb64 * 4 + i;
        if (rb < nrb) {
            const uint4 c = packed[lay.code_index(rb, kb) + lane];
            const uint32_t pw = reinterpret_cast<const uint32_t*>(packed)[lay.param_index(rb, kb) + lay.param_slot(q, r)];
            const float sf = FMT == kBf16 ? bf16_bits_to_float((uint16_t)(pw & 0xFFFFu)) : (float)param_scale(pw);
            const float bf = FMT == kBf16 ? bf16_bits_to_float((uint16_t)(pw >> 16)) : (float)param_bias(pw);
            const uint32_t words[4] = {c.x, c.y, c.z, c.w};
            const uint32_t fmask = frac_mask_vgpr();
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const half2_t p[4] = {w1_pair<0>(words[w], fmask), w1_pair<1>(words[w], fmask),
                                      w1_pair<2>(words[w], fmask), w1_pair<3>(words[w], fmask)};
                half8_t o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (FMT == kInt4) {
                        // (q - zero) is an exact small integer, its product with the scale exact in fp32
                        o[2 * j] = (half_t)(((float)extract_code(words[w], 2 * j) - bf) * sf);
                        o[2 * j + 1] = (half_t)(((float)extract_code(words[w], 2 * j + 1) - bf) * sf);
                    } else if (FMT == kBf16) {
                        // w1 = 2 + code/8 whatever the format; difference and product exact in fp32, one rounding
                        o[2 * j] = bits_half(float_to_bf16_bits(((float)p[j][0] - bf) * sf));
                        o[2 * j + 1] = bits_half(float_to_bf16_bits(((float)p[j][1] - bf) * sf));
                    } else {
                        // (w1 - bias) is exact and its product with the scale is exact in fp32: one rounding
                        o[2 * j] = (half_t)(((float)p[j][0] - bf) * sf);
                        o[2 * j + 1] = (half_t)(((float)p[j][1] - bf) * sf);
                    }
                }
                *reinterpret_cast<half8_t*>(&tile[(16 * i + r) * kStride + q * 32 + w * 8]) = o;
            }
        }
    }
    __syncthreads();
    const int piece = t & 15;
    const int64_t k = kb * kBlockK + piece * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (t >> 4) + 16 * i;
        const int64_t n = rb64 * kTileRows + r;
        if (k < K && n < N)
            *reinterpret_cast<half8_t*>(W_out + n * K + k) = *reinterpret_cast<const half8_t*>(&tile[r * kStride + piece * 8]);
    }
}

template <int G>
__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                          uint8_t* __restrict__ out, int shift)
{
    constexpr int kStride = kBlockK + 16;               // bytes per row in LDS
    __shared__ __attribute__((aligned(16))) uint8_t tile[kTileRows * kStride];
    const int t = threadIdx.x;
    const int64_t rb64 = blockIdx.x;
    const int64_t kb = blockIdx.y;
    const int64_t nrb = row_blocks(N);
    const PackedLayout<G> lay(K);
    {
        const int i = t >> 6, lane = t & 63;
        const int q = lane >> 4, r = lane & 15;
        const int64_t rb = rb64 * 4 + i;
        if (rb < nrb) {
            const uint4 c = packed[lay.code_index(rb, kb) + lane];
            const uint32_t words[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t lo = 0, hi = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    lo |= (extract_code(words[w], j) >> shift) << (8 * j);       // shift 1: 3-bit codes stored doubled
                    hi |= (extract_code(words[w], j + 4) >> shift) << (8 * j);
                }
                *reinterpret_cast<uint2*>(&tile[(16 * i + r) * kStride + q * 32 + w * 8]) = make_uint2(lo, hi);
            }
        }
    }
    __syncthreads();
    const int piece = t & 7;
    const int64_t k = kb * kBlockK + piece * 16;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (t >> 3) + 32 * i;
        const int64_t n = rb64 * kTileRows + r;
        if (k < K && n < N)
            *reinterpret_cast<uint4*>(out + n * K + k) = *reinterpret_cast<const uint4*>(&tile[r * kStride + piece * 16]);
    }
}

dim3 tile_grid(int64_t N, int64_t K)
{
    return dim3((unsigned)((N + kTileRows - 1) / kTileRows), (unsigned)k_blocks(K), 1);
}

}  // namespace

int launch_quantize(const void* W, int64_t N, int64_t K, int group, void* packed, void* scales, void* bias,
                    const void* scales_in, const void* bias_in, bool fit, int format, hipStream_t stream)
{
    const bool int4 = format == kInt4;
    const dim3 grid = tile_grid(N, K), block(kThreads);
    const half_t* w = static_cast<const half_t*>(W);
    uint4* c = static_cast<uint4*>(packed);
    half_t* so = static_cast<half_t*>(scales);
    half_t* bo = static_cast<half_t*>(bias);
    const half_t* si = static_cast<const half_t*>(scales_in);
    const half_t* bi = static_cast<const half_t*>(bias_in);
#define E0M4_LAUNCH_Q(G)                                                                              \
    do {                                                                                              \
        if (int4) hipLaunchKernelGGL((quantize_kernel<G, true, kInt4>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi); \
        else if (format == kE0M3) hipLaunchKernelGGL((quantize_kernel<G, true, kE0M3>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi); \
        else if (format == kBf16 && fit) hipLaunchKernelGGL((quantize_kernel<G, true, kBf16>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi); \
        else if (format == kBf16) hipLaunchKernelGGL((quantize_kernel<G, false, kBf16>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi); \
        else if (fit) hipLaunchKernelGGL((quantize_kernel<G, true>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi); \
        else hipLaunchKernelGGL((quantize_kernel<G, false>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi);    \
    } while (0)
    switch (group) {
        case 32: E0M4_LAUNCH_Q(32); break;
        case 64: E0M4_LAUNCH_Q(64); break;
        case 128: E0M4_LAUNCH_Q(128); break;
        default: return E0M4_ERR_GROUP;
    }
#undef E0M4_LAUNCH_Q
    return check_launch();
}

int launch_dequant(const void* packed, int64_t N, int64_t K, int group, void* W_out, int format, hipStream_t stream)
{
    const dim3 grid = tile_grid(N, K), block(kThreads);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* o = static_cast<half_t*>(W_out);
    const bool int4 = format == kInt4;
    if (format == kBf16) {
        switch (group) {
            case 32: hipLaunchKernelGGL((dequant_kernel<32, kBf16>), grid, block, 0, stream, c, N, K, o); break;
            case 64: hipLaunchKernelGGL((dequant_kernel<64, kBf16>), grid, block, 0, stream, c, N, K, o); break;
            case 128: hipLaunchKernelGGL((dequant_kernel<128, kBf16>), grid, block, 0, stream, c, N, K, o); break;
            default: return E0M4_ERR_GROUP;
        }
        return check_launch();
    }
    if (int4) {
        switch (group) {
            case 32: hipLaunchKernelGGL((dequant_kernel<32, kInt4>), grid, block, 0, stream, c, N, K, o); break;
            case 64: hipLaunchKernelGGL((dequant_kernel<64, kInt4>), grid, block, 0, stream, c, N, K, o); break;
            case 128: hipLaunchKernelGGL((dequant_kernel<128, kInt4>), grid, block, 0, stream, c, N, K, o); break;
            default: return E0M4_ERR_GROUP;
        }
        return check_launch();
    }
    switch (group) {
        case 32: hipLaunchKernelGGL(dequant_kernel<32>, grid, block, 0, stream, c, N, K, o); break;
        case 64: hipLaunchKernelGGL(dequant_kernel<64>, grid, block, 0, stream, c, N, K, o); break;
        case 128: hipLaunchKernelGGL(dequant_kernel<128>, grid, block, 0, stream, c, N, K, o); break;
        default: return E0M4_ERR_GROUP;
    }
    return check_launch();
}

int launch_unpack(const void* packed, int64_t N, int64_t K, int group, void* out, hipStream_t stream, int shift)
{
    const dim3 grid = tile_grid(N, K), block(kThreads);
    const uint4* c = static_cast<const uint4*>(packed);
    uint8_t* o = static_cast<uint8_t*>(out);
    switch (group) {
        case 32: hipLaunchKernelGGL(unpack_kernel<32>, grid, block, 0, stream, c, N, K, o, shift); break;
        case 64: hipLaunchKernelGGL(unpack_kernel<64>, grid, block, 0, stream, c, N, K, o, shift); break;
        case 128: hipLaunchKernelGGL(unpack_kernel<128>, grid, block, 0, stream, c, N, K, o, shift); break;
        default: return E0M4_ERR_GROUP;
    }
    return check_launch();
}

}  // namespace e0m4
