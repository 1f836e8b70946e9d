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

constexpr int kTileK = 128;             // k extent of one workgroup tile (4 chunks)
constexpr int kThreads = 256;

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

// One workgroup = 64 rows x 128 k.  Thread t owns the 8-weight piece t%16 of
// row (t/16 + 16*i), i = 0..3, so 16 consecutive lanes read 256 contiguous
// bytes of one row and a group of G weights is G/8 adjacent lanes.
template <int G, bool FIT>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const half_t* __restrict__ W, int64_t N, int64_t K,
                                                            uint32_t* __restrict__ codes,
                                                            half_t* __restrict__ scales_out,
                                                            half_t* __restrict__ bias_out,
                                                            const half_t* __restrict__ scales_in,
                                                            const half_t* __restrict__ bias_in)
{
    __shared__ uint32_t tile[4 * kRowsPerBlock * 4];    // [chunk][row][word]
    const int t = threadIdx.x;
    const int64_t rb = blockIdx.x;
    const int64_t k0 = (int64_t)blockIdx.y * kTileK;
    const int piece = t & 15;
    const int64_t k = k0 + piece * 8;
    const bool k_ok = k < K;
    const int64_t g = k / G;

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (t >> 4) + 16 * i;
        const int64_t n = rb * kRowsPerBlock + r;
        const bool ok = k_ok && n < N;
        half8_t v8 = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ok) v8 = *reinterpret_cast<const half8_t*>(W + n * K + k);
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (float)v8[j];

        float sf, bf;
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
            float s = range / kSpan;
            s = s < kMinScale ? kMinScale : s;
            s = s > kMaxScale ? kMaxScale : s;
            half_t sh = (half_t)s;
            sf = (float)sh;                             // encode with the stored scale
            float q = mn / sf;
            float b = kLo - q;                          // image of zero in the binade
            b = b < kLo ? kLo : b;
            b = b > kHi ? kHi : b;
            half_t bh = bits_half(half_bits((half_t)b) & 0xFFC0u);   // keep the four highest fraction bits
            bf = (float)bh;
            if (ok && (piece % (G / 8)) == 0) {
                scales_out[g * N + n] = sh;
                bias_out[g * N + n] = bh;
            }
        } else {
            sf = 1.0f;
            bf = kLo;
            if (ok) {
                sf = (float)scales_in[g * N + n];
                bf = (float)bias_in[g * N + n];
            }
        }

        uint32_t word = 0;
        if (ok) {
#pragma unroll
            for (int j = 0; j < 8; ++j) word |= encode_value(v[j], sf, bf) << nibble_shift(j);
        }
        tile[((piece >> 2) * kRowsPerBlock + r) * 4 + (piece & 3)] = word;
    }
    __syncthreads();
    // thread t writes chunk t/64 of row t%64: each wavefront stores 1 KiB contiguous
    const int q = t >> 6, r = t & 63;
    const int64_t chunk = k0 / kCodesPerChunk + q;
    if (chunk < K / kCodesPerChunk) {
        const uint4 out = *reinterpret_cast<const uint4*>(&tile[(q * kRowsPerBlock + r) * 4]);
        *reinterpret_cast<uint4*>(codes + ((rb * (K / kCodesPerChunk) + chunk) * kRowsPerBlock + r) * 4) = out;
    }
}

// Workgroup = 64 rows x 128 k.  Wavefront w reads chunk w of the tile (1 KiB
// contiguous, lane = row), dequantises it, and the tile goes through LDS so
// that rows are written out in 256-byte runs.
template <int G>
__global__ __launch_bounds__(kThreads) void dequant_kernel(const uint32_t* __restrict__ codes,
                                                           const half_t* __restrict__ scales,
                                                           const half_t* __restrict__ bias, int64_t N, int64_t K,
                                                           half_t* __restrict__ W_out)
{
    constexpr int kStride = kTileK + 8;                 // halves; +16 bytes keeps ds_write_b128 conflict-free
    __shared__ __attribute__((aligned(16))) half_t tile[kRowsPerBlock * kStride];
    const int t = threadIdx.x;
    const int64_t rb = blockIdx.x;
    const int64_t k0 = (int64_t)blockIdx.y * kTileK;
    {
        const int q = t >> 6, r = t & 63;
        const int64_t chunk = k0 / kCodesPerChunk + q;
        const int64_t n = rb * kRowsPerBlock + r;
        if (chunk < K / kCodesPerChunk) {
            const uint4 c = *reinterpret_cast<const uint4*>(codes + ((rb * (K / kCodesPerChunk) + chunk) * kRowsPerBlock + r) * 4);
            const int64_t g = chunk * kCodesPerChunk / G;
            const int64_t nn = n < N ? n : N - 1;
            const float sf = (float)scales[g * N + nn];
            const float bf = (float)bias[g * N + nn];
            const uint32_t words[4] = {c.x, c.y, c.z, c.w};
            const uint32_t fmask = frac_mask_vgpr();
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const half2_t p[4] = {w1_pair<0>(words[w], fmask), w1_pair<1>(words[w], fmask), w1_pair<2>(words[w], fmask),
                                      w1_pair<3>(words[w], fmask)};
                half8_t o;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // (w1 - bias) is exact and its product with the scale is exact in fp32: one rounding
                    o[2 * i] = (half_t)(((float)p[i][0] - bf) * sf);
                    o[2 * i + 1] = (half_t)(((float)p[i][1] - bf) * sf);
                }
                *reinterpret_cast<half8_t*>(&tile[r * kStride + q * 32 + w * 8]) = o;
            }
        }
    }
    __syncthreads();
    const int piece = t & 15;
    const int64_t k = k0 + piece * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (t >> 4) + 16 * i;
        const int64_t n = rb * kRowsPerBlock + r;
        if (k < K && n < N)
            *reinterpret_cast<half8_t*>(W_out + n * K + k) = *reinterpret_cast<const half8_t*>(&tile[r * kStride + piece * 8]);
    }
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint32_t* __restrict__ codes, int64_t N, int64_t K,
                                                          uint8_t* __restrict__ out)
{
    constexpr int kStride = kTileK + 16;                // bytes per row in LDS
    __shared__ __attribute__((aligned(16))) uint8_t tile[kRowsPerBlock * kStride];
    const int t = threadIdx.x;
    const int64_t rb = blockIdx.x;
    const int64_t k0 = (int64_t)blockIdx.y * kTileK;
    {
        const int q = t >> 6, r = t & 63;
        const int64_t chunk = k0 / kCodesPerChunk + q;
        if (chunk < K / kCodesPerChunk) {
            const uint4 c = *reinterpret_cast<const uint4*>(codes + ((rb * (K / kCodesPerChunk) + chunk) * kRowsPerBlock + r) * 4);
            const uint32_t words[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t lo = 0, hi = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    lo |= ((words[w] >> nibble_shift(j)) & 15u) << (8 * j);
                    hi |= ((words[w] >> nibble_shift(j + 4)) & 15u) << (8 * j);
                }
                *reinterpret_cast<uint2*>(&tile[r * kStride + q * 32 + w * 8]) = make_uint2(lo, hi);
            }
        }
    }
    __syncthreads();
    const int piece = t & 7;
    const int64_t k = k0 + piece * 16;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (t >> 3) + 32 * i;
        const int64_t n = rb * kRowsPerBlock + r;
        if (k < K && n < N)
            *reinterpret_cast<uint4*>(out + n * K + k) = *reinterpret_cast<const uint4*>(&tile[r * kStride + piece * 16]);
    }
}

dim3 tile_grid(int64_t N, int64_t K)
{
    return dim3((unsigned)(padded_rows(N) / kRowsPerBlock), (unsigned)((K + kTileK - 1) / kTileK), 1);
}

}  // namespace

int launch_quantize(const void* W, int64_t N, int64_t K, int group, void* codes, void* scales, void* bias,
                    const void* scales_in, const void* bias_in, bool fit, hipStream_t stream)
{
    const dim3 grid = tile_grid(N, K), block(kThreads);
    const half_t* w = static_cast<const half_t*>(W);
    uint32_t* c = static_cast<uint32_t*>(codes);
    half_t* so = static_cast<half_t*>(scales);
    half_t* bo = static_cast<half_t*>(bias);
    const half_t* si = static_cast<const half_t*>(scales_in);
    const half_t* bi = static_cast<const half_t*>(bias_in);
#define E0M4_LAUNCH_Q(G)                                                                              \
    do {                                                                                              \
        if (fit) hipLaunchKernelGGL((quantize_kernel<G, true>), grid, block, 0, stream, w, N, K, c, so, bo, si, bi); \
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

int launch_dequant(const void* codes, const void* scales, const void* bias, int64_t N, int64_t K, int group,
                   void* W_out, hipStream_t stream)
{
    const dim3 grid = tile_grid(N, K), block(kThreads);
    const uint32_t* c = static_cast<const uint32_t*>(codes);
    const half_t* s = static_cast<const half_t*>(scales);
    const half_t* b = static_cast<const half_t*>(bias);
    half_t* o = static_cast<half_t*>(W_out);
    switch (group) {
        case 32: hipLaunchKernelGGL(dequant_kernel<32>, grid, block, 0, stream, c, s, b, N, K, o); break;
        case 64: hipLaunchKernelGGL(dequant_kernel<64>, grid, block, 0, stream, c, s, b, N, K, o); break;
        case 128: hipLaunchKernelGGL(dequant_kernel<128>, grid, block, 0, stream, c, s, b, N, K, o); break;
        default: return E0M4_ERR_GROUP;
    }
    return check_launch();
}

int launch_unpack(const void* codes, int64_t N, int64_t K, void* out, hipStream_t stream)
{
    hipLaunchKernelGGL(unpack_kernel, tile_grid(N, K), dim3(kThreads), 0, stream, static_cast<const uint32_t*>(codes), N,
                       K, static_cast<uint8_t*>(out));
    return check_launch();
}

}  // namespace e0m4
