// Prefill path of e0m4_matmul: Y[M,N] = X[M,K] * dequant(codes)^T on the matrix
// cores.  Paper: section "Operator and lagging optimizations" (matrix-matrix
// product of the prefill stage, bound by compute) with the dequantisation of
// section "E0M4 FP4 quantization" fused into the tile loader.
//
// A workgroup owns a BM x BN tile of Y.  Per BK slice the activations go
// global -> registers -> LDS unchanged, the weight codes go global ->
// registers -> (shift, mask|exponent, minus bias, times scale; packed fp16,
// one rounding, bit-identical to e0m4_dequant) -> LDS, and the wavefronts run
// v_mfma_f32_32x32x16_f16 on 16-byte K-contiguous fragments of both tiles with
// fp32 accumulators.
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kThreads = 256;
constexpr int kLdsStride = BK + 8;      // halves; 144-byte rows make the 16-byte fragment reads conflict-free

__device__ inline half2_t dequant_pair(half2_t w1, half2_t bias2, half2_t scale2)
{
    return (w1 - bias2) * scale2;       // difference exact, product rounded once
}

template <int G>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const half_t* __restrict__ X, int64_t M,
                                                        const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                        half_t* __restrict__ Y, int m_tiles)
{
    __shared__ __attribute__((aligned(16))) half_t As[BM * kLdsStride];
    __shared__ __attribute__((aligned(16))) half_t Bs[BN * kLdsStride];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const uint32_t fmask = frac_mask_vgpr();
    const int64_t mt = blockIdx.x % m_tiles;
    const int64_t nt = blockIdx.x / m_tiles;
    const int64_t m0 = mt * BM, n0 = nt * BN;
    const PackedLayout<G> lay(K);
    const int64_t nrb = row_blocks(N);

    // A loader: 4 x 16 bytes per thread, 8 lanes cover one 128-byte row slice
    const int a_row = t >> 3, a_piece = t & 7;
    // B loader: one 16-byte chunk per thread.  The 128 x 64 weight tile is the left or right half of
    // 8 packed blocks; 32 consecutive threads read the 512 contiguous bytes of one half block.
    const int b_hb = t >> 5, b_q = (t >> 4) & 1, b_r = t & 15;
    const int64_t rb = n0 / kBlockRows + b_hb;
    const bool b_ok = rb < nrb;

    uint4 a_reg[4];
    uint4 b_reg;
    uint32_t pw_reg;

    auto load_tile = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t m = m0 + a_row + 32 * i;
            const int64_t k = k0 + a_piece * 8;
            a_reg[i] = make_uint4(0, 0, 0, 0);
            if (m < M && k < K) a_reg[i] = *reinterpret_cast<const uint4*>(X + m * K + k);
        }
        b_reg = make_uint4(0, 0, 0, 0);
        pw_reg = 0;                                      // scale 0, bias 0: dequantises to 0
        if (b_ok) {
            const int64_t kb = k0 / kBlockK;
            const int q = (int)(k0 % kBlockK) / kCodesPerChunk + b_q;
            b_reg = packed[lay.code_index(rb, kb) + q * kBlockRows + b_r];
            pw_reg = reinterpret_cast<const uint32_t*>(packed)[lay.param_index(rb, kb) + lay.param_slot(q, b_r)];
        }
    };

    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint4*>(&As[(a_row + 32 * i) * kLdsStride + a_piece * 8]) = a_reg[i];
        const half_t sc = param_scale(pw_reg), bi = param_bias(pw_reg);
        const half2_t s2 = {sc, sc}, b2 = {bi, bi};
        const uint32_t words[4] = {b_reg.x, b_reg.y, b_reg.z, b_reg.w};
        half_t* dst = &Bs[(b_hb * kBlockRows + b_r) * kLdsStride + b_q * 32];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            half2_t o[4];
            o[0] = dequant_pair(w1_pair<0>(words[w], fmask), b2, s2);
            o[1] = dequant_pair(w1_pair<1>(words[w], fmask), b2, s2);
            o[2] = dequant_pair(w1_pair<2>(words[w], fmask), b2, s2);
            o[3] = dequant_pair(w1_pair<3>(words[w], fmask), b2, s2);
            *reinterpret_cast<uint4*>(dst + w * 8) = *reinterpret_cast<const uint4*>(o);
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;     // wavefront tile origin inside the block tile
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;

    load_tile(0);
    for (int64_t k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();
        store_tile();
        __syncthreads();
        if (k0 + BK < K) load_tile(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            half8_t a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[i] = *reinterpret_cast<const half8_t*>(&As[(wm + 32 * i + frag_row) * kLdsStride + kk + frag_k]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = *reinterpret_cast<const half8_t*>(&Bs[(wn + 32 * j + frag_row) * kLdsStride + kk + frag_k]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

    // accumulator layout of the 32x32 block: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn + 32 * j + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M && n < N) Y[m * N + n] = (half_t)acc[i][j][r];
            }
        }
}

}  // namespace

int launch_gemm(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                hipStream_t stream)
{
    const int64_t m_tiles = (M + BM - 1) / BM, n_tiles = (N + BN - 1) / BN;
    if (m_tiles * n_tiles > 0x7fffffffLL) return E0M4_ERR_SHAPE;
    const dim3 grid((unsigned)(m_tiles * n_tiles)), block(kThreads);
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    switch (group) {
        case 32: hipLaunchKernelGGL(gemm_kernel<32>, grid, block, 0, stream, x, M, c, N, K, y, (int)m_tiles); break;
        case 64: hipLaunchKernelGGL(gemm_kernel<64>, grid, block, 0, stream, x, M, c, N, K, y, (int)m_tiles); break;
        case 128: hipLaunchKernelGGL(gemm_kernel<128>, grid, block, 0, stream, x, M, c, N, K, y, (int)m_tiles); break;
        default: return E0M4_ERR_GROUP;
    }
    return check_launch();
}

}  // namespace e0m4
