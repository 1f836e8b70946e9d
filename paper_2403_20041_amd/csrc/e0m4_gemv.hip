// Decode path of e0m4_matmul: Y[M,N] = X[M,K] * dequant(codes)^T for M <= 8.
// Paper: section "Operator and lagging optimizations" (vector-matrix product
// of the decoding stage, bound by memory bandwidth) with the dequantisation of
// section "E0M4 FP4 quantization" fused in registers.
//
// Work decomposition (gfx950, wave64): one lane owns one output row, so the
// activations are wavefront-uniform and are read through scalar loads; a
// wavefront streams the 1 KiB chunks of its 64-row block along K with
// dwordx4 loads.  Per group the kernel accumulates a = sum_k x_k * w1_k with
// v_dot2_f32_f16 on the raw binade values w1 = 2 + code/8 and applies the
// group's affine map once:  y += scale * (a - bias * sum_k x_k).
// K is split over the 4 wavefronts of a workgroup (reduced through LDS) and,
// when N alone cannot fill the chip, over several workgroups whose fp32
// partial sums are added in a fixed order by a second small kernel.
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kNumCU = 256;

struct GemvPlan {
    int64_t nrb;        // 64-row blocks
    int ngroups;        // K / G
    int gps;            // groups per workgroup (split length)
    int splits;         // workgroups along K
};

GemvPlan make_plan(int64_t N, int64_t K, int group)
{
    GemvPlan p;
    p.nrb = padded_rows(N) / kRowsPerBlock;
    p.ngroups = (int)(K / group);
    int wgs_per_cu = knob("gemv_wgs_per_cu");
    if (wgs_per_cu <= 0) wgs_per_cu = 4;
    int min_gps = knob("gemv_min_groups_per_wg");
    if (min_gps <= 0) min_gps = kWaves * (128 / group);           // at least 4 KiB of codes per wavefront
    const int64_t target = (int64_t)kNumCU * wgs_per_cu;
    int64_t s = (target + p.nrb - 1) / (p.nrb > 0 ? p.nrb : 1);
    const int forced = knob("gemv_splits");
    if (forced > 0) s = forced;
    int gps = (int)((p.ngroups + s - 1) / (s > 0 ? s : 1));
    if (forced <= 0 && gps < min_gps) gps = min_gps;
    if (gps > p.ngroups) gps = p.ngroups;
    if (gps < 1) gps = 1;
    p.gps = gps;
    p.splits = p.ngroups > 0 ? (p.ngroups + gps - 1) / gps : 1;
    return p;
}

template <int G, int M>
__global__ __launch_bounds__(kThreads) void gemv_kernel(const half_t* __restrict__ X,
                                                        const uint4* __restrict__ codes,
                                                        const half_t* __restrict__ scales,
                                                        const half_t* __restrict__ bias, int64_t N, int64_t K,
                                                        int ngroups, int gps, int splits, half_t* __restrict__ Y,
                                                        float* __restrict__ partial)
{
    constexpr int CPG = G / kCodesPerChunk;             // chunks per group
    constexpr int LPG = G / 8;                          // lanes that sum one group's activations
    extern __shared__ float smem[];
    float* sx = smem;                                   // [M][gps] sum of x over each group
    float* red = smem + M * gps;                        // [kWaves-1][M][64]

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t fmask = frac_mask_vgpr();
    const int split = blockIdx.x % splits;
    const int64_t rb = blockIdx.x / splits;
    const int gb = split * gps;
    const int ge = min(gb + gps, ngroups);
    const int64_t n = rb * kRowsPerBlock + lane;
    const int64_t nn = n < N ? n : N - 1;
    const int64_t nchunks = K / kCodesPerChunk;

    // group sums of the activations: LPG lanes x 8 halves per group
    for (int i = t / LPG; i < (ge - gb) * M; i += kThreads / LPG) {
        const int m = i / (ge - gb), gl = i % (ge - gb);
        const half8_t v = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + (int64_t)(gb + gl) * G + (t % LPG) * 8);
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (float)v[j];
#pragma unroll
        for (int d = LPG / 2; d >= 1; d >>= 1) s += __shfl_xor(s, d);
        if (t % LPG == 0) sx[m * gps + gl] = s;
    }
    __syncthreads();

    float acc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] = 0.f;

    const half2_t* __restrict__ X2 = reinterpret_cast<const half2_t*>(X);
    const uint4* cbase = codes + (rb * nchunks) * kRowsPerBlock + lane;

    uint4 cur[CPG];
    int g = gb + wave;
    if (g < ge) {
#pragma unroll
        for (int j = 0; j < CPG; ++j) cur[j] = cbase[((int64_t)g * CPG + j) * kRowsPerBlock];
    }
    for (; g < ge; g += kWaves) {
        const float sc = (float)scales[(int64_t)g * N + nn];
        const float bi = (float)bias[(int64_t)g * N + nn];
        uint4 nxt[CPG];
        const int gn = g + kWaves;
        if (gn < ge) {
#pragma unroll
            for (int j = 0; j < CPG; ++j) nxt[j] = cbase[((int64_t)gn * CPG + j) * kRowsPerBlock];
        }
        float a[M];
#pragma unroll
        for (int m = 0; m < M; ++m) a[m] = 0.f;
#pragma unroll
        for (int j = 0; j < CPG; ++j) {
            const uint32_t words[4] = {cur[j].x, cur[j].y, cur[j].z, cur[j].w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const half2_t p0 = w1_pair<0>(words[w], fmask), p1 = w1_pair<1>(words[w], fmask);
                const half2_t p2 = w1_pair<2>(words[w], fmask), p3 = w1_pair<3>(words[w], fmask);
                const int64_t kk = ((int64_t)g * G + j * 32 + w * 8) / 2;     // half2 index, wavefront-uniform
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    const half2_t* xr = X2 + (int64_t)m * (K / 2) + kk;
                    a[m] = __builtin_amdgcn_fdot2(p0, xr[0], a[m], false);
                    a[m] = __builtin_amdgcn_fdot2(p1, xr[1], a[m], false);
                    a[m] = __builtin_amdgcn_fdot2(p2, xr[2], a[m], false);
                    a[m] = __builtin_amdgcn_fdot2(p3, xr[3], a[m], false);
                }
            }
        }
#pragma unroll
        for (int m = 0; m < M; ++m) acc[m] += sc * (a[m] - bi * sx[m * gps + (g - gb)]);
        if (gn < ge) {
#pragma unroll
            for (int j = 0; j < CPG; ++j) cur[j] = nxt[j];
        }
    }

    // fixed-order reduction over the 4 wavefronts
    if (wave > 0) {
#pragma unroll
        for (int m = 0; m < M; ++m) red[((wave - 1) * M + m) * 64 + lane] = acc[m];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float s = acc[m];
#pragma unroll
            for (int w = 0; w < kWaves - 1; ++w) s += red[(w * M + m) * 64 + lane];
            if (splits == 1) {
                if (n < N) Y[(int64_t)m * N + n] = (half_t)s;
            } else {
                partial[((int64_t)split * M + m) * (gridDim.x / splits * kRowsPerBlock) + n] = s;
            }
        }
    }
}

// Y[m,n] = fp16( sum_s partial[s][m][n] ), s ascending.
__global__ __launch_bounds__(256) void gemv_reduce_kernel(const float* __restrict__ partial, int splits, int64_t M,
                                                          int64_t N, int64_t Npad, half_t* __restrict__ Y)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M * N) return;
    const int64_t m = i / N, n = i % N;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += partial[((int64_t)sp * M + m) * Npad + n];
    Y[i] = (half_t)s;
}

template <int G, int M>
int launch_one(const GemvPlan& p, const void* X, const void* codes, const void* scales, const void* bias, int64_t N,
               int64_t K, void* Y, void* workspace, hipStream_t stream)
{
    const size_t smem = sizeof(float) * ((size_t)M * p.gps + (size_t)(kWaves - 1) * M * 64);
    const dim3 grid((unsigned)(p.nrb * p.splits));
    hipLaunchKernelGGL((gemv_kernel<G, M>), grid, dim3(kThreads), smem, stream, static_cast<const half_t*>(X),
                       static_cast<const uint4*>(codes), static_cast<const half_t*>(scales),
                       static_cast<const half_t*>(bias), N, K, p.ngroups, p.gps, p.splits, static_cast<half_t*>(Y),
                       static_cast<float*>(workspace));
    int rc = check_launch();
    if (rc != E0M4_OK || p.splits == 1) return rc;
    const int64_t total = (int64_t)M * N;
    hipLaunchKernelGGL(gemv_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const float*>(workspace), p.splits, (int64_t)M, N, p.nrb * kRowsPerBlock,
                       static_cast<half_t*>(Y));
    return check_launch();
}

template <int G>
int launch_m(const GemvPlan& p, int64_t M, const void* X, const void* codes, const void* scales, const void* bias,
             int64_t N, int64_t K, void* Y, void* workspace, hipStream_t stream)
{
    switch (M) {
        case 1: return launch_one<G, 1>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 2: return launch_one<G, 2>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 3: return launch_one<G, 3>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 4: return launch_one<G, 4>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 5: return launch_one<G, 5>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 6: return launch_one<G, 6>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 7: return launch_one<G, 7>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 8: return launch_one<G, 8>(p, X, codes, scales, bias, N, K, Y, workspace, stream);
        default: return E0M4_ERR_SHAPE;
    }
}

}  // namespace

size_t gemv_workspace_bytes(int64_t M, int64_t N, int64_t K, int group)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const GemvPlan p = make_plan(N, K, group);
    if (p.splits <= 1) return 0;
    return sizeof(float) * (size_t)p.splits * (size_t)M * (size_t)(p.nrb * kRowsPerBlock);
}

int launch_gemv(const void* X, int64_t M, const void* codes, const void* scales, const void* bias, int64_t N,
                int64_t K, int group, void* Y, void* workspace, hipStream_t stream)
{
    const GemvPlan p = make_plan(N, K, group);
    switch (group) {
        case 32: return launch_m<32>(p, M, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 64: return launch_m<64>(p, M, X, codes, scales, bias, N, K, Y, workspace, stream);
        case 128: return launch_m<128>(p, M, X, codes, scales, bias, N, K, Y, workspace, stream);
        default: return E0M4_ERR_GROUP;
    }
}

}  // namespace e0m4
