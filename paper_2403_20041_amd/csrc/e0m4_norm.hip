// Row-wise rms-norm of the activations, the prologue of e0m4_matmul_fused on the GEMM path (on the
// decode paths the same arithmetic runs inside the matmul kernel while X is staged).  Paper: section
// "Operator and lagging optimizations" (the small operators of rms-norm fused into one).
//   out[m, k] = fp16((x[m, k] * r[m]) * gamma[k]),   r[m] = 1 / sqrt(mean_k x[m, k]^2 + eps),
// fp32 arithmetic, one rounding.  One workgroup per row; the row is read twice (the second read hits L2).
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr int kNormThreads = 256;

__global__ __launch_bounds__(kNormThreads) void rmsnorm_kernel(const half_t* __restrict__ X, int64_t K,
                                                               const half_t* __restrict__ gamma, float eps,
                                                               half_t* __restrict__ out)
{
    __shared__ float part[kNormThreads / 64];
    const half_t* __restrict__ x = X + (int64_t)blockIdx.x * K;
    half_t* __restrict__ o = out + (int64_t)blockIdx.x * K;
    const int t = threadIdx.x;
    const int pieces = (int)(K / 8);                    // K is a multiple of 32
    float ss = 0.f;
    for (int pc = t; pc < pieces; pc += kNormThreads) {
        const half8_t v = *reinterpret_cast<const half8_t*>(x + (int64_t)pc * 8);
        const half2_t x0 = {v[0], v[1]}, x1 = {v[2], v[3]}, x2 = {v[4], v[5]}, x3 = {v[6], v[7]};
        ss = __builtin_amdgcn_fdot2(x0, x0, ss, false);
        ss = __builtin_amdgcn_fdot2(x1, x1, ss, false);
        ss = __builtin_amdgcn_fdot2(x2, x2, ss, false);
        ss = __builtin_amdgcn_fdot2(x3, x3, ss, false);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) ss += __shfl_xor(ss, d);
    if ((t & 63) == 0) part[t >> 6] = ss;
    __syncthreads();
    float total = 0.f;
#pragma unroll
    for (int w = 0; w < kNormThreads / 64; ++w) total += part[w];
    const float r = 1.f / sqrtf(total / (float)K + eps);
    for (int pc = t; pc < pieces; pc += kNormThreads) {
        const half8_t v = *reinterpret_cast<const half8_t*>(x + (int64_t)pc * 8);
        const half8_t g = *reinterpret_cast<const half8_t*>(gamma + (int64_t)pc * 8);
        half8_t y;
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = (half_t)(((float)v[i] * r) * (float)g[i]);
        *reinterpret_cast<half8_t*>(o + (int64_t)pc * 8) = y;
    }
}

}  // namespace

int launch_rmsnorm(const void* X, int64_t M, int64_t K, const void* gamma, float eps, void* X_out, hipStream_t stream)
{
    if (M <= 0 || K <= 0) return E0M4_OK;
    hipLaunchKernelGGL(rmsnorm_kernel, dim3((unsigned)M), dim3(kNormThreads), 0, stream, static_cast<const half_t*>(X), K,
                       static_cast<const half_t*>(gamma), eps, static_cast<half_t*>(X_out));
    return check_launch();
}

}  // namespace e0m4
