// Host-side internals of libe0m4: launcher prototypes shared between the C-ABI
// file and the kernel files.  Not installed; the public interface is e0m4.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "e0m4.h"

namespace e0m4 {

// Records hipGetLastError(); returns E0M4_OK or E0M4_ERR_HIP.
int check_launch();
int record_hip_error(hipError_t e);

// Raises a kernel's dynamic LDS limit, once per device (it is an attribute of the function on the current
// device).  `done` is the caller's own mask of devices that have it; safe to call from several threads.
inline int allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip_error(e);
    const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;        // devices beyond 64 are not remembered
    if (done.load(std::memory_order_acquire) & bit) return E0M4_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return record_hip_error(e);
    done.fetch_or(bit, std::memory_order_release);
    return E0M4_OK;
}

// Tuning knobs (0 = use the heuristic).
int knob(const char* name);

// Operators folded into a matmul (e0m4_matmul_fused).  All-zero is the plain matmul.
struct Fusion {
    const void* gamma = nullptr;        // [K] fp16 rms-norm weight applied to the rows of X, or null
    float eps = 0.f;                    // rms-norm epsilon
    const void* residual = nullptr;     // [M, N_out] fp16 added to the result, or null
    bool swiglu = false;                // Y[m, j] = silu(a[m, j]) * a[m, N/2 + j], N_out = N/2
    bool any() const { return gamma || residual || swiglu; }
};

struct GemvFusion;
// Device view of `f` for the decode kernels (defined in e0m4_gemv.hip).
GemvFusion make_gemv_fusion(const Fusion& f, int64_t N, int64_t K, int group);

// `format`: 0 E0M4, 1 the INT4 comparison format, 2 E0M3 (codes stored as the E0M4 codes of the same values),
// 3 E0M4 on bfloat16 (W, scales and bias are bfloat16 bit patterns).
enum { kFormatE0M4 = 0, kFormatInt4 = 1, kFormatE0M3 = 2, kFormatBf16 = 3 };
int launch_quantize(const void* W, int64_t N, int64_t K, int group, void* packed, void* scales, void* bias,
                    const void* scales_in, const void* bias_in, bool fit, int format, hipStream_t stream);
int launch_dequant(const void* packed, int64_t N, int64_t K, int group, void* W_out, int format, hipStream_t stream);
// codes_u8[n,k] = stored 4-bit code >> shift (shift 1 for 3-bit codes, which are stored doubled)
int launch_unpack(const void* packed, int64_t N, int64_t K, int group, void* out, hipStream_t stream, int shift = 0);

// Small-M path (M <= kGemvMaxM).
constexpr int kGemvMaxM = 8;
int launch_gemv(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                hipStream_t stream);
// With fused operators.  gemv_fused_supported: false when the gated epilogue meets activations that do
// not fit the LDS in one piece (the caller then takes the GEMM path).
bool gemv_fused_supported(const Fusion& f, int64_t M, int64_t N, int64_t K);
int launch_gemv_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group,
                      void* Y, hipStream_t stream);
// Small-batch path on the matrix cores: 2 <= M <= 16 at group 128, 8 at group 64, 4 at group 32.
bool gemv_mfma_supported(int64_t M, int64_t N, int64_t K, int group);
// ... and, for groups of 64 and 32, whether it is expected to beat the kernel with dequantised operands
bool gemv_mfma_groups_pay(int64_t M, int64_t N, int64_t K, int group);
// `chunks` > 1: M (17 ... 64) rows in that many equal chunks of at most 16 rows, dealt to the y dimension of one launch
int launch_gemv_mfma(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream,
                     int chunks = 1, int group = 128);
bool gemv_mfma_fused_supported(const Fusion& f, int64_t M, int64_t N, int64_t K, int group);
// ... and all M rows of X fit the LDS at once (no phases along K)
// (`workgroups`: the launch's grid, when it is)
bool gemv_mfma_whole_rows(const Fusion& f, int64_t M, int64_t N, int64_t K, int group, int64_t* workgroups = nullptr);
bool gemv_mfma8_whole_rows(const Fusion& f, int64_t M, int64_t N, int64_t K);
int launch_gemv_mfma_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                           hipStream_t stream, int chunks = 1, int group = 128);
// Small-batch path with the weight operand dequantised in registers: 2 <= M <= 64, any group (e0m4_gemv_dq.hip).
// (`whole_rows`: all M rows of X fit the LDS at once, no phases along K)
bool gemv_dq_supported(int64_t M, int64_t N, int64_t K, int group, bool* whole_rows = nullptr);
int launch_gemv_dq(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                   hipStream_t stream);
// INT4 twin of the M = 1 kernel: same layout and work decomposition, codes turned into numbers with
// integer-to-float conversion instructions.
int launch_gemv_int4(const void* X, const void* packed, int64_t N, int64_t K, int group, void* Y, hipStream_t stream);

// E0M4 on bfloat16: decode kernel (M <= 8) and small-tile MFMA kernel (any M); no workspace.
int launch_gemv_bf16(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     hipStream_t stream);
int launch_gemm_bf16(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     hipStream_t stream);

// MFMA path.
int launch_gemm(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, bool swiglu = false, bool fused = false);
// The same with the epilogue operators of `f` (residual add, gated product of the two halves of N);
// rms-norm is not applied here: X must already be normalised.
int launch_gemm_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group,
                      void* Y, void* workspace, size_t workspace_bytes, hipStream_t stream);
int launch_gemm_pipe_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group,
                           void* Y, void* workspace, size_t workspace_bytes, hipStream_t stream);
// Row-wise rms-norm of X [M, K] into X_out (fp16): the prologue of e0m4_matmul_fused for the GEMM path.
int launch_rmsnorm(const void* X, int64_t M, int64_t K, const void* gamma, float eps, void* X_out, hipStream_t stream);
// Software-pipelined 256 x 256 tile kernel (needs K % 128 == 0).  Problems with too few tiles to
// fill the chip are split along K; the fp32 partial sums ([splits][M][N]) live in the caller's
// workspace of gemm_pipe_workspace_bytes() bytes and a second kernel adds them.
bool gemm_pipe_supported(int64_t K);
size_t gemm_pipe_workspace_bytes(int64_t M, int64_t N, int64_t K, bool swiglu = false, bool fused = false);
int launch_gemm_pipe(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     void* workspace, size_t workspace_bytes, hipStream_t stream);
// The bfloat16 member on the same kernel, whole tiles only (no workspace); `pays`: enough tiles to fill the chip that way.
bool gemm_pipe_bf16_pays(int64_t M, int64_t N, int64_t K);
int launch_gemm_pipe_bf16(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                          hipStream_t stream);

// 8-bit format (E0M8): offline side and decode kernel.
int launch_quantize8(const void* W, int64_t N, int64_t K, int group, void* packed, void* scales, void* bias,
                     hipStream_t stream);
int launch_dequant8(const void* packed, int64_t N, int64_t K, void* W_out, void* codes_out, hipStream_t stream);
int launch_gemm_pipe8(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, void* workspace,
                      size_t workspace_bytes, hipStream_t stream);
bool gemv_mfma8_supported(int64_t M, int64_t N, int64_t K);
int launch_gemv_mfma8(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream,
                      int chunks = 1);
int launch_gemv8_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                       hipStream_t stream);
bool gemv_mfma8_fused_supported(const Fusion& f, int64_t M, int64_t N, int64_t K);
int launch_gemv_mfma8_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                            hipStream_t stream, int chunks = 1);
int launch_gemm_pipe8_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                            void* workspace, size_t workspace_bytes, hipStream_t stream);
int launch_gemv8(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream);

// In-place KV-cache append: cache[position_ids[i], :] = src[i, :row_elems], src rows src_ld elements apart.
int launch_kv_append(void* cache, int64_t max_seq, int64_t row_elems, const void* src, int64_t n_new, int64_t src_ld,
                     const void* position_ids, hipStream_t stream);

}  // namespace e0m4
