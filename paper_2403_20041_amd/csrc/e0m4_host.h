// Host-side internals of libe0m4: launcher prototypes shared between the C-ABI
// file and the kernel files.  Not installed; the public interface is e0m4.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "e0m4.h"

namespace e0m4 {

// Records hipGetLastError(); returns E0M4_OK or E0M4_ERR_HIP.
int check_launch();
int record_hip_error(hipError_t e);

// Tuning knobs (0 = use the heuristic).
int knob(const char* name);

int launch_quantize(const void* W, int64_t N, int64_t K, int group, void* packed, void* scales, void* bias,
                    const void* scales_in, const void* bias_in, bool fit, bool int4, hipStream_t stream);
int launch_dequant(const void* packed, int64_t N, int64_t K, int group, void* W_out, bool int4, hipStream_t stream);
int launch_unpack(const void* packed, int64_t N, int64_t K, int group, void* out, hipStream_t stream);

// Small-M path (M <= kGemvMaxM).
constexpr int kGemvMaxM = 8;
int launch_gemv(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                hipStream_t stream);
// Small-batch path on the matrix cores: 3 <= M <= 16, group 128, X must fit the LDS of one compute unit.
bool gemv_mfma_supported(int64_t M, int64_t N, int64_t K, int group);
int launch_gemv_mfma(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream);
// INT4 twin of the M = 1 kernel: same layout and work decomposition, codes turned into numbers with
// integer-to-float conversion instructions.
int launch_gemv_int4(const void* X, const void* packed, int64_t N, int64_t K, int group, void* Y, hipStream_t stream);

// MFMA path.
int launch_gemm(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
// Software-pipelined 256 x 256 tile kernel (needs K % 128 == 0).  Problems with too few tiles to
// fill the chip are split along K; the fp32 partial sums ([splits][M][N]) live in the caller's
// workspace of gemm_pipe_workspace_bytes() bytes and a second kernel adds them.
bool gemm_pipe_supported(int64_t K);
size_t gemm_pipe_workspace_bytes(int64_t M, int64_t N, int64_t K);
int64_t gemm_pipe_work_items(int64_t M, int64_t N, int64_t K);      // tiles x K splits
int launch_gemm_pipe(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     void* workspace, size_t workspace_bytes, hipStream_t stream);

}  // namespace e0m4
