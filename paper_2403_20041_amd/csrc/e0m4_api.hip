// C ABI of libe0m4: argument validation and dispatch.  Every check happens on
// the host before anything is enqueued, so an error return means no kernel ran.
#include <string.h>

#include <atomic>

#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

thread_local char g_hip_error[256] = "";

// Diagnostic knobs belong to the calling thread: a size query and the call it sizes, made from one thread,
// always see the same values, and a thread that never sets a knob always gets the built-in heuristics.
struct Knob {
    const char* name;
    int value;
};
thread_local Knob g_knobs[] = {
    {"gemv_waves", 0},                 // wavefronts per workgroup of the small-M kernel (4, 8 or 16)
    {"gemv_workgroups", 0},            // target number of workgroups of the small-M kernel
    {"gemv_mfma", 0},                  // 1: never use the matrix-core small-batch kernel (2 <= M <= 16); 2: use it, activations always from LDS; 3: use it, wavefront sums reduced per row block
    {"gemv_xreg", 0},                  // M = 1 kernel, a wavefront's activations in registers: 2 never
    {"gemm_variant", 0},               // 1: small-tile kernel; pipelined kernel with tiles of 2: 256 x 256, 3: 128 x 128, 4: 64 x 256, 5: 128 x 256
    {"gemm_splits", 0},                // force the number of K splits of the pipelined GEMM kernel
    {"gemm_sk", 0},                    // even scheduling of the 256 x 256 tiles over the compute units: 1 whenever the last round is partly filled, 2 never
    {"gemm_panel", 0},                 // row tiles per panel of the pipelined GEMM's tile numbering (0: the default, -1: whole columns)
    {"gemm_split_order", 0},           // work items of a K-split launch: 1 by tile, 2 by split (0: by the length of a split)
};

// Scratch of e0m4_matmul_static: the split-K partial sums that e0m4_matmul keeps in the caller's workspace.
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = E0M4_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device, looked up once per device (in host code the array's
// name is only a handle for this lookup, never an address a kernel may use).
constexpr int kMaxTrackedDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxTrackedDevices];

int static_scratch(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip_error(e);
    if (dev >= 0 && dev < kMaxTrackedDevices) {
        void* known = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (known) {
            *out = known;
            return E0M4_OK;
        }
    }
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return record_hip_error(e);
    if (!ptr) return record_hip_error(hipErrorInvalidSymbol);
    if (dev >= 0 && dev < kMaxTrackedDevices) g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    *out = ptr;
    return E0M4_OK;
}

__global__ void zero_fill_kernel(half_t* y, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) y[i] = (half_t)0.f;
}

bool group_ok(int group) { return group == 32 || group == 64 || group == 128; }
// (gemv_mfma 1: off; 6: also for groups of 64 and 32 wherever it can run, which by default it does where it pays)
bool use_gemv_mfma(int64_t M, int64_t N, int64_t K, int group)
{
    const int k = knob("gemv_mfma");
    if (k == 1 || !gemv_mfma_supported(M, N, K, group)) return false;
    return group == 128 || k == 6 || gemv_mfma_groups_pay(M, N, K, group);
}
// The small-batch kernel with dequantised weight operands serves groups of 32 and 64 at 3 <= M <= 16 where the
// kernel above does not run (more than 8 or 4 rows) or does not pay: measured against the vector kernel and the GEMM on layer shapes of 6B and 14B
// models it is 20 - 45 % faster for 4 <= M <= 8 whatever K is, and for 9 <= M <= 16 when all of X fits the LDS
// (4608 x 4096 at M = 16: 8.9 against 13.2 us); with K in phases at those M it equals or loses to the GEMM
// (15360 x 5120 at M = 16: 22.9 against 20.2 us), and at M = 2 the vector kernel is faster.  It runs up to 64
// rows (two to four row tiles per weight operand), but from 17 rows on every workgroup stages more of X than it
// reads weights and it measured 1.3 - 5 x slower than the GEMM, so those M are not sent to it by default.
// gemv_mfma 4 forces it wherever it can run (2 <= M <= 64), 5 switches it off.
bool use_gemv_dq(int64_t M, int64_t N, int64_t K, int group)
{
    const int k = knob("gemv_mfma");
    if (k == 1 || k == 5 || M < 2) return false;
    if (k == 4) return gemv_dq_supported(M, N, K, group);
    if (group == 128 || M < 3 || M > 16) return false;
    bool whole = false;
    return gemv_dq_supported(M, N, K, group, &whole) && (whole || M <= 8);
}
// M <= kGemvMaxM rows take the vector decode kernel, whose time grows with M, unless the matrix-core GEMM
// (64 x 256 tile, time nearly independent of M) is faster: measured crossover at about M * N * K = 3.8e8
// (27392 x 4096 from M = 4 on, 4096 x 13696 from M = 7 on, never for 4096 x 4096).
bool small_m_on_vector(int64_t M, int64_t N, int64_t K)
{
    if (M > kGemvMaxM) return false;
    if (M < 2 || !gemm_pipe_supported(K) || N > (int64_t)1 << 24) return true;
    return (double)M * (double)N * (double)K < 3.8e8;
}
// 17 <= M <= kChunkedMaxM on small weights: the small-batch matrix-core kernel on equal chunks of at most 16 rows,
// dealt to the y dimension of one launch (the chunks of a workgroup's row blocks follow each other on a compute unit
// or run side by side on the same XCD: the weights come from HBM once), instead of the GEMM, whose 64 x 256 tile with
// its split along K costs 12 - 20 us whatever M is.  The launch takes about as long as one chunk times the rounds its
// workgroups make on the 256 compute units (staging a chunk of X costs a workgroup more than its weights do):
// 4608 x 4096 (144 workgroups) 7.3 us at M = 16, 11.9 at M = 32 and 12.1 at M = 48 (two rounds; GEMM 15.2 and 16.4),
// 17.0 at M = 64 (three; GEMM 17.6); 4096 x 4096 (256 workgroups) 10.8 at M = 32 (GEMM 14.8), 15.0 at M = 48 (16.1),
// 19.1 at M = 64 (four rounds; GEMM 17.1).  So: two rounds at most, or three on small weights.  Not when a chunk of X
// needs phases along K.
constexpr int64_t kChunkRows = 16, kChunkedMaxM = 64, kChunked8MaxM = 32;
int row_chunks(int64_t M) { return (int)((M + kChunkRows - 1) / kChunkRows); }
int64_t rows_per_chunk(int64_t M) { return (M + row_chunks(M) - 1) / row_chunks(M); }
bool small_batch_in_chunks(const Fusion& f, int64_t M, int64_t N, int64_t K, int group)
{
    if (M <= kChunkRows || M > kChunkedMaxM || knob("gemv_mfma") == 1 || (double)N * (double)K > 7e7) return false;
    int64_t wgs = 0;
    if (!gemv_mfma_whole_rows(f, rows_per_chunk(M), N, K, group, &wgs)) return false;
    const int64_t rounds = (row_chunks(M) * wgs + 255) / 256;
    return rounds <= 2 || (rounds == 3 && (double)N * (double)K <= 2e7);
}
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape rules shared by all entry points.
int check_shape(int64_t N, int64_t K, int group)
{
    if (!group_ok(group)) return E0M4_ERR_GROUP;
    if (N < 0 || K < 0 || (K % kCodesPerChunk) != 0 || (K % group) != 0) return E0M4_ERR_SHAPE;
    if (N > (int64_t)1 << 31 || K > (int64_t)1 << 20) return E0M4_ERR_SHAPE;   // 32-bit offsets in the kernels
    return E0M4_OK;
}

}  // namespace

int record_hip_error(hipError_t e)
{
    if (e == hipSuccess) return E0M4_OK;
    strncpy(g_hip_error, hipGetErrorString(e), sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = 0;
    return E0M4_ERR_HIP;
}

int check_launch() { return record_hip_error(hipGetLastError()); }

int knob(const char* name)
{
    for (auto& k : g_knobs)
        if (strcmp(k.name, name) == 0) return k.value;
    return 0;
}

}  // namespace e0m4

using namespace e0m4;

extern "C" {

int e0m4_abi_version(void) { return E0M4_ABI_VERSION; }

const char* e0m4_strerror(int code)
{
    switch (code) {
        case E0M4_OK: return "ok";
        case E0M4_ERR_NULL: return "a required pointer is NULL";
        case E0M4_ERR_SHAPE: return "bad shape: sizes must be >= 0 and within their limits, K a multiple of 32 and of the group size";
        case E0M4_ERR_GROUP: return "unsupported group size (supported: 32, 64, 128)";
        case E0M4_ERR_ALIGN: return "a data pointer is not 16-byte aligned";
        case E0M4_ERR_WORKSPACE: return "workspace is smaller than e0m4_workspace_bytes()";
        case E0M4_ERR_HIP: return "HIP launch failed (see e0m4_last_hip_error)";
        default: return "unknown error code";
    }
}

const char* e0m4_last_hip_error(void) { return g_hip_error; }

size_t e0m4_codes_bytes(int64_t N, int64_t K, int group)
{
    if (check_shape(N, K, group) != E0M4_OK) return 0;
    return (size_t)row_blocks(N) * (size_t)k_blocks(K) * (size_t)block_bytes(group);
}

size_t e0m4_params_elems(int64_t N, int64_t K, int group)
{
    if (check_shape(N, K, group) != E0M4_OK) return 0;
    return (size_t)N * (size_t)(K / group);
}

size_t e0m4_workspace_bytes(int64_t M, int64_t N, int64_t K, int group)
{
    if (check_shape(N, K, group) != E0M4_OK || M <= 0 || N == 0 || K == 0) return 0;             // invalid or empty: nothing runs
    if (small_m_on_vector(M, N, K)) return 0;           // the small-M kernels need none
    if (use_gemv_dq(M, N, K, group)) return 0;
    if (use_gemv_mfma(M, N, K, group) || small_batch_in_chunks(Fusion{}, M, N, K, group)) return 0;
    return gemm_workspace_bytes(M, N, K);       // partial tiles of the split-K GEMM, if it splits
}

// Fused matmul: the normalised copy of X (GEMM path with rms-norm) comes first in the workspace,
// rounded up to 256 bytes, then the partial sums of the split along K.
static size_t norm_bytes(int64_t M, int64_t K) { return ((size_t)M * (size_t)K * 2 + 255) & ~(size_t)255; }

// Which kernel family serves a fused matmul: 0 the decode kernel, 2 the small-batch kernel on the matrix
// cores (both: everything in one launch), 3 that kernel on two chunks of rows, 1 the GEMM kernels (rms-norm,
// if any, as a launch of its own before them).
static int fused_path(const Fusion& f, int64_t M, int64_t N, int64_t K, int group)
{
    // (groups of 64 and 32 from three rows on: 1.1 - 2 x the vector kernel and the GEMM there, 10 - 25 % slower than the
    // vector kernel at two rows)
    if (knob("gemv_mfma") != 1 && gemv_mfma_fused_supported(f, M, N, K, group) &&
        (group == 128 || M >= 3 || knob("gemv_mfma") == 6))
        return 2;
    if (small_batch_in_chunks(f, M, N, K, group)) return 3;
    return (small_m_on_vector(M, N, K) && gemv_fused_supported(f, M, N, K)) ? 0 : 1;
}

size_t e0m4_fused_workspace_bytes(int64_t M, int64_t N, int64_t K, int group, int with_rmsnorm, int epilogue)
{
    if (check_shape(N, K, group) != E0M4_OK || M <= 0 || N == 0 || K == 0) return 0;
    if (epilogue != E0M4_EPILOGUE_NONE && epilogue != E0M4_EPILOGUE_SWIGLU) return 0;
    Fusion f;
    f.swiglu = epilogue == E0M4_EPILOGUE_SWIGLU;
    if (fused_path(f, M, N, K, group) != 1) return 0;
    return (with_rmsnorm ? norm_bytes(M, K) : 0) + gemm_workspace_bytes(M, N, K, f.swiglu, true);
}

int e0m4_set_knob(const char* name, int value)
{
    if (!name) return E0M4_ERR_NULL;
    for (auto& k : g_knobs)
        if (strcmp(k.name, name) == 0) {
            k.value = value;
            return E0M4_OK;
        }
    return E0M4_ERR_SHAPE;
}

int e0m4_quantize(const void* W, int64_t N, int64_t K, int group, void* codes, void* scales, void* bias, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !bias) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(bias)) return E0M4_ERR_ALIGN;
    return launch_quantize(W, N, K, group, codes, scales, bias, nullptr, nullptr, true, kFormatE0M4, (hipStream_t)stream);
}

int e0m4_encode(const void* W, int64_t N, int64_t K, int group, const void* scales, const void* bias, void* codes,
                void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !bias) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(bias)) return E0M4_ERR_ALIGN;
    return launch_quantize(W, N, K, group, codes, nullptr, nullptr, scales, bias, false, kFormatE0M4, (hipStream_t)stream);
}

int e0m4_dequant(const void* codes, const void* scales, const void* bias, int64_t N, int64_t K, int group, void* W_out,
                 void* stream)
{
    (void)scales; (void)bias;                   // the packed buffer carries its own copy of the parameters
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W_out || !codes) return E0M4_ERR_NULL;
    if (!aligned16(W_out) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    return launch_dequant(codes, N, K, group, W_out, kFormatE0M4, (hipStream_t)stream);
}

int e0m4_int4_quantize(const void* W, int64_t N, int64_t K, int group, void* codes, void* scales, void* zeros,
                       void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !zeros) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(zeros)) return E0M4_ERR_ALIGN;
    return launch_quantize(W, N, K, group, codes, scales, zeros, nullptr, nullptr, true, kFormatInt4, (hipStream_t)stream);
}

int e0m4_int4_dequant(const void* codes, int64_t N, int64_t K, int group, void* W_out, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W_out || !codes) return E0M4_ERR_NULL;
    if (!aligned16(W_out) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    return launch_dequant(codes, N, K, group, W_out, kFormatInt4, (hipStream_t)stream);
}

int e0m4_int4_gemv(const void* X, const void* codes, int64_t N, int64_t K, int group, void* Y, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0) return E0M4_OK;
    if (!Y) return E0M4_ERR_NULL;
    if (!aligned16(Y)) return E0M4_ERR_ALIGN;
    if (K == 0) {                                   // empty contraction: Y = 0
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                           static_cast<half_t*>(Y), N);
        return check_launch();
    }
    if (!X || !codes) return E0M4_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    return launch_gemv_int4(X, codes, N, K, group, Y, (hipStream_t)stream);
}

int e0m4_unpack_codes(const void* codes, int64_t N, int64_t K, int group, void* out, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!codes || !out) return E0M4_ERR_NULL;
    if (!aligned16(codes) || !aligned16(out)) return E0M4_ERR_ALIGN;
    return launch_unpack(codes, N, K, group, out, (hipStream_t)stream);
}

int e0m4_matmul(const void* X, int64_t M, const void* codes, const void* scales, const void* bias, int64_t N, int64_t K,
                int group, void* Y, void* workspace, size_t workspace_bytes, void* stream)
{
    (void)scales; (void)bias;
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (M < 0 || M > (int64_t)1 << 31) return E0M4_ERR_SHAPE;
    if (M == 0 || N == 0) return E0M4_OK;
    if (!Y) return E0M4_ERR_NULL;
    if (!aligned16(Y)) return E0M4_ERR_ALIGN;
    if (K == 0) {                                   // empty contraction: Y = 0
        const int64_t total = M * N;
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                           static_cast<half_t*>(Y), total);
        return check_launch();
    }
    if (!X || !codes) return E0M4_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    if (knob("gemv_mfma") == 4 && use_gemv_dq(M, N, K, group))
        return launch_gemv_dq(X, M, codes, N, K, group, Y, (hipStream_t)stream);
    if (use_gemv_mfma(M, N, K, group)) return launch_gemv_mfma(X, M, codes, N, K, Y, (hipStream_t)stream, 1, group);
    if (use_gemv_dq(M, N, K, group)) return launch_gemv_dq(X, M, codes, N, K, group, Y, (hipStream_t)stream);
    if (small_m_on_vector(M, N, K)) return launch_gemv(X, M, codes, N, K, group, Y, (hipStream_t)stream);
    if (small_batch_in_chunks(Fusion{}, M, N, K, group))
        return launch_gemv_mfma(X, M, codes, N, K, Y, (hipStream_t)stream, row_chunks(M), group);
    if (N > (int64_t)1 << 24) return E0M4_ERR_SHAPE;    // the GEMM epilogue forms 32-bit offsets of up to 256 rows of Y
    if (workspace_bytes > 0 && (!workspace || !aligned16(workspace))) return workspace ? E0M4_ERR_ALIGN : E0M4_ERR_NULL;
    return launch_gemm(X, M, codes, N, K, group, Y, workspace, workspace_bytes, (hipStream_t)stream);
}

int e0m4_matmul_static(const void* X, int64_t M, const void* codes, int64_t N, int64_t K, int group, void* Y, void* stream)
{
    // the shape decides the scratch size before anything else is looked at; nothing is allocated anywhere below
    const size_t need = e0m4_workspace_bytes(M, N, K, group);
    if (need > kStaticScratchBytes) return E0M4_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0) {
        const int rc = static_scratch(&ws);
        if (rc != E0M4_OK) return rc;
    }
    return e0m4_matmul(X, M, codes, nullptr, nullptr, N, K, group, Y, ws, need, stream);
}

int e0m4_matmul_fused(const void* X, int64_t M, const void* rms_gamma, float rms_eps, const void* codes, int64_t N,
                      int64_t K, int group, int epilogue, const void* residual, void* Y, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (M < 0 || M > (int64_t)1 << 31) return E0M4_ERR_SHAPE;
    if (epilogue != E0M4_EPILOGUE_NONE && epilogue != E0M4_EPILOGUE_SWIGLU) return E0M4_ERR_SHAPE;
    Fusion f;
    f.gamma = rms_gamma;
    f.eps = rms_eps;
    f.residual = residual;
    f.swiglu = epilogue == E0M4_EPILOGUE_SWIGLU;
    // the gated epilogue pairs weight row j with row N/2 + j: the halves must be whole pairs of 16-row blocks
    if (f.swiglu && (N % (4 * kBlockRows)) != 0) return E0M4_ERR_SHAPE;
    if (M == 0 || N == 0) return E0M4_OK;
    if (K == 0) return E0M4_ERR_SHAPE;                  // nothing to normalise or to gate
    if (!X || !codes || !Y) return E0M4_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes) || !aligned16(Y) || (rms_gamma && !aligned16(rms_gamma)) ||
        (residual && !aligned16(residual)))
        return E0M4_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int path = fused_path(f, M, N, K, group);
    if (path == 2) return launch_gemv_mfma_fused(f, X, M, codes, N, K, Y, st, 1, group);
    if (path == 0) return launch_gemv_fused(f, X, M, codes, N, K, group, Y, st);
    if (path == 3) return launch_gemv_mfma_fused(f, X, M, codes, N, K, Y, st, row_chunks(M), group);      // rows are independent
    if (N > (int64_t)1 << 24) return E0M4_ERR_SHAPE;    // 32-bit offsets in the GEMM epilogue
    const size_t nb = rms_gamma ? norm_bytes(M, K) : 0;
    const size_t need = nb + gemm_workspace_bytes(M, N, K, f.swiglu, true);
    if (need > 0) {
        if (!workspace) return E0M4_ERR_NULL;
        if (!aligned16(workspace)) return E0M4_ERR_ALIGN;
        if (workspace_bytes < need) return E0M4_ERR_WORKSPACE;
    }
    const void* x = X;
    if (rms_gamma) {
        rc = launch_rmsnorm(X, M, K, rms_gamma, rms_eps, workspace, st);
        if (rc != E0M4_OK) return rc;
        x = workspace;
        f.gamma = nullptr;
    }
    return launch_gemm_fused(f, x, M, codes, N, K, group, Y, static_cast<char*>(workspace) + nb,
                             workspace_bytes - nb, st);
}

// ---- E0M3: the 3-bit member of the family, stored in 4-bit slots ---------------------------------------
int e0m3_quantize(const void* W, int64_t N, int64_t K, int group, void* codes, void* scales, void* bias, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !bias) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(bias)) return E0M4_ERR_ALIGN;
    return launch_quantize(W, N, K, group, codes, scales, bias, nullptr, nullptr, true, kFormatE0M3, (hipStream_t)stream);
}

int e0m3_unpack_codes(const void* codes, int64_t N, int64_t K, int group, void* out, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!codes || !out) return E0M4_ERR_NULL;
    if (!aligned16(codes) || !aligned16(out)) return E0M4_ERR_ALIGN;
    return launch_unpack(codes, N, K, group, out, (hipStream_t)stream, 1);
}

// ---- E0M4 on bfloat16 ----------------------------------------------------------------------------------
int e0m4_bf16_quantize(const void* W, int64_t N, int64_t K, int group, void* codes, void* scales, void* bias,
                       void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !bias) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(bias)) return E0M4_ERR_ALIGN;
    return launch_quantize(W, N, K, group, codes, scales, bias, nullptr, nullptr, true, kFormatBf16, (hipStream_t)stream);
}

int e0m4_bf16_encode(const void* W, int64_t N, int64_t K, int group, const void* scales, const void* bias, void* codes,
                     void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !bias) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(bias)) return E0M4_ERR_ALIGN;
    return launch_quantize(W, N, K, group, codes, nullptr, nullptr, scales, bias, false, kFormatBf16, (hipStream_t)stream);
}

int e0m4_bf16_dequant(const void* codes, int64_t N, int64_t K, int group, void* W_out, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W_out || !codes) return E0M4_ERR_NULL;
    if (!aligned16(W_out) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    return launch_dequant(codes, N, K, group, W_out, kFormatBf16, (hipStream_t)stream);
}

int e0m4_bf16_matmul(const void* X, int64_t M, const void* codes, int64_t N, int64_t K, int group, void* Y, void* stream)
{
    int rc = check_shape(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (M < 0 || M > (int64_t)1 << 31) return E0M4_ERR_SHAPE;
    if (M == 0 || N == 0) return E0M4_OK;
    if (!Y) return E0M4_ERR_NULL;
    if (!aligned16(Y)) return E0M4_ERR_ALIGN;
    if (K == 0) {                                   // empty contraction: Y = +0 (the same bits in both formats)
        const int64_t total = M * N;
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                           static_cast<half_t*>(Y), total);
        return check_launch();
    }
    if (!X || !codes) return E0M4_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    if (M <= kGemvMaxM) return launch_gemv_bf16(X, M, codes, N, K, group, Y, (hipStream_t)stream);
    if (N > (int64_t)1 << 24) return E0M4_ERR_SHAPE;    // 32-bit offsets in the GEMM epilogue
    return launch_gemm_bf16(X, M, codes, N, K, group, Y, (hipStream_t)stream);
}

// ---- E0M8: the 8-bit member of the format family ------------------------------------------------------
static int check_shape8(int64_t N, int64_t K, int group)
{
    if (group != 64 && group != 128) return E0M4_ERR_GROUP;
    if (N < 0 || K < 0 || (K % 16) != 0 || (K % group) != 0) return E0M4_ERR_SHAPE;
    if (N > (int64_t)1 << 31 || K > (int64_t)1 << 19) return E0M4_ERR_SHAPE;   // 2K 4-bit slots within the K limit
    return E0M4_OK;
}

size_t e0m8_codes_bytes(int64_t N, int64_t K, int group)
{
    if (check_shape8(N, K, group) != E0M4_OK) return 0;
    return (size_t)row_blocks(N) * (size_t)k_blocks(2 * K) * (size_t)block_bytes(128);
}

int e0m8_quantize(const void* W, int64_t N, int64_t K, int group, void* codes, void* scales, void* bias, void* stream)
{
    int rc = check_shape8(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!W || !codes || !scales || !bias) return E0M4_ERR_NULL;
    if (!aligned16(W) || !aligned16(codes) || !aligned16(scales) || !aligned16(bias)) return E0M4_ERR_ALIGN;
    return launch_quantize8(W, N, K, group, codes, scales, bias, (hipStream_t)stream);
}

int e0m8_dequant(const void* codes, int64_t N, int64_t K, int group, void* W_out, void* stream)
{
    int rc = check_shape8(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!codes || !W_out) return E0M4_ERR_NULL;
    if (!aligned16(codes) || !aligned16(W_out)) return E0M4_ERR_ALIGN;
    return launch_dequant8(codes, N, K, W_out, nullptr, (hipStream_t)stream);
}

int e0m8_unpack_codes(const void* codes, int64_t N, int64_t K, int group, void* out, void* stream)
{
    int rc = check_shape8(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (N == 0 || K == 0) return E0M4_OK;
    if (!codes || !out) return E0M4_ERR_NULL;
    if (!aligned16(codes) || !aligned16(out)) return E0M4_ERR_ALIGN;
    return launch_dequant8(codes, N, K, nullptr, out, (hipStream_t)stream);
}

// The pipelined GEMM serves M > 8 when K is a multiple of 128 (its K slices come in pairs).
static bool e0m8_use_mfma_decode(int64_t M, int64_t N, int64_t K)
{
    return knob("gemv_mfma") != 1 && gemv_mfma8_supported(M, N, K);
}

// The 8-bit form of small_batch_in_chunks.  Twice the weight bytes per launch: the two launches only win on
// small weights with short rows (2048 x 2048: 9 against 11 us, 8192 x 1024: 10 against 10.7; 4096 x 4096 equal,
// 512 x 4096 and larger weights 5 - 20 % slower).
static bool small_batch8_in_chunks(const Fusion& f, int64_t M, int64_t N, int64_t K)
{
    return M > kChunkRows && M <= kChunked8MaxM && knob("gemv_mfma") != 1 && K <= 2048 && (double)N * (double)K <= 1e7 &&
           gemv_mfma8_whole_rows(f, rows_per_chunk(M), N, K);
}

static bool e0m8_use_gemm(int64_t M, int64_t N, int64_t K)
{
    return !e0m8_use_mfma_decode(M, N, K) && !small_batch8_in_chunks(Fusion{}, M, N, K) && !small_m_on_vector(M, N, K) &&
           gemm_pipe_supported(K) && N <= (int64_t)1 << 24;
}

size_t e0m8_workspace_bytes(int64_t M, int64_t N, int64_t K, int group)
{
    if (check_shape8(N, K, group) != E0M4_OK || M <= 0 || N == 0 || K == 0) return 0;
    return e0m8_use_gemm(M, N, K) ? gemm_pipe_workspace_bytes(M, N, K, false, true) : 0;
}

int e0m8_matmul(const void* X, int64_t M, const void* codes, int64_t N, int64_t K, int group, void* Y, void* workspace,
                size_t workspace_bytes, void* stream)
{
    int rc = check_shape8(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (M < 0 || M > (int64_t)1 << 31) return E0M4_ERR_SHAPE;
    if (M == 0 || N == 0) return E0M4_OK;
    if (!Y) return E0M4_ERR_NULL;
    if (!aligned16(Y)) return E0M4_ERR_ALIGN;
    if (K == 0) {
        const int64_t total = M * N;
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                           static_cast<half_t*>(Y), total);
        return check_launch();
    }
    if (!X || !codes) return E0M4_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes)) return E0M4_ERR_ALIGN;
    if (e0m8_use_mfma_decode(M, N, K)) return launch_gemv_mfma8(X, M, codes, N, K, Y, (hipStream_t)stream);
    if (small_batch8_in_chunks(Fusion{}, M, N, K))
        return launch_gemv_mfma8(X, M, codes, N, K, Y, (hipStream_t)stream, row_chunks(M));
    if (e0m8_use_gemm(M, N, K)) {
        if (workspace_bytes > 0 && (!workspace || !aligned16(workspace))) return workspace ? E0M4_ERR_ALIGN : E0M4_ERR_NULL;
        return launch_gemm_pipe8(X, M, codes, N, K, Y, workspace, workspace_bytes, (hipStream_t)stream);
    }
    if (M > kGemvMaxM && ((N % 8) != 0)) return E0M4_ERR_SHAPE;    // row chunks of Y must stay 16-byte aligned
    // otherwise up to 8 rows of X per launch of the decode kernel
    for (int64_t m0 = 0; m0 < M; m0 += kGemvMaxM) {
        const int64_t rows = M - m0 < kGemvMaxM ? M - m0 : kGemvMaxM;
        rc = launch_gemv8(static_cast<const half_t*>(X) + m0 * K, rows, codes, N, K, static_cast<half_t*>(Y) + m0 * N,
                          (hipStream_t)stream);
        if (rc != E0M4_OK) return rc;
    }
    return E0M4_OK;
}

// Fused matmul on 8-bit codes: 2 the small-batch kernel, 0 the decode kernel, 1 the GEMM kernels (K % 128 == 0), -1 none.
static int fused_path8(const Fusion& f, int64_t M, int64_t N, int64_t K)
{
    if (knob("gemv_mfma") != 1 && gemv_mfma8_fused_supported(f, M, N, K)) return 2;
    if (small_batch8_in_chunks(f, M, N, K)) return 3;
    if (small_m_on_vector(M, N, K) && gemv_fused_supported(f, M, N, 2 * K)) return 0;
    return gemm_pipe_supported(K) && N <= (int64_t)1 << 24 ? 1 : -1;
}

size_t e0m8_fused_workspace_bytes(int64_t M, int64_t N, int64_t K, int group, int with_rmsnorm, int epilogue)
{
    if (check_shape8(N, K, group) != E0M4_OK || M <= 0 || N == 0 || K == 0) return 0;
    if (epilogue != E0M4_EPILOGUE_NONE && epilogue != E0M4_EPILOGUE_SWIGLU) return 0;
    Fusion f;
    f.swiglu = epilogue == E0M4_EPILOGUE_SWIGLU;
    if (fused_path8(f, M, N, K) != 1) return 0;
    return (with_rmsnorm ? norm_bytes(M, K) : 0) + gemm_pipe_workspace_bytes(M, N, K, f.swiglu, true);
}

int e0m8_matmul_fused(const void* X, int64_t M, const void* rms_gamma, float rms_eps, const void* codes, int64_t N,
                      int64_t K, int group, int epilogue, const void* residual, void* Y, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    int rc = check_shape8(N, K, group);
    if (rc != E0M4_OK) return rc;
    if (M < 0 || M > (int64_t)1 << 31) return E0M4_ERR_SHAPE;
    if (epilogue != E0M4_EPILOGUE_NONE && epilogue != E0M4_EPILOGUE_SWIGLU) return E0M4_ERR_SHAPE;
    Fusion f;
    f.gamma = rms_gamma;
    f.eps = rms_eps;
    f.residual = residual;
    f.swiglu = epilogue == E0M4_EPILOGUE_SWIGLU;
    if (f.swiglu && (N % (4 * kBlockRows)) != 0) return E0M4_ERR_SHAPE;
    if (M == 0 || N == 0) return E0M4_OK;
    if (K == 0) return E0M4_ERR_SHAPE;
    if (!X || !codes || !Y) return E0M4_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes) || !aligned16(Y) || (rms_gamma && !aligned16(rms_gamma)) ||
        (residual && !aligned16(residual)))
        return E0M4_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int path = fused_path8(f, M, N, K);
    if (path == 2) return launch_gemv_mfma8_fused(f, X, M, codes, N, K, Y, st);
    if (path == 0) return launch_gemv8_fused(f, X, M, codes, N, K, Y, st);
    if (path == 3) return launch_gemv_mfma8_fused(f, X, M, codes, N, K, Y, st, row_chunks(M));
    if (path != 1) return E0M4_ERR_SHAPE;               // larger M needs K % 128 == 0 (GEMM kernels)
    const size_t nb = rms_gamma ? norm_bytes(M, K) : 0;
    const size_t need = nb + gemm_pipe_workspace_bytes(M, N, K, f.swiglu, true);
    if (need > 0) {
        if (!workspace) return E0M4_ERR_NULL;
        if (!aligned16(workspace)) return E0M4_ERR_ALIGN;
        if (workspace_bytes < need) return E0M4_ERR_WORKSPACE;
    }
    const void* x = X;
    if (rms_gamma) {
        rc = launch_rmsnorm(X, M, K, rms_gamma, rms_eps, workspace, st);
        if (rc != E0M4_OK) return rc;
        x = workspace;
        f.gamma = nullptr;
    }
    return launch_gemm_pipe8_fused(f, x, M, codes, N, K, Y, static_cast<char*>(workspace) + nb, workspace_bytes - nb, st);
}

int e0m4_kv_append(void* cache, int64_t max_seq, int64_t row_elems, const void* new_rows, int64_t n_new,
                   int64_t new_ld, const void* position_ids, void* stream)
{
    if (max_seq < 0 || row_elems < 0 || n_new < 0 || (row_elems % 8) != 0 || (new_ld % 8) != 0 || new_ld < row_elems)
        return E0M4_ERR_SHAPE;
    if (row_elems > (int64_t)1 << 31 || max_seq > (int64_t)1 << 40 || n_new > (int64_t)1 << 31) return E0M4_ERR_SHAPE;
    if (n_new == 0 || row_elems == 0 || max_seq == 0) return E0M4_OK;
    if (!cache || !new_rows || !position_ids) return E0M4_ERR_NULL;
    if (!aligned16(cache) || !aligned16(new_rows) || (reinterpret_cast<uintptr_t>(position_ids) & 7u) != 0)
        return E0M4_ERR_ALIGN;
    return launch_kv_append(cache, max_seq, row_elems, new_rows, n_new, new_ld, position_ids, (hipStream_t)stream);
}

}  // extern "C"
