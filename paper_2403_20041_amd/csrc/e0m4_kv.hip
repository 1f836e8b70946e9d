// In-place KV-cache append (paper: section "KV cache copy optimization").  The cache is one tensor of the
// maximum sequence length with the sequence position as its first dimension, [max_seq, row] fp16; the
// rows produced for the new tokens (a column range of the QKV projection's output, hence the source row
// stride) are written at the positions given by position_ids, so old cache and new rows are never
// concatenated or copied.  One thread moves 16 bytes; a row outside [0, max_seq) is skipped.
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr int kKvThreads = 256;

__global__ __launch_bounds__(kKvThreads) void kv_append_kernel(uint4* __restrict__ cache, int64_t max_seq,
                                                               int row_pieces, const uint4* __restrict__ src,
                                                               int64_t n_new, int64_t src_ld_pieces,
                                                               const int64_t* __restrict__ position_ids)
{
    const int64_t idx = (int64_t)blockIdx.x * kKvThreads + threadIdx.x;
    if (idx >= n_new * row_pieces) return;
    const int64_t i = idx / row_pieces;
    const int pc = (int)(idx - i * row_pieces);
    const int64_t pos = position_ids[i];
    if (pos < 0 || pos >= max_seq) return;
    cache[pos * row_pieces + pc] = src[i * src_ld_pieces + pc];
}

}  // namespace

int launch_kv_append(void* cache, int64_t max_seq, int64_t row_elems, const void* src, int64_t n_new, int64_t src_ld,
                     const void* position_ids, hipStream_t stream)
{
    const int64_t row_pieces = row_elems / 8, total = n_new * row_pieces;
    if (total == 0) return E0M4_OK;
    const int64_t blocks = (total + kKvThreads - 1) / kKvThreads;
    if (blocks > 0x7fffffffLL) return E0M4_ERR_SHAPE;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(kKvThreads), 0, stream, static_cast<uint4*>(cache),
                       max_seq, (int)row_pieces, static_cast<const uint4*>(src), n_new, src_ld / 8,
                       static_cast<const int64_t*>(position_ids));
    return check_launch();
}

}  // namespace e0m4
