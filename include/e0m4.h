/*
 * libe0m4 -- E0M4 FP4 weight-only quantised matrix multiplication for AMD
 * MI355X (gfx950), C ABI.
 *
 * E0M4 is the 4-bit weight format of the paper "Transformer-Lite" (section
 * "E0M4 FP4 quantization"): each group of `group` consecutive weights along K
 * is mapped by a per-group scale and bias into one fp16 binade, [2,4) here,
 * and the four highest fraction bits of the mapped fp16 value are the code.
 * Dequantisation is the paper's two bitwise operations,
 *     w1 = as_half(0x4000 | (code << 6)),
 * followed by the inverse of the group's map, w = (w1 - bias) * scale.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises; every call only enqueues kernels
 *     on `stream` (a hipStream_t passed as void*, NULL = the default stream).
 *   - fp16 is IEEE binary16.  W is [N,K] row-major (N = output features,
 *     K = input features, K contiguous), X is [M,K] row-major, Y is [M,N]
 *     row-major.
 *   - `scales` and `bias` are [N, K/group] fp16 row-major: the parameters of
 *     group g of row n are at index n*(K/group) + g.  `scale` is the
 *     dequantisation multiplier, `bias` the binade image of zero (always
 *     2 + z/8, z in 0..15).
 *   - `codes` is the packed weight buffer, an opaque device layout of
 *     e0m4_codes_bytes(N,K,group) bytes: blocks of 16 rows x 128 k, each 1 KiB
 *     of codes (one wavefront-wide 16-byte-per-lane read) followed by a copy of
 *     the block's scales and biases, ordered so that everything a block of 16
 *     output rows needs is one contiguous stream.  The kernels that consume
 *     weights (e0m4_matmul, e0m4_dequant) read the parameters from this
 *     embedded copy; the separate `scales`/`bias` arrays are the plain view of
 *     the same values.  Use e0m4_unpack_codes / e0m4_dequant to look inside.
 *   - Shape rules: 0 <= N <= 2^31, 0 <= M <= 2^31, 0 <= K <= 2^20,
 *     K % 32 == 0, K % group == 0, group in {32, 64, 128}; e0m4_matmul with
 *     M > 8 also needs N <= 2^24.  (The K limit keeps
 *     every 32-bit offset the kernels form inside one workgroup's share of the
 *     packed buffer, or inside one tile's rows of X, below 2 GiB.)  Data
 *     pointers must be 16-byte aligned.
 *   - Return value: 0 on success; a negative E0M4_ERR_* code otherwise, in
 *     which case nothing was enqueued (except E0M4_ERR_HIP, where a launch
 *     itself failed; see e0m4_last_hip_error).  Nothing throws.
 *   - Empty problems (M, N or K equal to 0) succeed and enqueue nothing,
 *     except that a matmul with K == 0 writes zeros to Y.
 */
#ifndef E0M4_H
#define E0M4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define E0M4_ABI_VERSION 4

#define E0M4_OK              0
#define E0M4_ERR_NULL      (-1)   /* a required pointer is NULL */
#define E0M4_ERR_SHAPE     (-2)   /* size negative or above its limit, K not a multiple of 32 or of group */
#define E0M4_ERR_GROUP     (-3)   /* unsupported group size */
#define E0M4_ERR_ALIGN     (-4)   /* a data pointer is not 16-byte aligned */
#define E0M4_ERR_WORKSPACE (-5)   /* workspace smaller than e0m4_workspace_bytes() */
#define E0M4_ERR_HIP       (-6)   /* the HIP runtime refused a launch */

int         e0m4_abi_version(void);
const char* e0m4_strerror(int code);
/* Text of the last HIP error seen by this thread's calls ("" if none). */
const char* e0m4_last_hip_error(void);

/* Size in bytes of the packed weight buffer:
 * ceil(N/16) * ceil(K/128) * (1024 + 64 * (128/group)).  0 on invalid shape. */
size_t e0m4_codes_bytes(int64_t N, int64_t K, int group);
/* Number of fp16 elements in `scales` (and in `bias`): N * (K/group). */
size_t e0m4_params_elems(int64_t N, int64_t K, int group);
/* Scratch bytes e0m4_matmul needs for this shape: 0 for the small-M paths
 * (partial sums stay on chip) and for GEMM shapes whose output tiles fill the GPU in whole rounds;
 * otherwise fp32 partial sums of the GEMM's split along K: splits * M * N * 4 bytes for a fixed
 * number of splits, or 1 KiB of tile counters and (256 + t) slabs of 256 KiB when the last t tiles
 * are shared out evenly over the 256 compute units (at most 128 MiB).  A pure function of the shape (0 for empty or invalid problems), unless the calling
 * thread has set a diagnostic knob (e0m4_set_knob), which then applies to its queries and calls alike. */
size_t e0m4_workspace_bytes(int64_t M, int64_t N, int64_t K, int group);

/*
 * Quantise (paper: quantization paragraph).  Per (row, group): fit scale and
 * bias from the group's min/max (range extended to contain 0; top of the
 * binade is 4 - 2^-9; bias keeps its four highest fraction bits), map every
 * weight as w/scale + bias in fp32, clamp into the binade, round once to fp16
 * and take code = min(y1 + y2, 15) from the four highest fraction bits y1 and
 * the next bit y2.  Outputs: codes (packed buffer), scales, bias.
 */
int e0m4_quantize(const void* W_f16, int64_t N, int64_t K, int group,
                  void* codes, void* scales_f16, void* bias_f16, void* stream);

/*
 * Encode only: packed buffer of W under caller-supplied scales/bias (same map,
 * clamp and rounding as e0m4_quantize, no fitting).  This is the seam for
 * weight quantisers that choose their own group parameters (the paper notes
 * E0M4 composes with GPTQ/AWQ-style methods).
 */
int e0m4_encode(const void* W_f16, int64_t N, int64_t K, int group,
                const void* scales_f16, const void* bias_f16, void* codes, void* stream);

/*
 * Dequantise (paper: dequantization formula): W_out[n,k] =
 * fp16((as_half(0x4000 | code << 6) - bias) * scale), one rounding.
 * W_out is [N,K] row-major fp16.  `scales_f16`/`bias_f16` may be NULL (the
 * packed buffer carries the parameters).
 */
int e0m4_dequant(const void* codes, const void* scales_f16, const void* bias_f16,
                 int64_t N, int64_t K, int group, void* W_f16_out, void* stream);

/* Test hook: codes_u8_out[n,k] = code of weight (n,k), one byte each, [N,K] row-major. */
int e0m4_unpack_codes(const void* codes, int64_t N, int64_t K, int group, void* codes_u8_out, void* stream);

/*
 * Y = X * dequant(codes)^T  (paper: section "Operator and lagging
 * optimizations", fp16 activation x 4-bit weight matmul; vector-matrix for
 * decode, matrix-matrix for prefill).  Dequantisation is fused in registers;
 * accumulation is fp32; Y is rounded once to fp16.
 *   M <= 8 : HBM-bound GEMV path (a workgroup owns whole blocks of 16 output
 *            rows over all of K; no partial sums leave the compute unit).
 *   2 <= M <= 16, group 128: same decomposition, the dot products run on
 *            the matrix cores so the cost stays near the weight stream for
 *            every such M.  X is staged in the LDS of the compute unit, all
 *            of it (about M * K * 2 <= 140 KiB) or one part of K after the
 *            other; the weights are read once either way.
 *   3 <= M <= 16, group 32 or 64: the same kernel with every row of X staged
 *            once per group of a block (M <= 8 at group 64, M <= 4 at group 32,
 *            where a workgroup has several row blocks or the staged rows fit
 *            the LDS), else a kernel that dequantises the weight operand in
 *            registers (when all of X fits the LDS, or M <= 8).
 *   17 <= M <= 64, group 128, N * K <= 7e7, a chunk of X within the LDS:
 *            that kernel on equal chunks of at most 16 rows in one launch,
 *            when its workgroups make at most two rounds on the compute
 *            units (three on small weights).
 *   M >= 9 otherwise, and 2 <= M <= 8 when M * N * K is about 3.8e8 or
 *            more (the vector kernel's time grows with M): MFMA GEMM path
 *            (tiles of 64 x 256, 128 x 256 or 256 x 256 outputs, whichever
 *            an estimate of the launch's duration puts ahead; split along
 *            K when tiles are few, a partly filled last round of many large
 *            tiles shared out evenly when the estimate favours that).
 *            e0m4_workspace_bytes() tells when a workspace is needed.
 * `scales_f16`/`bias_f16` may be NULL (see `codes` above); `workspace` may be
 * NULL when e0m4_workspace_bytes() is 0, else it is device memory of at least
 * that many bytes, 16-byte aligned, owned by the caller, overwritten by the
 * call and free for reuse once the call's work on `stream` has completed
 * (E0M4_ERR_WORKSPACE if too small).  The result is deterministic: every
 * reduction, the split along K included, has a fixed order.
 */
int e0m4_matmul(const void* X_f16, int64_t M,
                const void* codes, const void* scales_f16, const void* bias_f16,
                int64_t N, int64_t K, int group,
                void* Y_f16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * e0m4_matmul for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same result, bit for bit, and same argument and
 * error rules as e0m4_matmul(X, M, codes, NULL, NULL, N, K, group, Y, ...),
 * but the scratch memory of the split along K (fp32 partial sums, and the tile
 * counters of the even scheduling) is a fixed array inside the library,
 * E0M4_STATIC_SCRATCH_BYTES = 128 MiB of device memory that every GPU
 * the library runs on holds from the first use until the process ends.  The
 * call allocates and frees nothing (no hipMalloc, no allocating runtime or
 * library routine); its first call on a device looks up the array's address on
 * that device (make that call outside a graph capture).
 *   - E0M4_ERR_WORKSPACE if e0m4_workspace_bytes(M, N, K, group) exceeds the
 *     array; nothing is enqueued then.  (With the built-in choices no shape needs
 *     more than 128 MiB; only a forced number of K splits can.)
 *   - All calls on one GPU share the one array: calls whose work may overlap
 *     on that GPU (different streams, different threads) race on it; issue them on
 *     one stream or order them with events.  The array keeps the last call's
 *     contents; a call reads only what it has written itself, and zeroes the
 *     counters it uses with a small kernel of its own (no memset node: the call
 *     can be captured into a graph).
 */
#define E0M4_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
int e0m4_matmul_static(const void* X_f16, int64_t M, const void* codes, int64_t N, int64_t K, int group,
                       void* Y_f16, void* stream);

/*
 * The matmul with its neighbouring operators folded in (paper: section
 * "Operator and lagging optimizations": the small operators of rms-norm are
 * fused into one, element-wise operators are fused into the operator next to
 * them; the paper names the operators and gives no formulas, these are the
 * textbook ones):
 *   1. rms-norm of the rows of X, if `rms_gamma_f16` ([K] fp16) is not NULL:
 *        x'[m,k] = fp16(x[m,k] * gamma[k] / sqrt(mean_k x[m,k]^2 + rms_eps));
 *   2. a[m,n] = sum_k x'[m,k] * dequant(codes)[n,k], fp32 accumulation;
 *   3. epilogue E0M4_EPILOGUE_SWIGLU: the first N/2 weight rows are the gate and
 *      the last N/2 the up projection, y[m,j] = silu(a[m,j]) * a[m,N/2+j] with
 *      silu(g) = g / (1 + exp(-g)), and N_out = N/2 (N must be a multiple of
 *      64); E0M4_EPILOGUE_NONE: y = a, N_out = N;
 *   4. y += residual[m,j], if `residual_f16` ([M, N_out] fp16) is not NULL; it
 *      may be the same buffer as Y (in-place residual stream);
 *   5. Y[m,j] = fp16(y), the only rounding after step 1.  Y is [M, N_out].
 * On the decode paths (M <= 8, and the small-batch path of e0m4_matmul up to
 * M = 16) everything happens inside the one kernel; for larger M the epilogue
 * runs inside the GEMM kernels (or the kernel that adds the K splits) and the
 * rms-norm is a launch of its own that writes x' to the workspace.
 * Workspace: e0m4_fused_workspace_bytes() bytes, same rules as e0m4_matmul.
 * With no operator selected the result is that of e0m4_matmul (up to the order of
 * the fp32 additions, which the two may choose differently for a large problem).  K == 0 is
 * rejected (E0M4_ERR_SHAPE); other shape, pointer and error rules as above.
 */
#define E0M4_EPILOGUE_NONE   0
#define E0M4_EPILOGUE_SWIGLU 1
size_t e0m4_fused_workspace_bytes(int64_t M, int64_t N, int64_t K, int group, int with_rmsnorm, int epilogue);
int e0m4_matmul_fused(const void* X_f16, int64_t M, const void* rms_gamma_f16, float rms_eps,
                      const void* codes, int64_t N, int64_t K, int group,
                      int epilogue, const void* residual_f16,
                      void* Y_f16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * In-place KV-cache append (paper: section "KV cache copy optimization").  The
 * cache of a layer is ONE tensor of the maximum sequence length with the
 * sequence position as its first dimension, `cache_f16` = [max_seq, row_elems]
 * fp16 row-major (e.g. row_elems = kv_heads * head_dim, or both K and V of a
 * position side by side); the rows produced for the new tokens are written
 * where they belong instead of being concatenated to a copy of the old cache:
 *     cache[position_ids[i], e] = new_rows[i * new_ld + e],
 *         0 <= i < n_new, 0 <= e < row_elems.
 * `new_rows_f16` may be a column range of a wider matrix (the K/V columns of
 * the QKV projection's output): new_ld is the distance between consecutive new
 * rows in elements, new_ld >= row_elems.  `position_ids_i64` is a DEVICE array
 * of n_new int64 positions.  A row whose position lies outside [0, max_seq) is
 * skipped; positions must otherwise be distinct (two rows aimed at one position
 * race).  row_elems and new_ld must be multiples of 8, cache and new_rows
 * 16-byte aligned, position_ids 8-byte aligned.  Same stream and error rules as
 * the other entry points; n_new == 0 succeeds and enqueues nothing.
 */
int e0m4_kv_append(void* cache_f16, int64_t max_seq, int64_t row_elems,
                   const void* new_rows_f16, int64_t n_new, int64_t new_ld,
                   const void* position_ids_i64, void* stream);

/*
 * E0M8, the 8-bit member of the format family (paper: closing remark of the
 * section "E0M4 FP4 quantization": the approach carries over to other bit
 * widths).  The E0M4 definition with eight bits in place of four: the code is the
 * eight highest fraction bits of the mapped fp16 value plus the next one for
 * rounding, saturated at 255; w1 = as_half(0x4000 | code << 2); the bias keeps
 * its eight highest fraction bits; w = fp16((w1 - bias) * scale).
 *   - group is 64 or 128; K % 16 == 0, K % group == 0, K <= 2^19; N as above.
 *   - `codes` is a packed buffer of e0m8_codes_bytes(N, K, group) bytes: the E0M4
 *     block layout with two 4-bit slots per code, arranged so that one mask-or
 *     turns two codes into two fp16 values (blocks of 16 rows x 64 weights, each
 *     followed by a (scale, bias) word per row).  `scales`/`bias` are
 *     [N, K/group] fp16.
 *   - e0m8_unpack_codes writes one byte per weight, [N, K] row-major.
 *   - e0m8_matmul: Y[M,N] = X[M,K] * dequant(codes)^T, fp32 accumulation, one
 *     rounding.  M <= 8: the HBM-bound decode kernel (2 <= M <= 16: its
 *     matrix-core variant, any group).  M > 16 with K % 128 == 0
 *     (and N <= 2^24): the MFMA GEMM kernels, workspace of
 *     e0m8_workspace_bytes() bytes under the rules of e0m4_matmul (17 <= M <=
 *     32 with K <= 2048 and N * K <= 1e7: the matrix-core variant on two
 *     chunks of rows in one launch instead).  Other M > 16:
 *     the decode kernel on 8 rows of X at a time (needs N % 8 == 0).
 * Pointer, alignment, stream and error rules as for the E0M4 entry points.
 */
size_t e0m8_codes_bytes(int64_t N, int64_t K, int group);
int e0m8_quantize(const void* W_f16, int64_t N, int64_t K, int group,
                  void* codes, void* scales_f16, void* bias_f16, void* stream);
int e0m8_dequant(const void* codes, int64_t N, int64_t K, int group, void* W_f16_out, void* stream);
int e0m8_unpack_codes(const void* codes, int64_t N, int64_t K, int group, void* codes_u8_out, void* stream);
size_t e0m8_workspace_bytes(int64_t M, int64_t N, int64_t K, int group);
/* e0m4_matmul_fused on 8-bit codes: same operators, arguments and rules (N a multiple of 64 for the gated
 * epilogue).  M > 16 needs K % 128 == 0 (E0M4_ERR_SHAPE otherwise). */
size_t e0m8_fused_workspace_bytes(int64_t M, int64_t N, int64_t K, int group, int with_rmsnorm, int epilogue);
int e0m8_matmul_fused(const void* X_f16, int64_t M, const void* rms_gamma_f16, float rms_eps,
                      const void* codes, int64_t N, int64_t K, int group,
                      int epilogue, const void* residual_f16,
                      void* Y_f16, void* workspace, size_t workspace_bytes, void* stream);
int e0m8_matmul(const void* X_f16, int64_t M, const void* codes, int64_t N, int64_t K, int group,
                void* Y_f16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * E0M3, the 3-bit member of the format family (paper: same closing remark).  The
 * E0M4 definition with three code bits: code = min(fraction bits 9..7 of the
 * mapped fp16 value + bit 6, 7), w1 = as_half(0x4000 | code << 7) = 2 + code/4,
 * the bias keeps its three highest fraction bits.  Codes are stored in 4-bit
 * slots of the E0M4 packed buffer (e0m4_codes_bytes), a code c as 2c -- the E0M4
 * code with the same value -- so e0m4_dequant, e0m4_matmul, e0m4_matmul_fused and
 * e0m4_matmul_static serve the buffer unchanged; the storage saving of a true
 * 3-bit packing is not realised.  e0m3_unpack_codes writes the codes 0..7.
 */
int e0m3_quantize(const void* W_f16, int64_t N, int64_t K, int group,
                  void* codes, void* scales_f16, void* bias_f16, void* stream);
int e0m3_unpack_codes(const void* codes, int64_t N, int64_t K, int group, void* codes_u8_out, void* stream);

/*
 * E0M4 on bfloat16 (paper: same closing remark; the paper works the method out
 * for FP16 only).  bfloat16 has 7 fraction bits, so the code sits in fraction
 * bits 6..3: w1 = as_bfloat16(0x4000 | code << 3) = 2 + code/8, the same sixteen
 * values; the top of the binade is 4 - 2^-6 (one unit in the last place below
 * 4), rounding takes bit 2, the bias keeps bits 6..3, the scale lies between the
 * smallest normal and the largest finite bfloat16.  W, scales, bias, X and Y
 * are bfloat16 (16-bit patterns, round to nearest even); accumulation is fp32.
 * `codes` has the E0M4 layout and size (e0m4_codes_bytes; e0m4_unpack_codes
 * reads it), its embedded parameter words hold bfloat16 pairs.
 *   e0m4_bf16_matmul: M <= 8 the decode kernel with bfloat16 dot products
 *   (a shift and a mask-or per pair of codes), larger M the pipelined MFMA
 *   kernel of e0m4_matmul with the weights dequantised in registers (fp32 fused
 *   multiply-add, one rounding to bfloat16), in whole tiles (no workspace, so
 *   no split along K); when K is not a multiple of 128 an MFMA kernel with
 *   128 x 128 tiles that dequantises into LDS.
 * Shape, pointer, stream and error rules as for the E0M4 entry points.
 */
int e0m4_bf16_quantize(const void* W_bf16, int64_t N, int64_t K, int group,
                       void* codes, void* scales_bf16, void* bias_bf16, void* stream);
int e0m4_bf16_encode(const void* W_bf16, int64_t N, int64_t K, int group,
                     const void* scales_bf16, const void* bias_bf16, void* codes, void* stream);
int e0m4_bf16_dequant(const void* codes, int64_t N, int64_t K, int group, void* W_bf16_out, void* stream);
int e0m4_bf16_matmul(const void* X_bf16, int64_t M, const void* codes, int64_t N, int64_t K, int group,
                     void* Y_bf16, void* stream);

/*
 * INT4 twin (paper: section "Evaluation of FP4 quantization", Table 1 and
 * Table 2, which compare E0M4 with "INT4 quantization").  The paper does not
 * define that quantiser; this library's reading is group-wise asymmetric
 * min/max quantisation with 15 steps and an integer zero point:
 *     scale = fp16((max - min) / 15)   (range extended to contain 0),
 *     zero  = clamp(rne(-min / scale), 0, 15),
 *     q     = clamp(rne(w / scale) + zero, 0, 15),
 *     w^    = fp16((q - zero) * scale).
 * The packed buffer has the E0M4 layout (same e0m4_codes_bytes, readable with
 * e0m4_unpack_codes); its embedded parameter words hold (scale, zero).
 * `scales_f16` and `zeros_f16` are [N, K/group] fp16, zero being the integer
 * 0..15 as an fp16 number.  Same pointer, alignment, stream and error rules as
 * the E0M4 entry points.
 *
 * e0m4_int4_gemv computes Y[1,N] = X[1,K] * dequant(codes)^T like e0m4_matmul
 * at M = 1, with the same data layout, launch shape and accumulation, but it
 * turns every code into a number with an integer extraction and an integer-to-
 * float conversion instruction instead of E0M4's bit operations: the pair of
 * kernels re-runs the paper's latency comparison.  (An INT4 group with an
 * integer zero point is also a valid E0M4 group with scale' = 8 * scale and
 * bias' = 2 + zero / 8, so INT4 data can take the E0M4 path unchanged.)
 */
int e0m4_int4_quantize(const void* W_f16, int64_t N, int64_t K, int group,
                       void* codes, void* scales_f16, void* zeros_f16, void* stream);
int e0m4_int4_dequant(const void* codes, int64_t N, int64_t K, int group, void* W_f16_out, void* stream);
int e0m4_int4_gemv(const void* X_f16, const void* codes, int64_t N, int64_t K, int group, void* Y_f16, void* stream);

/*
 * Diagnostics for tuning sweeps and for tests that force every kernel variant;
 * not needed for normal use.  Sets an integer knob by name (e.g. "gemv_waves");
 * unknown names return E0M4_ERR_SHAPE.  A value of 0 restores the built-in
 * heuristic.  Knobs belong to the CALLING THREAD: they change that thread's later
 * size queries and launches only, so a query and the call it sizes always agree
 * and other threads keep the built-in choices.
 */
int e0m4_set_knob(const char* name, int value);

#ifdef __cplusplus
}
#endif
#endif /* E0M4_H */
