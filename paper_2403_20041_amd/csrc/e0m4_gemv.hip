// Decode path of e0m4_matmul: Y[M,N] = X[M,K] * dequant(packed)^T for M <= 8.
// Paper: section "Operator and lagging optimizations" (vector-matrix product
// of the decoding stage, bound by memory bandwidth) with the dequantisation of
// section "E0M4 FP4 quantization" fused in registers.
//
// Work decomposition (gfx950, wave64): a workgroup owns a few consecutive blocks
// of 16 output rows over the whole of K, so no partial sums ever leave the
// compute unit and no second kernel, atomics or scratch memory are needed.  Its
// W wavefronts take the 16 x 128 weight blocks of that contiguous run
// round-robin and keep several in flight; each block is one dwordx4 load per
// lane (1 KiB contiguous per wavefront) plus one dword of group parameters.
// Lane q*16 + r holds 32 codes of row r: it turns them into the raw binade
// values w1 = 2 + code/8 with a shift and a mask-or per pair, accumulates
// a = sum x*w1 with v_dot2_f32_f16 against activations staged in LDS, and
// applies the group's affine map once per block:
//     y += scale * (a - bias * sum x).
// The four k-quarters of a row are added with two cross-lane steps, the
// wavefronts' sums through LDS in a fixed order (deterministic result).
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kXBudgetBytes = 48 * 1024;        // LDS spent on activations and their chunk sums
constexpr int kRedBudgetBytes = 16 * 1024;      // LDS spent on the per-wavefront partial sums
constexpr int kBytesPerBlockX = kBlockK * 2 + (kBlockK / kCodesPerChunk) * 8;   // 288 per row of X per k block
constexpr int kTargetWorkgroups = 512;          // two resident workgroups of 16 wavefronts per compute unit
constexpr int kDepth = 4;                       // weight blocks in flight per wavefront
constexpr int kEarlyX = 2;                      // activation pieces per thread requested before the weights

struct GemvPlan {
    int waves;          // wavefronts per workgroup
    int seg_blocks;     // k blocks whose activations are resident in LDS at a time (multiple of waves)
    int rb_per_wg;      // consecutive row blocks owned by one workgroup
    int64_t grid;
    size_t lds_bytes;
};

GemvPlan make_plan(int64_t M, int64_t N, int64_t K)
{
    GemvPlan p;
    const int64_t nrb = row_blocks(N), nkb = k_blocks(K);
    int w = knob("gemv_waves");
    // 16 wavefronts per row block when there is at most one row block per compute unit (that is the
    // only parallelism there is); 8 otherwise (measured faster) and for many rows of X, whose
    // accumulators need the larger register budget of the smaller workgroup
    if (w != 4 && w != 8 && w != 16) w = (M <= 4 && nrb <= 256) ? 16 : 8;
    while (w > 4 && w > nkb) w /= 2;                          // a wavefront steps W k blocks at a time
    p.waves = w;
    int64_t max_blocks = kXBudgetBytes / (M * kBytesPerBlockX) / w * w;
    if (max_blocks < w) max_blocks = w;
    const int64_t need = (nkb + w - 1) / w * w;
    const bool single_segment = need <= max_blocks;
    p.seg_blocks = (int)(single_segment ? need : max_blocks);
    int64_t t_max = kRedBudgetBytes / ((int64_t)w * M * kBlockRows * sizeof(float));
    if (t_max < 1) t_max = 1;
    int target = knob("gemv_workgroups");
    if (target <= 0) target = kTargetWorkgroups * 8 / w;      // 16 wavefronts resident per compute unit
    int64_t t = (nrb + target - 1) / target;
    if (t > t_max) t = t_max;
    if (t < 1 || !single_segment) t = 1;       // several activation segments: one row block per workgroup
    p.rb_per_wg = (int)t;                       // the most row blocks any workgroup owns
    // Row blocks are dealt out evenly: workgroup b owns [b * nrb / grid, (b + 1) * nrb / grid).  When
    // the target number of workgroups can be reached with at most t row blocks each, use exactly the
    // target (every compute unit then holds the same number of workgroups); else the fewest that do.
    p.grid = (nrb + t - 1) / t;
    if (t > 1 && p.grid < target && (int64_t)target * t >= nrb) p.grid = target;
    p.lds_bytes = (size_t)M * p.seg_blocks * kBytesPerBlockX + (size_t)t * w * M * kBlockRows * sizeof(float);
    return p;
}

// A workgroup owns `rb_per_wg` consecutive row blocks; its work items are their weight blocks in
// memory order (row block major, k block minor).  Wavefront w takes items w, w+W, w+2W, ... and
// keeps a ring of D of them in flight.  VARIANT != 0 are timing experiments (wrong results).
template <int G, int M, int W, bool SMALLK = false, int VARIANT = 0, int OCC = 1>
__global__ __launch_bounds__(W * 64, OCC) void gemv_kernel(const half_t* __restrict__ X,
                                                           const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                           half_t* __restrict__ Y, int seg_blocks, int rb_per_wg)
{
    constexpr int kThreads = W * 64;
    // fewer blocks in flight when the accumulators need the registers
    constexpr int D = VARIANT == 3 ? 8 : (VARIANT == 4 ? 6 : (M <= 2 ? kDepth : (M <= 4 ? 3 : 2)));
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int seg_k = seg_blocks * kBlockK;
    half_t* xs = reinterpret_cast<half_t*>(smem);                               // [M][seg_k]
    // per 32-wide chunk of X: (sum of the chunk, 30 x sum of its elements with k % 8 in 2..5)
    float2* sxs = reinterpret_cast<float2*>(smem + (size_t)M * seg_k * 2);      // [M][seg_k/32]
    float* red = reinterpret_cast<float*>(sxs + (size_t)M * (seg_k / kCodesPerChunk));   // [rb_per_wg][W][M][16]

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int q = lane >> 4, r = lane & 15;
    const uint32_t fmask = frac_mask_vgpr(), fmask_low = frac_mask_low_vgpr();
    const PackedLayout<G> lay(K);
    const int nkb = (int)lay.nkb;
    const int64_t nrb = row_blocks(N);
    const int64_t rb0 = (int64_t)blockIdx.x * nrb / gridDim.x;      // even deal of row blocks (<= rb_per_wg each)
    const int n_rb = (int)((int64_t)(blockIdx.x + 1) * nrb / gridDim.x - rb0);
    const int nitems = n_rb * nkb;
    // Weights are read with buffer loads: a wavefront-uniform resource (base of this workgroup's run
    // of row blocks, far smaller than 2 GiB), a scalar offset per block and a constant lane offset.
    const __amdgpu_buffer_rsrc_t wg_codes = make_rsrc(packed + lay.code_index(rb0, 0));
    const __amdgpu_buffer_rsrc_t wg_params = make_rsrc(reinterpret_cast<const char*>(packed) + 4 * lay.param_index(rb0, 0));
    const uint32_t rb_stride = (uint32_t)nkb * block_bytes(G);                  // bytes from one row block to the next
    const uint32_t lane_code_off = lane * 16, lane_param_off = lay.param_slot(q, r) * 4;
    // step a (row block slot, k block) cursor by W items; W <= nkb unless SMALLK
    auto advance = [&](int& s_, int& k_) {
        k_ += W;
        if (SMALLK) {
            while (k_ >= nkb) { k_ -= nkb; ++s_; }
        } else if (k_ >= nkb) {
            k_ -= nkb;
            ++s_;
        }
    };

    // ---- activations of the first segment: request them before the weights so that they are not
    // queued behind a ring full of weight blocks (loads return in order)
    const int pieces = seg_k / 8;                       // 16-byte pieces per row of X per segment
    auto x_piece = [&](int idx, int sb) {
        const int m = idx / pieces, pc = idx % pieces;
        const int64_t k = (int64_t)sb * kBlockK + pc * 8;
        half8_t v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (VARIANT < 5 && idx < M * pieces && k < K) v = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + k);
        return v;
    };
    // store one piece and, from every fourth lane, the two sums of its 32-wide chunk (a piece is the
    // k range of one code word: elements 2..5 meet the code pairs that are read at 1/128 scale)
    auto x_store = [&](int idx, const half8_t& v) {
        const int m = idx / pieces, pc = idx % pieces;
        const half2_t ones = {(half_t)1.f, (half_t)1.f};
        const half2_t x0 = {v[0], v[1]}, x1 = {v[2], v[3]}, x2 = {v[4], v[5]}, x3 = {v[6], v[7]};
        float sl = __builtin_amdgcn_fdot2(x1, ones, 0.f, false);
        sl = __builtin_amdgcn_fdot2(x2, ones, sl, false);
        float s = __builtin_amdgcn_fdot2(x0, ones, sl, false);
        s = __builtin_amdgcn_fdot2(x3, ones, s, false);
        s += __shfl_xor(s, 1);
        sl += __shfl_xor(sl, 1);
        s += __shfl_xor(s, 2);
        sl += __shfl_xor(sl, 2);
        if (VARIANT < 5 && idx < M * pieces) {
            *reinterpret_cast<half8_t*>(&xs[m * seg_k + pc * 8]) = v;
            if ((pc & 3) == 0) sxs[m * (seg_k / kCodesPerChunk) + (pc >> 2)] = make_float2(s, 30.f * sl);
        }
    };
    half8_t xearly[kEarlyX];
#pragma unroll
    for (int e = 0; e < kEarlyX; ++e) xearly[e] = x_piece(t + e * kThreads, 0);

    // ---- ring of weight blocks
    uint4 c[D];
    uint32_t pw[D];
    int fs = 0, fk = wave;                              // fetch cursor (row block slot, k block)
    if (SMALLK) while (fk >= nkb) { fk -= nkb; ++fs; }
    auto fetch = [&](uint4& cd, uint32_t& pwd) {        // past the end the last block is read again
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, k_ = in ? fk : nkb - 1;
        const uint32_t row_off = __builtin_amdgcn_readfirstlane(s_ * rb_stride);
        const u32x4 cv = __builtin_amdgcn_raw_buffer_load_b128(wg_codes, (int)lane_code_off,
                                                               (int)(row_off + k_ * kBlockCodeBytes), 0);
        cd = make_uint4(cv.x, cv.y, cv.z, cv.w);
        if (VARIANT >= 6) pwd = 0x3c003c00u;
        else
            pwd = __builtin_amdgcn_raw_buffer_load_b32(wg_params, (int)lane_param_off,
                                                       (int)(row_off + k_ * (4 * lay.kParamWords)), 0);
        advance(fs, fk);
    };
#pragma unroll
    for (int d = 0; d < D; ++d) fetch(c[d], pw[d]);

    int i = wave;                                       // current item, as flat index and (row block slot, k block)
    int slot = 0, kb = wave;
    if (SMALLK) while (kb >= nkb) { kb -= nkb; ++slot; }

    for (int j = t; j < n_rb * W * M * kBlockRows; j += kThreads) red[j] = 0.f;

    float acc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] = 0.f;

    // add the four k-quarters of each row and park the wavefront's sums for row block `sl`
    auto flush = [&](int sl) {
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float v = acc[m];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < kBlockRows) red[((sl * W + wave) * M + m) * kBlockRows + lane] = v;
            acc[m] = 0.f;
        }
    };

    for (int sb = 0; sb < nkb; sb += seg_blocks) {
        // stage the segment's activations and the sum of every 32-wide chunk
        if (sb == 0) {
#pragma unroll
            for (int e = 0; e < kEarlyX; ++e) x_store(t + e * kThreads, xearly[e]);
            if (VARIANT < 5)
                for (int idx = t + kEarlyX * kThreads; idx < M * pieces; idx += kThreads) x_store(idx, x_piece(idx, 0));
        } else {
            __syncthreads();                            // everyone is done with the previous segment's activations
            fs = slot;                                  // refill the ring from the current item
            fk = kb;
#pragma unroll
            for (int d = 0; d < D; ++d) fetch(c[d], pw[d]);
            for (int idx = t; idx < M * pieces; idx += kThreads) x_store(idx, x_piece(idx, sb));
        }
        if (VARIANT < 5) __syncthreads();

        // one item: its codes and parameter word are in a ring slot
        auto process = [&](const uint4& cd, const uint32_t pwd) {
            const float sc = (float)param_scale(pwd);
            const float bi = (float)param_bias(pwd);
            const uint32_t words[4] = {cd.x, cd.y, cd.z, cd.w};
            const int xoff = (kb - sb) * kBlockK + q * kCodesPerChunk;
            float a[M][2];          // per row of X: sum x*(2 + c/8) over code pairs 0 and 3, sum x*(2 + c/128) over 1 and 2
#pragma unroll
            for (int m = 0; m < M; ++m) a[m][0] = a[m][1] = 0.f;
            if (VARIANT == 1 || VARIANT >= 5) {         // timing experiment: stream only, no arithmetic
                acc[0] += __builtin_bit_cast(float, words[0] ^ words[1] ^ words[2] ^ words[3]) * sc;
            } else {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    half2_t p[4];
                    w1_pairs_mixed(words[w], fmask, fmask_low, p);
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        half8_t xv;
                        if (VARIANT == 2) xv = half8_t{1, 1, 1, 1, 1, 1, 1, 1};     // timing experiment: no LDS reads
                        else xv = *reinterpret_cast<const half8_t*>(&xs[m * seg_k + xoff + 8 * w]);
                        const half2_t x0 = {xv[0], xv[1]}, x1 = {xv[2], xv[3]}, x2 = {xv[4], xv[5]}, x3 = {xv[6], xv[7]};
                        a[m][0] = __builtin_amdgcn_fdot2(p[0], x0, a[m][0], false);
                        a[m][1] = __builtin_amdgcn_fdot2(p[1], x1, a[m][1], false);
                        a[m][1] = __builtin_amdgcn_fdot2(p[2], x2, a[m][1], false);
                        a[m][0] = __builtin_amdgcn_fdot2(p[3], x3, a[m][0], false);
                    }
                }
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    // sum x*w1 = a0 + 16*a1 - 30*(sum of x over pairs 1 and 2); then the group's affine map
                    const float2 sx = VARIANT == 2 ? make_float2(32.f, 480.f) : sxs[m * (seg_k / kCodesPerChunk) + (xoff >> 5)];
                    acc[m] += sc * ((a[m][0] + 16.f * a[m][1] - sx.y) - bi * sx.x);
                }
            }
            i += W;
            const int prev = slot;
            advance(slot, kb);
            if (VARIANT < 7 && slot != prev) flush(prev);       // the next item belongs to a later row block
        };

        // with one segment the loop runs over all items; otherwise (one row block) up to the segment's end
        const int limit = seg_blocks >= nkb ? nitems : min(sb + seg_blocks, nkb);
        // Entering the steady-state loop with nothing but the ring outstanding lets the compiler's
        // wait-count bookkeeping keep D blocks in flight across the back edge (vmcnt(0), others free).
        __builtin_amdgcn_s_waitcnt(0x0F70);
        while (i + (D - 1) * W < limit) {               // full turns of the ring, refilled as it is consumed
#pragma unroll
            for (int d = 0; d < D; ++d) {
                process(c[d], pw[d]);
                fetch(c[d], pw[d]);
            }
        }
#pragma unroll
        for (int d = 0; d < D; ++d)                     // last partial turn
            if (i < limit) process(c[d], pw[d]);
    }
    if (VARIANT >= 7) {
        if (acc[0] == 1.2345f) Y[t] = (half_t)acc[0];
        return;
    }
    if (slot < n_rb) flush(slot);                       // sums of a row block this wavefront left unfinished (several segments)
    __syncthreads();
    for (int idx = t; idx < n_rb * M * kBlockRows; idx += kThreads) {
        const int sl = idx / (M * kBlockRows), m = (idx / kBlockRows) % M, rr = idx % kBlockRows;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) s += red[((sl * W + w) * M + m) * kBlockRows + rr];
        const int64_t n = (rb0 + sl) * kBlockRows + rr;
        if (n < N) Y[(int64_t)m * N + n] = (half_t)s;
    }
}

template <int G, int M, int W>
int launch_one(const GemvPlan& p, const void* X, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    const dim3 grid((unsigned)p.grid), block(W * 64);
    const int dbg = (G == 128 && M == 1 && W >= 8) ? knob("gemv_debug") : 0;     // timing experiments only
    if (W == 4 && k_blocks(K) < W)                      // K < 512: the generic cursor
        hipLaunchKernelGGL((gemv_kernel<G, M, 4, true>), grid, block, p.lds_bytes, stream, x, c, N, K, y, p.seg_blocks,
                           p.rb_per_wg);
    else if (dbg == 1)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 1>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (dbg == 2)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 2>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (dbg == 3)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 3>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (dbg == 4)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 4>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (dbg == 5)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 5>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (dbg == 6)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 6>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (dbg == 7)
        hipLaunchKernelGGL((gemv_kernel<128, 1, W, false, 7>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else if (M == 1 && knob("gemv_occ") == 8)           // experiment: cap registers for 8 wavefronts per SIMD
        hipLaunchKernelGGL((gemv_kernel<G, 1, W, false, 0, 8>), grid, block, p.lds_bytes, stream, x, c, N, K, y,
                           p.seg_blocks, p.rb_per_wg);
    else
        hipLaunchKernelGGL((gemv_kernel<G, M, W>), grid, block, p.lds_bytes, stream, x, c, N, K, y, p.seg_blocks,
                           p.rb_per_wg);
    return check_launch();
}

template <int G, int M>
int launch_w(const GemvPlan& p, const void* X, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream)
{
    switch (p.waves) {
        case 4: return launch_one<G, M, 4>(p, X, packed, N, K, Y, stream);
        case 8: return launch_one<G, M, 8>(p, X, packed, N, K, Y, stream);
        default: return launch_one<G, M, 16>(p, X, packed, N, K, Y, stream);
    }
}

template <int G>
int launch_m(const GemvPlan& p, int64_t M, const void* X, const void* packed, int64_t N, int64_t K, void* Y,
             hipStream_t stream)
{
    switch (M) {
        case 1: return launch_w<G, 1>(p, X, packed, N, K, Y, stream);
        case 2: return launch_w<G, 2>(p, X, packed, N, K, Y, stream);
        case 3: return launch_w<G, 3>(p, X, packed, N, K, Y, stream);
        case 4: return launch_w<G, 4>(p, X, packed, N, K, Y, stream);
        case 5: return launch_w<G, 5>(p, X, packed, N, K, Y, stream);
        case 6: return launch_w<G, 6>(p, X, packed, N, K, Y, stream);
        case 7: return launch_w<G, 7>(p, X, packed, N, K, Y, stream);
        case 8: return launch_w<G, 8>(p, X, packed, N, K, Y, stream);
        default: return E0M4_ERR_SHAPE;
    }
}

}  // namespace

int launch_gemv(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                hipStream_t stream)
{
    const GemvPlan p = make_plan(M, N, K);
    switch (group) {
        case 32: return launch_m<32>(p, M, X, packed, N, K, Y, stream);
        case 64: return launch_m<64>(p, M, X, packed, N, K, Y, stream);
        case 128: return launch_m<128>(p, M, X, packed, N, K, Y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

}  // namespace e0m4
