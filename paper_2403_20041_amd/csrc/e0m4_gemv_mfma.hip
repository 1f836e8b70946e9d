// Small-batch decode path of e0m4_matmul: Y[M,N] = X[M,K] * dequant(packed)^T for 2 <= M <= 16 and
// group size 128.  Paper: section "Operator and lagging optimizations" (vector-matrix product of the
// decoding stage, bound by memory bandwidth) with the dequantisation of section "E0M4 FP4
// quantization" fused in registers.
//
// Same work decomposition as the M = 1 kernel (a workgroup owns whole 16-row blocks over all of K, a
// work item is four consecutive 16 x 128 weight blocks, the next item is in flight while the current
// one is processed), but the dot products run on the matrix cores: per weight block four
// v_mfma_f32_16x16x32_f16 compute the 16 (rows of X, padded) x 16 (weight rows) products over the
// block's 128 k, so the vector work per block (bit operations on the codes, the group's affine map)
// no longer grows with M and the kernel stays close to the memory stream for every M up to 16.
//
// Operands.  The weight operand of an MFMA is taken straight from the lane's 16-byte chunk: lane
// (n = l%16, q = l/16) owns the 32 codes of weight row n, k = 32q..32q+31, and supplies 8 of them per
// MFMA, which is exactly the k-group layout of the instruction (lane l supplies k-group l/16).  The
// code pairs that read 2 + c/8 after the mask-or (pairs 0 and 3 of a word) and those that read
// 2 + c/128 (pairs 1 and 2) go to separate MFMAs and accumulators, and are folded back with
//     sum x*(2 + c/8) = 16 * sum x*(2 + c/128) - 30 * sum x       (over the k of pairs 1 and 2).
// The activation operand comes from LDS, where X is staged once per workgroup in the order the
// MFMAs consume it (one 16-byte unit per MFMA and lane); the two sums per (row of X, block) that the
// factored form needs are MFMAs of the same operands with an all-ones weight operand.
// One group of 128 k is one block, so the group's affine map  y += scale * (a - bias * sum x)  is
// applied once per block on the MFMA result.
//
// Groups of 64 and 32 (GS = 2 or 4 groups per block; at most 8 or 4 rows of X).  A lane's 32 codes lie inside one
// group (k-groups 2g and 2g + 1 of the block belong to group g of two, k-group g to group g of four), but an MFMA
// adds all four k-groups.  So every row m of X is staged GS times, as row m + (16 / GS) * g with everything but the
// k-groups of group g set to zero: the sixteen rows of the MFMA then hold, per group, the sums over that group
// alone (the all-ones MFMAs likewise), the four output rows of a lane belong to one group, whose parameters the
// lane picks, and the GS rows of a row of X are added when the wavefront sums are.  The loop over the weights is
// the same as for one group per block.
//
// Long rows.  When M rows of X exceed the LDS, K is walked in phases: a phase stages its part of X,
// visits that part of every row block of the workgroup and adds to the wavefront sums, which stay in
// LDS until the last phase.  The weight stream is the same, each byte once; what a phase costs is
// the barrier before X is replaced and the restart of the wavefronts' prefetch.
#include "e0m4_device.h"
#include "e0m4_host.h"

#include <algorithm>

namespace e0m4 {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSuper = 4;                       // weight blocks (of 128 k) per work item
constexpr int kG = 128;                         // group size: one group per block
constexpr int kMinM = 2;                         // a single row is faster on the vector kernel
constexpr int kMaxM = 16;
constexpr int kPW = block_param_words(kG);      // 16 parameter words per block
constexpr int kXBlockBytes = kBlockK * 2;       // one row of X, one block: 256 bytes
constexpr int kRowPadBytes = 16;                // keeps the 16 rows of X in different LDS bank groups
constexpr int kLdsLimitBytes = 156 * 1024;      // of the 160 KiB of a compute unit
constexpr int kTargetWorkgroups = 256;          // one workgroup per compute unit

struct MfmaPlan {
    int late;                                   // reduce the wavefront sums once at the end (they fit the LDS)
    int waves;
    int step_slots, step_item;                  // a wavefront's next work item: W items ahead, as (row blocks, items) with carry
    int rb_base, rb_rem;                        // even deal of row blocks
    int64_t grid;
    size_t lds_bytes;
    uint32_t pieces_magic;                      // ceil(2^32 / pieces of 8 activations per row): row of a piece by multiplication
    // X longer than the LDS holds: K is walked in phases of kb_phase blocks (a multiple of kSuper; 0: one phase),
    // each phase stages its part of X and visits all row blocks of the workgroup
    int kb_phase;
    uint32_t pieces_magic_last;                 // the same for the (shorter) last phase
};

constexpr int kNormBytes = (16 + 1) * kMaxM * 4;        // rms-norm: per-wavefront sums of squares and the row scales

// (nkb blocks of 128 4-bit codes or of 64 8-bit codes: 256 or 128 bytes of X per row and block)
size_t lds_need(int64_t M, int64_t nkb, int waves, bool e8 = false)
{
    return (size_t)M * (nkb * (e8 ? kXBlockBytes / 2 : kXBlockBytes) + kRowPadBytes) +
           2 * (size_t)waves * kMaxM * kBlockRows * sizeof(float) + kNormBytes;
}

// LDS for the wavefront sums of all `slots` row blocks of a workgroup at once
size_t late_red_bytes(int64_t M, int slots, int waves)
{
    return (size_t)slots * waves * M * kBlockRows * sizeof(float);
}

// Byte offset, inside one block of one row of X, of the 8-byte half-unit that holds the elements of
// word w (k = 8w..8w+7 of chunk q) for the MFMA of pair set hl (0: elements 0,1,6,7; 1: elements 2..5).
__device__ inline int x_unit_off(int q, int w, int hl) { return ((q * 4 + (w >> 1) * 2 + hl) << 4) + ((w & 1) << 3); }

// FUSED adds the operators of GemvFusion (e0m4_device.h): rms-norm while X is staged, the gated epilogue
// (the workgroup owns pairs of a gate and an up row block and writes silu(gate) * up), the residual add.
// XREG: the wavefront count is a multiple of the work items per row block, so a wavefront meets the same
// four k blocks in every row block and keeps their activation operands in registers (64 per lane)
// instead of reading them from LDS for every weight block.
// E8: the 8-bit format E0M8 (e0m8_pack.hip).  A block holds 64 weights, a lane's chunk 16, and one MFMA
// takes the eight weights of two words per lane, each word turned into two pairs of binade values by a
// mask-or and a rotation; there is only one kind of code slot, so one accumulator and the plain sum of X.
// PHASED: M rows of X do not fit the LDS.  K is walked in phases of kb_phase blocks: every phase stages its
// part of X, visits all row blocks of the workgroup and adds to the wavefront sums, which stay in LDS
// (`late`) until the last phase.  The weights are still read exactly once.
template <int W, bool FUSED, bool XREG, bool E8 = false, bool PHASED = false, int GS = 1>
__global__ __launch_bounds__(W * 64) void gemv_mfma_kernel(const half_t* __restrict__ X,
                                                           const uint4* __restrict__ packed, half_t* __restrict__ Y,
                                                           int M, uint32_t N32, uint32_t K32, int step_slots_arg,
                                                           int step_item_arg, int rb_base, int rb_rem, int late,
                                                           uint32_t pieces_magic_arg, int kb_phase,
                                                           uint32_t pieces_magic_last, GemvFusion fu)
{
    // (the arguments up to `late` fill the 14 scalar registers the launch can preload; N <= 2^31, K <= 2^20)
    const int64_t N = N32, K = K32;
    // Row chunks: workgroups with blockIdx.y = c do rows c * M ... of X (rows are independent, the rms-norm and the
    // epilogues included).  The chunks of one set of row blocks run one after the other on a compute unit, or side by
    // side on two of the same XCD, so the second reads the weights from L2.
    if (gridDim.y > 1) {
        const int row0 = (int)blockIdx.y * M;
        const int64_t ylen = (FUSED && fu.swiglu) ? fu.n_out : N;
        X += (int64_t)row0 * K;
        Y += (int64_t)row0 * ylen;
        if (FUSED && fu.residual) fu.residual += (int64_t)row0 * ylen;
        M = min(M, fu.m_total - row0);
    }
    static_assert(!(PHASED && XREG), "a wavefront meets other k blocks in every phase");
    static_assert(GS == 1 || ((GS == 2 || GS == 4) && !E8 && !XREG), "several groups per block: 4-bit codes, X from LDS");
    constexpr int kThreads = W * 64;
    constexpr int G = kG / GS;                          // group size
    constexpr int PW = kPW * GS;                        // parameter words per block
    constexpr int SLOT = kMaxM / GS;                    // MFMA rows per group (GS > 1): row m of X is rows m + SLOT * g
    const int Ms = GS == 1 ? M : (GS - 1) * SLOT + M;   // staged rows of X
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int XBB = E8 ? kXBlockBytes / 2 : kXBlockBytes;   // bytes of X per row and block
    constexpr int UB = E8 ? 16 : 32;                            // bytes per (k-group, MFMA pair) unit of a block
    const PackedLayout<G> lay(E8 ? 2 * K : K);
    const int nkb = (int)lay.nkb;
    const int nkb_lds = PHASED ? kb_phase : nkb;        // k blocks of X that the LDS holds at a time
    const int n_ph = PHASED ? (nkb + kb_phase - 1) / kb_phase : 1;
    const int row_stride = nkb_lds * XBB + kRowPadBytes;
    unsigned char* xs = smem;                                                   // [M] rows of X in MFMA order
    float* norm_part = reinterpret_cast<float*>(smem + (size_t)Ms * row_stride); // [W][16] sums of squares, then [16] row scales
    // wavefront sums: [2][W][16 m][16 n], reduced row block by row block; or, when `late` (LDS permitting),
    // [row blocks][W][M][16 n], reduced once at the end without a barrier per row block
    float* red = norm_part + kNormBytes / 4;

    if (PHASED) late = 1;                               // the sums of a row block are complete after the last phase only
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n_l = lane & 15, g_l = lane >> 4;         // weight row / k-group of this lane; also (row of X, k-group)
    const uint32_t fmask = frac_mask_vgpr(), fmask_low = frac_mask_low_vgpr();
    // even deal of row blocks; gated: of pairs of row blocks (rb0 is then the pair, i.e. its gate row block)
    const bool gated = FUSED && fu.swiglu;
    const int64_t rb0 = (int64_t)blockIdx.x * rb_base + min((int)blockIdx.x, rb_rem);
    const int n_rb = (rb_base + ((int)blockIdx.x < rb_rem ? 1 : 0)) * (gated ? 2 : 1);
    const __amdgpu_buffer_rsrc_t wg_codes = make_rsrc(packed + lay.code_index(rb0, 0));
    const __amdgpu_buffer_rsrc_t wg_params = make_rsrc(reinterpret_cast<const char*>(packed) + 4 * lay.param_index(rb0, 0));
    const uint32_t rb_stride = (uint32_t)nkb * block_bytes(G);
    const uint32_t lane_code_off = lane * 16;
    const int param_words_rb = nkb * PW;
    auto slot_off = [&](uint32_t s_) -> uint32_t {      // byte offset of row block slot s from the first row block
        if (FUSED && fu.swiglu) return (s_ >> 1) * rb_stride + (s_ & 1) * fu.half_bytes;
        return s_ * rb_stride;
    };

    // ---- per phase: the k blocks [kb_lo, kb_lo + nkb_ph) of every row block, as nsi work items per row block
    int kb_lo = 0, nkb_ph = nkb, nsi = (nkb + kSuper - 1) / kSuper;
    int step_slots = step_slots_arg, step_item = step_item_arg;
    auto advance = [&](int& s_, int& i_) {              // W work items ahead
        s_ += step_slots;
        i_ += step_item;
        if (i_ >= nsi) {
            i_ -= nsi;
            ++s_;
        }
    };
    int slot = 0, si = 0;                               // current work item: row block slot, item inside the row block
    int nslot = 0, nitem = 0;                           // the one after it (in flight)

    // ---- the work item in flight: four code blocks and their 64 parameter words (one per lane)
    uint4 c[kSuper];
    uint32_t pwraw[GS];                                 // the item's 64 * GS parameter words: word 64 n + lane in pwraw[n]
    auto fetch_params = [&](int fs, int fi) {           // past the end the last item is read again
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, i_ = in ? fi : nsi - 1;
        const uint32_t first = (uint32_t)kb_lo * PW + i_ * (kSuper * PW);       // the item's first parameter word
        const uint32_t soff = __builtin_amdgcn_readfirstlane(slot_off(s_) + first * 4);
        const int last = param_words_rb - 1 - (int)first;
#pragma unroll
        for (int n = 0; n < GS; ++n)
            pwraw[n] = __builtin_amdgcn_raw_buffer_load_b32(wg_params, min(n * 64 + lane, last) * 4, (int)soff, 0);
    };
    auto fetch_code = [&](int j, int fs, int fi) {      // k blocks beyond K: the last block again (left out of the sums)
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, i_ = in ? fi : nsi - 1;
        const uint32_t kb = min((uint32_t)kb_lo + i_ * kSuper + j, (uint32_t)nkb - 1);
        const uint32_t soff = __builtin_amdgcn_readfirstlane(slot_off(s_) + kb * kBlockCodeBytes);
        const u32x4 cv = __builtin_amdgcn_raw_buffer_load_b128(wg_codes, (int)lane_code_off, (int)soff, 0);
        c[j] = make_uint4(cv.x, cv.y, cv.z, cv.w);
    };
    auto first_item = [&]() {                           // of a phase: where this wavefront starts, and its first requests
        slot = 0;
        si = wave;
        while (si >= nsi) {
            si -= nsi;
            ++slot;
        }
        nslot = slot;
        nitem = si;
        advance(nslot, nitem);
        fetch_params(slot, si);
#pragma unroll
        for (int j = 0; j < kSuper; ++j) fetch_code(j, slot, si);
    };
    if (PHASED) {
        nkb_ph = min(kb_phase, nkb);
        nsi = (nkb_ph + kSuper - 1) / kSuper;
        step_slots = W / nsi;
        step_item = W % nsi;
    }
    first_item();

    // ---- stage X in pieces of 8 elements (k = 8*pc .. 8*pc+7 of row m); no piece index needs a division
    const int pieces = nkb * (XBB / 16);
    const bool normed = FUSED && fu.gamma != nullptr;
    const int cpr = (pieces + kThreads - 1) / kThreads;        // chunks per row
    constexpr int kStageBatch = W >= 16 ? 4 : 8;        // loads in flight per thread and staging step (register budget)
    const half8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    // XREG with every k block in exactly one wavefront (step_slots == 1): a wavefront needs only the pieces of its
    // own four k blocks, also for the rms-norm, since the row's sum of squares is the sum of the wavefronts' own.
    // The pieces (one per lane and row of X) stay in registers until the row scales are known.
    constexpr int kItemPieces = kSuper * XBB / 16;      // pieces of one row of X per work item: 64 (32 for 8-bit codes)
    // (not with sixteen wavefronts: 64 more registers do not fit their budget of 128)
    const bool own_norm = W <= 8 && normed && XREG && step_slots == 1;
    const int pc_own = si * kItemPieces + lane;
    const bool own_ok = lane < kItemPieces && pc_own < pieces;      // (a last work item may reach beyond the row's blocks)
    half8_t keep[kMaxM], g_own = zero8;
    if (own_norm) {
        const bool in_k = own_ok && (int64_t)pc_own * 8 < K;
#pragma unroll
        for (int m = 0; m < kMaxM; ++m) {
            keep[m] = zero8;
            if (m < M && in_k) keep[m] = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + (int64_t)pc_own * 8);
        }
        if (in_k) g_own = *reinterpret_cast<const half8_t*>(fu.gamma + (int64_t)pc_own * 8);
#pragma unroll
        for (int m0 = 0; m0 < kMaxM; m0 += 8) {         // eight rows' reductions at a time (their latencies overlap)
            if (m0 >= M) break;
            float sq[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const half8_t v = keep[m0 + r];
                const half2_t x0 = {v[0], v[1]}, x1 = {v[2], v[3]}, x2 = {v[4], v[5]}, x3 = {v[6], v[7]};
                float d = __builtin_amdgcn_fdot2(x0, x0, 0.f, false);
                d = __builtin_amdgcn_fdot2(x1, x1, d, false);
                d = __builtin_amdgcn_fdot2(x2, x2, d, false);
                sq[r] = __builtin_amdgcn_fdot2(x3, x3, d, false);
            }
#pragma unroll
            for (int d = 1; d < 64; d <<= 1)
#pragma unroll
                for (int r = 0; r < 8; ++r) sq[r] += __shfl_xor(sq[r], d);
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (m0 + r < M) norm_part[wave * kMaxM + m0 + r] = sq[r];
            }
        }
    }
    if (normed && !own_norm) {
        // rms-norm: sum of squares of every row (first pass over X; the staging pass below reads it again,
        // from the cache), reduced in a fixed order: lanes, then wavefronts;
        // kNormRows rows at a time: their loads are in flight together and their wavefront reductions (chains of
        // cross-lane steps, each with the latency of an LDS access) overlap instead of running row after row
        constexpr int kNormRows = 8;
        for (int m0 = 0; m0 < M; m0 += kNormRows) {
            float sq[kNormRows];
#pragma unroll
            for (int r = 0; r < kNormRows; ++r) sq[r] = 0.f;
            for (int c0 = 0; c0 < cpr; ++c0) {
                const int pc = c0 * kThreads + t;
                const int64_t k = (int64_t)pc * 8;
                half8_t vb[kNormRows];
#pragma unroll
                for (int r = 0; r < kNormRows; ++r) {
                    vb[r] = zero8;
                    if (m0 + r < M && pc < pieces && k < K) vb[r] = *reinterpret_cast<const half8_t*>(X + (int64_t)(m0 + r) * K + k);
                }
#pragma unroll
                for (int r = 0; r < kNormRows; ++r) {
                    const half8_t v = vb[r];
                    const half2_t x0 = {v[0], v[1]}, x1 = {v[2], v[3]}, x2 = {v[4], v[5]}, x3 = {v[6], v[7]};
                    float d = __builtin_amdgcn_fdot2(x0, x0, sq[r], false);
                    d = __builtin_amdgcn_fdot2(x1, x1, d, false);
                    d = __builtin_amdgcn_fdot2(x2, x2, d, false);
                    sq[r] = __builtin_amdgcn_fdot2(x3, x3, d, false);
                }
            }
#pragma unroll
            for (int d = 1; d < 64; d <<= 1)
#pragma unroll
                for (int r = 0; r < kNormRows; ++r) sq[r] += __shfl_xor(sq[r], d);
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < kNormRows; ++r)
                    if (m0 + r < M) norm_part[wave * kMaxM + m0 + r] = sq[r];
            }
        }
    }
    if (normed) {                                       // the wavefronts' sums, in wavefront order, then the row scales
        __syncthreads();
        float tot = 0.f;
        if (t < M) {
#pragma unroll
            for (int w = 0; w < W; ++w) tot += norm_part[w * kMaxM + t];
        }
        __syncthreads();
        if (t < M) norm_part[t] = 1.f / sqrtf(tot / (float)K + fu.eps);
        __syncthreads();
    }
    // one piece into the LDS image of X, in the order the MFMAs consume it
    auto store_piece = [&](int m, int pc, bool ok, half8_t v, const half8_t& g) {
        if (!ok) return;
        if (normed) {                                   // (x * row scale) * gamma, one rounding
            const float r = norm_part[m];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (half_t)(((float)v[i] * r) * (float)g[i]);
        }
        if (E8) {                                       // piece = the 8 weights of (k-group q, MFMA wp)
            const int kb = pc >> 3, q = (pc >> 1) & 3, wp = pc & 1;
            *reinterpret_cast<half8_t*>(xs + (size_t)m * row_stride + kb * XBB + q * 2 * UB + wp * UB) = v;
        } else {
            const int kb = pc >> 4, q = (pc >> 2) & 3, w = pc & 3;
            const half4_t hpart = {v[0], v[1], v[6], v[7]}, lpart = {v[2], v[3], v[4], v[5]};
            const half4_t none = {0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < GS; ++g) {              // (GS > 1: the piece in the row of its own group, zeros in the others)
                const bool own = GS == 1 || g == q * GS / 4;
                unsigned char* blk = xs + (size_t)(m + SLOT * g) * row_stride + kb * XBB;
                *reinterpret_cast<half4_t*>(blk + x_unit_off(q, w, 0)) = own ? hpart : none;
                *reinterpret_cast<half4_t*>(blk + x_unit_off(q, w, 1)) = own ? lpart : none;
            }
        }
    };
    for (int ph = 0; ph < n_ph; ++ph) {
        if (PHASED && ph > 0) {
            kb_lo = ph * kb_phase;
            nkb_ph = min(kb_phase, nkb - kb_lo);
            nsi = (nkb_ph + kSuper - 1) / kSuper;
            step_slots = W / nsi;
            step_item = W % nsi;
            first_item();                               // its requests are in flight while X is staged
            __syncthreads();                            // every wavefront has finished with the previous part of X
        }
        // XREG without rms-norm: a wavefront needs nothing but the activations of its own four k blocks, so it
        // stages exactly those and waits for no other wavefront before it starts.  (Wavefronts on the same k
        // blocks write the same bytes; not done when they would each load many rows twice.)
        const bool own_x = XREG && !normed && (step_slots == 1 || M <= 4);
        if (own_norm) {
#pragma unroll
            for (int m = 0; m < kMaxM; ++m)
                if (m < M) store_piece(m, pc_own, own_ok, keep[m], g_own);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // read back by the wavefront that wrote it
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else if (own_x) {
            for (int i0 = 0; i0 < M * kItemPieces; i0 += kStageBatch * 64) {
                half8_t vb[kStageBatch];
#pragma unroll
                for (int u = 0; u < kStageBatch; ++u) {
                    const int idx = i0 + u * 64 + lane;
                    const int m = idx / kItemPieces, pc = si * kItemPieces + idx % kItemPieces;
                    vb[u] = zero8;
                    if (m < M && pc < pieces && (int64_t)pc * 8 < K) vb[u] = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + (int64_t)pc * 8);
                }
#pragma unroll
                for (int u = 0; u < kStageBatch; ++u) {
                    const int idx = i0 + u * 64 + lane;
                    const int m = idx / kItemPieces, pc = si * kItemPieces + idx % kItemPieces;
                    store_piece(m, pc, m < M && pc < pieces, vb[u], zero8);     // (a last work item may reach beyond the row's blocks)
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // read back by the wavefront that wrote it
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            // all M * ph_pieces pieces (of this phase: all of them unless PHASED), kThreads at a time; the row of
            // piece idx is idx / ph_pieces, taken as the high half of idx * ceil(2^32 / ph_pieces) (exact while
            // M * ph_pieces^2 < 2^32, which the LDS limit implies)
            const int ph_pieces = PHASED ? nkb_ph * (XBB / 16) : pieces;
            const int pc_lo = PHASED ? kb_lo * (XBB / 16) : 0;
            const uint32_t pieces_magic = PHASED && ph == n_ph - 1 ? pieces_magic_last : pieces_magic_arg;
            for (int base = 0; base < M * ph_pieces; base += kStageBatch * kThreads) {
                half8_t vb[kStageBatch], gb[kStageBatch];
#pragma unroll
                for (int u = 0; u < kStageBatch; ++u) {
                    const int idx = base + u * kThreads + t;
                    const int m = (int)__umulhi((uint32_t)idx, pieces_magic), pc = idx - m * ph_pieces;
                    const int64_t k = (int64_t)(pc_lo + pc) * 8;
                    vb[u] = zero8;
                    gb[u] = zero8;
                    if (idx < M * ph_pieces && k < K) {
                        vb[u] = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + k);
                        if (normed) gb[u] = *reinterpret_cast<const half8_t*>(fu.gamma + k);
                    }
                }
#pragma unroll
                for (int u = 0; u < kStageBatch; ++u) {
                    const int idx = base + u * kThreads + t;
                    const int m = (int)__umulhi((uint32_t)idx, pieces_magic), pc = idx - m * ph_pieces;
                    store_piece(m, pc, idx < M * ph_pieces, vb[u], gb[u]);     // (pc: inside the staged part of the row)
                }
            }
            __syncthreads();
        }

        // X operand address of this lane: row min(l%16, M-1) (rows beyond M repeat the last one; their
        // results are never stored), k-group l/16
        const int x_row = GS == 1 ? min(n_l, M - 1) : (n_l / SLOT) * SLOT + min(n_l % SLOT, M - 1);
        const unsigned char* x_lane = xs + (size_t)x_row * row_stride + g_l * 2 * UB;

        half8_t xreg_h[XREG ? kSuper : 1][2], xreg_l[XREG ? kSuper : 1][2];
        if (XREG) {
#pragma unroll
            for (int j = 0; j < kSuper; ++j) {
                const unsigned char* xb = x_lane + (size_t)min(si * kSuper + j, nkb_ph - 1) * XBB;
#pragma unroll
                for (int wp = 0; wp < 2; ++wp) {
                    xreg_h[j][wp] = *reinterpret_cast<const half8_t*>(xb + wp * UB);
                    xreg_l[j][wp] = E8 ? xreg_h[j][wp] : *reinterpret_cast<const half8_t*>(xb + wp * UB + 16);
                }
            }
        }

        // The two sums of a block's activations per row of X (all of them, and those that meet the code pairs
        // read at 1/128 scale) come from the matrix cores as well: products with an all-ones weight operand.
        const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
        const half8_t ones8 = {(half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f};
        auto block_sums = [&](const half8_t (&xh)[2], const half8_t (&xl)[2], floatx4& sx, floatx4& sx30) {
            floatx4 sh = zero4, sl = zero4;
#pragma unroll
            for (int wp = 0; wp < 2; ++wp) {
                sh = __builtin_amdgcn_mfma_f32_16x16x32_f16(xh[wp], ones8, sh, 0, 0, 0);
                if (!E8) sl = __builtin_amdgcn_mfma_f32_16x16x32_f16(xl[wp], ones8, sl, 0, 0, 0);
            }
            sx = sh + sl;
            sx30 = 30.f * sl;
        };
        floatx4 sxr[XREG ? kSuper : 1], sx30r[XREG ? kSuper : 1];
        if (XREG) {
#pragma unroll
            for (int j = 0; j < kSuper; ++j) block_sums(xreg_h[j], xreg_l[j], sxr[j], sx30r[j]);
        }

        for (int s_rb = 0; s_rb < n_rb; ++s_rb) {
            floatx4 ysum = zero4;                           // this wavefront's share of Y[4*g_l .. 4*g_l+3][row n_l] of row block s_rb
            while (slot == s_rb) {
                // parameter word of (block j, weight row n_l): lane 16 j + n_l of the item's 64 words
                uint32_t pwj[kSuper];
#pragma unroll
                for (int j = 0; j < kSuper; ++j) {       // (GS > 1: of the group that this lane's four output rows belong to)
                    const int word = j * PW + (g_l * GS / 4) * kBlockRows + n_l;
                    pwj[j] = (uint32_t)__builtin_amdgcn_ds_bpermute((word & 63) * 4, (int)pwraw[GS == 1 ? 0 : (j * PW) / 64]);
                }
                fetch_params(nslot, nitem);
#pragma unroll
                for (int j = 0; j < kSuper; ++j) {
                    const int kb = si * kSuper + j;         // (inside the phase) may lie beyond K in the last item: such a block is left out below
                    const float sc = (float)param_scale(pwj[j]);
                    const float bi = (float)param_bias(pwj[j]);
                    const uint32_t words[4] = {c[j].x, c[j].y, c[j].z, c[j].w};
                    half2_t p[4][4];
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        if (E8) {                           // (w1_0, w1_1) and, after the rotation, (w1_2, w1_3)
                            const uint32_t m8 = fmask | fmask_low;
                            p[w][0] = __builtin_bit_cast(half2_t, (words[w] & m8) | kExpBits2);
                            p[w][1] = __builtin_bit_cast(half2_t, (__builtin_amdgcn_alignbit(words[w], words[w], 8) & m8) | kExpBits2);
                        } else {
                            w1_pairs_mixed(words[w], fmask, fmask_low, p[w]);
                        }
                    }
                    fetch_code(j, nslot, nitem);            // the block's registers are free: request the next item's
                    floatx4 acc_h = zero4, acc_l = zero4;
                    const unsigned char* xb = x_lane + (size_t)min(kb, nkb_ph - 1) * XBB;
                    half8_t xh2[2], xl2[2];
#pragma unroll
                    for (int wp = 0; wp < 2; ++wp) {
                        xh2[wp] = XREG ? xreg_h[XREG ? j : 0][wp] : *reinterpret_cast<const half8_t*>(xb + wp * UB);
                        xl2[wp] = E8 ? xh2[wp] : XREG ? xreg_l[XREG ? j : 0][wp] : *reinterpret_cast<const half8_t*>(xb + wp * UB + 16);
                    }
#pragma unroll
                    for (int wp = 0; wp < 2; ++wp) {
                        if (E8) {
                            const half2_t* w0 = p[2 * wp];
                            const half2_t* w1 = p[2 * wp + 1];
                            const half8_t w8 = {w0[0][0], w0[0][1], w0[1][0], w0[1][1], w1[0][0], w1[0][1], w1[1][0], w1[1][1]};
                            acc_h = __builtin_amdgcn_mfma_f32_16x16x32_f16(xh2[wp], w8, acc_h, 0, 0, 0);
                            continue;
                        }
                        const half8_t xh = xh2[wp], xl = xl2[wp];
                        const half2_t* w0 = p[2 * wp];
                        const half2_t* w1 = p[2 * wp + 1];
                        const half8_t wh = {w0[0][0], w0[0][1], w0[3][0], w0[3][1], w1[0][0], w1[0][1], w1[3][0], w1[3][1]};
                        const half8_t wl = {w0[1][0], w0[1][1], w0[2][0], w0[2][1], w1[1][0], w1[1][1], w1[2][0], w1[2][1]};
                        acc_h = __builtin_amdgcn_mfma_f32_16x16x32_f16(xh, wh, acc_h, 0, 0, 0);
                        acc_l = __builtin_amdgcn_mfma_f32_16x16x32_f16(xl, wl, acc_l, 0, 0, 0);
                    }
                    if (kb < nkb_ph) {
                        floatx4 sx, sx30;
                        if (XREG) {
                            sx = sxr[XREG ? j : 0];
                            sx30 = sx30r[XREG ? j : 0];
                        } else {
                            block_sums(xh2, xl2, sx, sx30);
                        }
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            ysum[r] += sc * ((acc_h[r] + 16.f * acc_l[r] - sx30[r]) - bi * sx[r]);
                    }
                }
                slot = nslot;
                si = nitem;
                advance(nslot, nitem);
            }
            if (late) {                                 // (a cell belongs to one wavefront, which adds later phases to it)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float* cell = red + ((s_rb * W + wave) * Ms + 4 * g_l + r) * kBlockRows + n_l;
                    if ((GS == 1 ? 4 * g_l + r : (4 * g_l + r) % SLOT) < M) *cell = PHASED && ph > 0 ? *cell + ysum[r] : ysum[r];
                }
                continue;
            }
            if (gated) {
                // slot 2p is the gate block and slot 2p + 1 the up block of pair p: park the gate sums in
                // half 0 of `red`, the up sums in half 1, then combine
                float* mine = red + (((s_rb & 1) * W + wave) * kMaxM + 4 * g_l) * kBlockRows + n_l;
#pragma unroll
                for (int r = 0; r < 4; ++r) mine[r * kBlockRows] = ysum[r];
                if ((s_rb & 1) == 0) continue;
                __syncthreads();
                if (t < kMaxM * kBlockRows) {
                    const int m = t >> 4, n = t & 15;
                    float g = 0.f, u = 0.f;
#pragma unroll
                    for (int w = 0; w < W; ++w)
#pragma unroll
                        for (int gg = 0; gg < GS; ++gg) {   // (the GS rows of a row of X; rows beyond M are not used)
                            const int mr = min(m + SLOT * gg, kMaxM - 1);
                            g += red[((0 * W + w) * kMaxM + mr) * kBlockRows + n];
                            u += red[((1 * W + w) * kMaxM + mr) * kBlockRows + n];
                        }
                    const int64_t col = (rb0 + (s_rb >> 1)) * kBlockRows + n;
                    if (m < M && col < fu.n_out) {
                        float y = silu_f32(g) * u;
                        if (fu.residual) y += (float)fu.residual[(int64_t)m * fu.n_out + col];
                        Y[(int64_t)m * fu.n_out + col] = (half_t)y;
                    }
                }
                __syncthreads();                            // both halves of `red` are free again
                continue;
            }
            // the wavefronts' shares of row block s_rb are added in wavefront order
            float* mine = red + (((s_rb & 1) * W + wave) * kMaxM + 4 * g_l) * kBlockRows + n_l;
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[r * kBlockRows] = ysum[r];
            __syncthreads();
            if (t < kMaxM * kBlockRows) {
                const int m = t >> 4, n = t & 15;
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < W; ++w)
#pragma unroll
                    for (int gg = 0; gg < GS; ++gg)
                        s += red[(((s_rb & 1) * W + w) * kMaxM + min(m + SLOT * gg, kMaxM - 1)) * kBlockRows + n];
                const int64_t row = (rb0 + s_rb) * kBlockRows + n;
                if (FUSED && fu.residual && m < M && row < N) s += (float)fu.residual[(int64_t)m * N + row];
                if (m < M && row < N) Y[(int64_t)m * N + row] = (half_t)s;
            }
            // no second barrier: row block s_rb + 1 uses the other half of `red`, and nobody writes this
            // half again before passing the barrier of s_rb + 1, which the readers above reach after reading
        }
    }
    if (late) {
        __syncthreads();
        const int units = gated ? n_rb / 2 : n_rb;      // one result per (row block or pair, row of X, weight row)
        for (int idx = t; idx < units * M * kBlockRows; idx += kThreads) {
            const int u = idx / (M * kBlockRows), m = (idx / kBlockRows) % M, n = idx % kBlockRows;
            const int sl = gated ? 2 * u : u;
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < W; ++w)
#pragma unroll
                for (int gg = 0; gg < GS; ++gg) v += red[((sl * W + w) * Ms + m + SLOT * gg) * kBlockRows + n];
            if (gated) {
                float up = 0.f;
#pragma unroll
                for (int w = 0; w < W; ++w)
#pragma unroll
                    for (int gg = 0; gg < GS; ++gg) up += red[(((sl + 1) * W + w) * Ms + m + SLOT * gg) * kBlockRows + n];
                v = silu_f32(v) * up;
            }
            const int64_t n_out = gated ? fu.n_out : N;
            const int64_t col = (rb0 + u) * kBlockRows + n;
            if (col < n_out) {
                if (FUSED && fu.residual) v += (float)fu.residual[(int64_t)m * n_out + col];
                Y[(int64_t)m * n_out + col] = (half_t)v;
            }
        }
    }
}

// M rows of X do not fit the LDS: K in phases.  The wavefront sums of all row blocks of a workgroup stay in LDS
// through the phases, the rest holds one phase's X; the phases are of equal length up to the last one's
// remainder.  One round of workgroups as long as that leaves room for kPhasedMinItems work items of X per
// phase, more workgroups with fewer row blocks each otherwise.
constexpr int kPhasedMinItems = 4;
bool make_phased_plan(int64_t M, int64_t nrb, int64_t nkb, MfmaPlan& p, int unit, bool e8, int w_knob, int target)
{
    const int64_t nsi = (nkb + kSuper - 1) / kSuper;
    const size_t xbb = e8 ? kXBlockBytes / 2 : kXBlockBytes;
    auto plan = [&](int w) -> bool {
        int64_t most = (nrb + std::min<int64_t>(nrb, target) - 1) / std::min<int64_t>(nrb, target);    // row blocks (or pairs) of a workgroup
        const size_t per_item = (size_t)M * kSuper * xbb, other = kNormBytes + (size_t)M * kRowPadBytes;
        const size_t min_x = other + (size_t)std::min<int64_t>(kPhasedMinItems, nsi) * per_item;
        const size_t room = (size_t)kLdsLimitBytes > min_x ? (size_t)kLdsLimitBytes - min_x : 0;    // for the sums
        most = std::min<int64_t>(most, std::max<int64_t>(1, (int64_t)(room / late_red_bytes(M, unit, w))));
        p.grid = (nrb + most - 1) / most;
        const size_t fixed = late_red_bytes(M, (int)most * unit, w) + other;
        if (fixed + per_item > (size_t)kLdsLimitBytes) return false;
        const int64_t fit = (int64_t)(((size_t)kLdsLimitBytes - fixed) / per_item);     // work items of X at a time
        const int64_t phases = (nsi + fit - 1) / fit;
        const int64_t nsi_ph = (nsi + phases - 1) / phases;
        p.waves = w;
        p.kb_phase = (int)(nsi_ph * kSuper);
        p.step_slots = (int)(w / nsi_ph);               // (the kernel derives them per phase)
        p.step_item = (int)(w % nsi_ph);
        p.rb_base = (int)(nrb / p.grid);
        p.rb_rem = (int)(nrb % p.grid);
        p.late = 1;
        p.lds_bytes = fixed + (size_t)nsi_ph * per_item;
        const uint64_t pieces = (uint64_t)p.kb_phase * (xbb / 16);
        const uint64_t pieces_last = (uint64_t)(nkb - (nkb - 1) / p.kb_phase * p.kb_phase) * (xbb / 16);
        p.pieces_magic = (uint32_t)(((1ull << 32) + pieces - 1) / pieces);      // (M * pieces^2 < 2^32: M * pieces * 16 bytes fit the LDS)
        p.pieces_magic_last = (uint32_t)(((1ull << 32) + pieces_last - 1) / pieces_last);
        return true;
    };
    if (w_knob >= 8) return plan(w_knob);
    if (!plan(8)) return false;
    // sixteen wavefronts for a single row block per workgroup (measured 7 - 14 % faster there: 4096 x 11008 and
    // 2048 x 16384 from M = 8 on; slower or equal with more row blocks) and for very long phases
    if (nrb <= target || p.kb_phase / kSuper > 16) {
        const MfmaPlan with8 = p;
        if (!plan(16)) p = with8;
    }
    return true;
}

// `unit`: 2 when row blocks are dealt in (gate, up) pairs; rb_base and rb_rem then count pairs
// (e8: K counts 4-bit slots, two per weight, and a block of X is half as long)
// Groups per block of a group size, and the rows of X the kernel stages for M rows (see the kernel's header).
int groups_per_block(int group) { return kG / group; }
int64_t staged_rows(int64_t M, int gs) { return gs == 1 ? M : (gs - 1) * (kMaxM / gs) + M; }

// (`gs`: groups per block; every LDS size below is for the staged rows)
bool make_mfma_plan(int64_t M_rows, int64_t N, int64_t K, MfmaPlan& p, int unit = 1, bool e8 = false, int gs = 1)
{
    const int64_t M = staged_rows(M_rows, gs);
    const int64_t nrb = row_blocks(N) / unit, nkb = k_blocks(K);
    const int64_t nsi = (nkb + kSuper - 1) / kSuper;
    int w = knob("gemv_waves");
    // (sixteen wavefronts for more than 16 work items per row block; with exactly 16 eight are faster: 8192 x 8192
    // at M = 4 takes 10.5 us, 12.1 with sixteen; 8-bit 4096 x 4096 at M = 2 5.9 against 6.7)
    const int w_knob = (w == 4 || w == 8 || w == 16) ? w : 0;
    if (!w_knob) w = nsi > 16 ? 16 : 8;
    const int w_wanted = w;
    while (w > 4 && lds_need(M, nkb, w, e8) > (size_t)kLdsLimitBytes) w /= 2;   // (smaller buffers for the wavefront sums)
    int target = knob("gemv_workgroups");
    if (target <= 0) target = kTargetWorkgroups;
    p.kb_phase = 0;
    p.pieces_magic_last = 0;
    // X does not fit beside the sums of eight wavefronts: K in phases rather than all of X with four wavefronts
    // (36864 x 7168 at M = 10: 33 us against 52)
    if (w < 8 && w_wanted >= 8 && knob("gemv_mfma") != 3 && make_phased_plan(M, nrb, nkb, p, unit, e8, w_knob, target))
        return true;
    if (lds_need(M, nkb, w, e8) > (size_t)kLdsLimitBytes) return false;
    p.grid = std::min<int64_t>(nrb, target);
    if (nrb > target) {                                 // the fewest workgroups with the same largest share of row
        const int64_t most = (nrb + target - 1) / target;   // blocks (or pairs), so that (nearly) all of them end together
        p.grid = (nrb + most - 1) / most;
    }
    p.waves = w;
    p.step_slots = (int)(w / nsi);
    p.step_item = (int)(w % nsi);
    p.rb_base = (int)(nrb / p.grid);
    p.rb_rem = (int)(nrb % p.grid);
    p.lds_bytes = lds_need(M, nkb, w, e8);
    const uint64_t row_pieces = (uint64_t)nkb * (e8 ? 8 : 16);
    if ((uint64_t)M * row_pieces * row_pieces >= (1ull << 32)) return false;    // (never within the LDS limit)
    p.pieces_magic = (uint32_t)(((1ull << 32) + row_pieces - 1) / row_pieces);
    const size_t per_rb = 2 * (size_t)w * kMaxM * kBlockRows * sizeof(float);
    const size_t late_bytes = late_red_bytes(M, (p.rb_base + 1) * unit, w);
    p.late = knob("gemv_mfma") != 3 && p.lds_bytes - per_rb + late_bytes <= (size_t)kLdsLimitBytes;
    if (p.late) p.lds_bytes = p.lds_bytes - per_rb + std::max(late_bytes, (size_t)16);
    return true;
}

template <int W, bool FUSED, bool XREG, bool E8 = false, bool PHASED = false, int GS = 1>
int launch_mfma_x(const MfmaPlan& p, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                  hipStream_t stream, const GemvFusion& fu)
{
    if (PHASED != (p.kb_phase > 0) || (PHASED && !p.late) || p.lds_bytes > (size_t)kLdsLimitBytes) return E0M4_ERR_SHAPE;
    static std::atomic<uint64_t> lds_allowed{0};
    const int arc = allow_dynamic_lds(reinterpret_cast<const void*>(&gemv_mfma_kernel<W, FUSED, XREG, E8, PHASED, GS>),
                                      kLdsLimitBytes, lds_allowed);
    if (arc != E0M4_OK) return arc;
    // (M: rows per chunk; fu.m_total: all rows, when there are several chunks)
    const unsigned chunks = fu.m_total > 0 ? (unsigned)((fu.m_total + M - 1) / M) : 1u;
    hipLaunchKernelGGL((gemv_mfma_kernel<W, FUSED, XREG, E8, PHASED, GS>), dim3((unsigned)p.grid, chunks), dim3(W * 64),
                       p.lds_bytes, stream, static_cast<const half_t*>(X), static_cast<const uint4*>(packed),
                       static_cast<half_t*>(Y), (int)M, (uint32_t)N, (uint32_t)K, p.step_slots, p.step_item, p.rb_base,
                       p.rb_rem, p.late, p.pieces_magic, p.kb_phase, p.pieces_magic_last, fu);
    return check_launch();
}

// K in phases (plans with kb_phase > 0; they have eight or sixteen wavefronts)
template <int W, bool FUSED, bool E8, int GS = 1>
int launch_mfma_phased(const MfmaPlan& p, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                       hipStream_t stream, const GemvFusion& fu)
{
    if constexpr (W >= 8)
        return launch_mfma_x<W, FUSED, false, E8, true, GS>(p, X, M, packed, N, K, Y, stream, fu);
    else
        return E0M4_ERR_SHAPE;
}

// Activations in registers when a wavefront always meets the same k blocks (step_item == 0); the kernel
// then needs about 125 registers per lane -- more than sixteen wavefronts have without spilling (that form measured
// twice as slow as reading X from LDS), so it is used with up to eight.
template <int W, bool FUSED, int GS>
int launch_mfma_groups(const MfmaPlan& p, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                       hipStream_t stream, const GemvFusion& fu)
{
    if (p.kb_phase > 0) return launch_mfma_phased<W, FUSED, false, GS>(p, X, M, packed, N, K, Y, stream, fu);
    return launch_mfma_x<W, FUSED, false, false, false, GS>(p, X, M, packed, N, K, Y, stream, fu);
}

template <int W, bool FUSED>
int launch_mfma(const MfmaPlan& p, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                hipStream_t stream, const GemvFusion& fu = GemvFusion{}, int gs = 1)
{
    if (gs == 2) return launch_mfma_groups<W, FUSED, 2>(p, X, M, packed, N, K, Y, stream, fu);
    if (gs == 4) return launch_mfma_groups<W, FUSED, 4>(p, X, M, packed, N, K, Y, stream, fu);
    if (p.kb_phase > 0) return launch_mfma_phased<W, FUSED, false>(p, X, M, packed, N, K, Y, stream, fu);
    if (p.step_item == 0 && W <= 8 && knob("gemv_mfma") != 2)
        return launch_mfma_x<W, FUSED, true>(p, X, M, packed, N, K, Y, stream, fu);
    return launch_mfma_x<W, FUSED, false>(p, X, M, packed, N, K, Y, stream, fu);
}

}  // namespace

bool gemv_mfma_supported(int64_t M, int64_t N, int64_t K, int group)
{
    if ((group != 128 && group != 64 && group != 32) || M < kMinM || M > kMaxM / groups_per_block(group) || N <= 0 || K <= 0)
        return false;
    MfmaPlan p;
    return make_mfma_plan(M, N, K, p, 1, false, groups_per_block(group));
}

// Rows per chunk when M rows go out in `chunks` equal chunks (the last may be shorter; never fewer than two rows for
// the M and chunk counts the callers use: 17 ... 64 rows in ceil(M / 16) chunks).
int64_t chunk_rows(int64_t M, int chunks) { return (M + chunks - 1) / chunks; }

// Groups of 64 and 32 stage every row of X two or four times (16 rows of LDS traffic whatever M is), which the
// kernel with dequantised operands (e0m4_gemv_dq.hip) does not: this one pays when a workgroup has several row
// blocks to spend its staging on, or (group 64) when the staged rows fit the LDS at once.  15360 x 5120 at M = 4:
// 12.4 us against 16.2; 27392 x 5120 at M = 8: 22.6 against 26.5; 5120 x 5120 at M = 4 7.5 against 8.8 but at
// M = 8, in phases, 11.1 against 9.5; 5120 x 13696 at M = 4, in phases, 18.9 against 16.8; at M = 2 the vector
// kernel is as fast or faster.
bool gemv_mfma_groups_pay(int64_t M, int64_t N, int64_t K, int group)
{
    const int gs = groups_per_block(group);
    MfmaPlan p;
    if (gs == 1 || M < 3 || !gemv_mfma_supported(M, N, K, group) || !make_mfma_plan(M, N, K, p, 1, false, gs)) return false;
    return p.rb_base >= 3 || (gs == 2 && p.kb_phase == 0);
}

int launch_gemv_mfma(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream,
                     int chunks, int group)
{
    MfmaPlan p;
    const int64_t mc = chunk_rows(M, chunks);
    const int gs = groups_per_block(group);
    if (chunks < 1 || M - (chunks - 1) * mc < kMinM || !gemv_mfma_supported(mc, N, K, group) ||
        !make_mfma_plan(mc, N, K, p, 1, false, gs))
        return E0M4_ERR_SHAPE;
    GemvFusion fu{};
    fu.m_total = chunks > 1 ? (int)M : 0;
    switch (p.waves) {
        case 4: return launch_mfma<4, false>(p, X, mc, packed, N, K, Y, stream, fu, gs);
        case 8: return launch_mfma<8, false>(p, X, mc, packed, N, K, Y, stream, fu, gs);
        default: return launch_mfma<16, false>(p, X, mc, packed, N, K, Y, stream, fu, gs);
    }
}

// 8-bit format: K in weights; group 64 or 128 (the packed buffer carries one parameter word per block either way).
bool gemv_mfma8_supported(int64_t M, int64_t N, int64_t K)
{
    if (M < kMinM || M > kMaxM || N <= 0 || K <= 0) return false;
    MfmaPlan p;
    return make_mfma_plan(M, N, 2 * K, p, 1, true);
}

namespace {
template <bool FUSED>
int launch_mfma8(const MfmaPlan& p, const GemvFusion& fu, const void* X, int64_t M, const void* packed, int64_t N,
                 int64_t K, void* Y, hipStream_t stream)
{
    if (p.kb_phase > 0)
        return p.waves == 8 ? launch_mfma_phased<8, FUSED, true>(p, X, M, packed, N, K, Y, stream, fu)
                            : launch_mfma_phased<16, FUSED, true>(p, X, M, packed, N, K, Y, stream, fu);
    const bool xreg = p.step_item == 0 && knob("gemv_mfma") != 2;
    switch (p.waves) {
        case 4:
            return xreg ? launch_mfma_x<4, FUSED, true, true>(p, X, M, packed, N, K, Y, stream, fu)
                        : launch_mfma_x<4, FUSED, false, true>(p, X, M, packed, N, K, Y, stream, fu);
        case 8:
            return xreg ? launch_mfma_x<8, FUSED, true, true>(p, X, M, packed, N, K, Y, stream, fu)
                        : launch_mfma_x<8, FUSED, false, true>(p, X, M, packed, N, K, Y, stream, fu);
        default:
            return xreg ? launch_mfma_x<16, FUSED, true, true>(p, X, M, packed, N, K, Y, stream, fu)
                        : launch_mfma_x<16, FUSED, false, true>(p, X, M, packed, N, K, Y, stream, fu);
    }
}
}  // namespace

int launch_gemv_mfma8(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream,
                      int chunks)
{
    MfmaPlan p;
    const int64_t mc = chunk_rows(M, chunks);
    if (chunks < 1 || M - (chunks - 1) * mc < kMinM || !make_mfma_plan(mc, N, 2 * K, p, 1, true)) return E0M4_ERR_SHAPE;
    GemvFusion fu{};
    fu.m_total = chunks > 1 ? (int)M : 0;
    return launch_mfma8<false>(p, fu, X, mc, packed, N, K, Y, stream);
}

bool gemv_mfma8_fused_supported(const Fusion& f, int64_t M, int64_t N, int64_t K)
{
    if (M < kMinM || M > kMaxM || N <= 0 || K <= 0) return false;
    if (f.swiglu && (N % (2 * kBlockRows) != 0 || gated_half_bytes(N, 2 * K, kG) > kMaxHalfBytes)) return false;
    MfmaPlan p;
    return make_mfma_plan(M, N, 2 * K, p, f.swiglu ? 2 : 1, true);
}

bool gemv_mfma8_whole_rows(const Fusion& f, int64_t M, int64_t N, int64_t K)
{
    MfmaPlan p;
    return gemv_mfma8_fused_supported(f, M, N, K) && make_mfma_plan(M, N, 2 * K, p, f.swiglu ? 2 : 1, true) && p.kb_phase == 0;
}

int launch_gemv_mfma8_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                            hipStream_t stream, int chunks)
{
    MfmaPlan p;
    const int64_t mc = chunk_rows(M, chunks);
    if (chunks < 1 || M - (chunks - 1) * mc < kMinM || !gemv_mfma8_fused_supported(f, mc, N, K) ||
        !make_mfma_plan(mc, N, 2 * K, p, f.swiglu ? 2 : 1, true))
        return E0M4_ERR_SHAPE;
    GemvFusion fu = make_gemv_fusion(f, N, 2 * K, kG);
    fu.m_total = chunks > 1 ? (int)M : 0;
    return launch_mfma8<true>(p, fu, X, mc, packed, N, K, Y, stream);
}

bool gemv_mfma_fused_supported(const Fusion& f, int64_t M, int64_t N, int64_t K, int group)
{
    if (!gemv_mfma_supported(M, N, K, group)) return false;
    if (!f.swiglu) return true;
    if (N % (2 * kBlockRows) != 0 || gated_half_bytes(N, K, group) > kMaxHalfBytes) return false;
    MfmaPlan p;
    return make_mfma_plan(M, N, K, p, 2, false, groups_per_block(group));
}

bool gemv_mfma_whole_rows(const Fusion& f, int64_t M, int64_t N, int64_t K, int group, int64_t* workgroups)
{
    MfmaPlan p;
    if (!gemv_mfma_fused_supported(f, M, N, K, group) ||
        !make_mfma_plan(M, N, K, p, f.swiglu ? 2 : 1, false, groups_per_block(group)) || p.kb_phase != 0)
        return false;
    if (workgroups) *workgroups = p.grid;
    return true;
}

int launch_gemv_mfma_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                           hipStream_t stream, int chunks, int group)
{
    MfmaPlan p;
    const int64_t mc = chunk_rows(M, chunks);
    const int gs = groups_per_block(group);
    if (chunks < 1 || M - (chunks - 1) * mc < kMinM || !gemv_mfma_fused_supported(f, mc, N, K, group) ||
        !make_mfma_plan(mc, N, K, p, f.swiglu ? 2 : 1, false, gs))
        return E0M4_ERR_SHAPE;
    GemvFusion fu = make_gemv_fusion(f, N, K, group);
    fu.m_total = chunks > 1 ? (int)M : 0;
    switch (p.waves) {
        case 4: return launch_mfma<4, true>(p, X, mc, packed, N, K, Y, stream, fu, gs);
        case 8: return launch_mfma<8, true>(p, X, mc, packed, N, K, Y, stream, fu, gs);
        default: return launch_mfma<16, true>(p, X, mc, packed, N, K, Y, stream, fu, gs);
    }
}

}  // namespace e0m4
