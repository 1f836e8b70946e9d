// Decode path of e0m4_matmul: Y[M,N] = X[M,K] * dequant(packed)^T for M <= 8.
// Paper: section "Operator and lagging optimizations" (vector-matrix product
// of the decoding stage, bound by memory bandwidth) with the dequantisation of
// section "E0M4 FP4 quantization" fused in registers.
//
// Work decomposition (gfx950, wave64): a workgroup owns a few consecutive blocks
// of 16 output rows over the whole of K, so no partial sums ever leave the
// compute unit and no second kernel, atomics or scratch memory are needed.  A
// work item is four consecutive 16 x 128 weight blocks of one row block (4 KiB
// of codes, contiguous, plus their group parameters); the W wavefronts take the
// work items of the workgroup's contiguous run round-robin and keep one item
// (four dwordx4 loads per lane) in flight while they process the previous one.
// Lane q*16 + r holds 32 codes of row r per block: it turns them into the raw
// binade values with one rotate and four mask-or per eight codes, accumulates
// a = sum x*w1 with v_dot2_f32_f16, and applies the group's affine map once per
// block:  y += scale * (a - bias * sum x).
// Activations are staged in LDS, with the sums of every 32-wide chunk: once per
// workgroup, or, when a wavefront only ever needs the activations of its own work
// items, by every wavefront for itself, without a workgroup barrier.  A wavefront
// that meets the same k blocks in every row block (M = 1, see XREG below) copies
// them to registers once, otherwise they are read from LDS block by block.  The four k-quarters of a row are added with two
// cross-lane steps, the wavefronts' sums through LDS in a fixed order
// (deterministic result).  The same kernel serves the INT4 comparison format and
// the 8-bit format E0M8 (template argument DEQ) and, as FUSED, folds in the
// operators of e0m4_matmul_fused.
#include "e0m4_device.h"
#include "e0m4_host.h"

#include <algorithm>
#include <type_traits>

namespace e0m4 {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSuper = 4;                       // weight blocks (of 128 k) per work item
constexpr int kXBudgetBytes = 112 * 1024;       // LDS spent on activations and their chunk sums, at most
constexpr int kRedBudgetBytes = 32 * 1024;      // LDS spent on the per-wavefront partial sums, at most
constexpr int kLdsLimitBytes = 144 * 1024;      // of the 160 KiB of a compute unit (one workgroup per unit)
constexpr int kLdsDefaultBytes = 64 * 1024;     // dynamic LDS a kernel may ask for without opting in to more
constexpr int kBytesPerBlockX = kBlockK * 2 + (kBlockK / kCodesPerChunk) * 8;   // 288 per row of X per k block
constexpr int kTargetWorkgroups = 256;          // one workgroup per compute unit (measured best: activations are staged once per workgroup)
constexpr int kEarlyX = 2;                      // activation pieces per thread requested before the weights

struct GemvPlan {
    int waves;          // wavefronts per workgroup
    int seg_items;      // work items (per row block) whose activations are resident in LDS at a time
    int rb_per_wg;      // the most consecutive row blocks one workgroup owns
    int step_slots;     // a wavefront's next work item: this many row blocks further ...
    int step_item;      // ... and this many items further (with carry), i.e. W items ahead
    int64_t grid;
    int rb_base, rb_rem;  // even deal of row blocks: workgroup b owns rb_base (+1 if b < rb_rem) consecutive row blocks
    int own_items;        // M = 1, one row block per workgroup, few items per wavefront: each stages its own activations
    size_t lds_bytes;
};

// `unit`: row blocks are dealt to workgroups in units of this many (2 for the gated epilogue, whose
// workgroups own pairs of a gate and an up row block; the plan then counts units where it says row blocks,
// except rb_per_wg, which counts row blocks).  `single_segment` tells whether all of X fits the LDS.
// `more_waves`: the caller also has the kernels with 10, 12 and 14 wavefronts (E0M4 codes, M = 1).
GemvPlan make_plan(int64_t M, int64_t N, int64_t K, int unit = 1, bool* single_segment_out = nullptr,
                   bool more_waves = false)
{
    GemvPlan p;
    const int64_t nrb = row_blocks(N) / unit, nkb = k_blocks(K);
    const int64_t nsi = (nkb + kSuper - 1) / kSuper;           // work items per row block
    int w = knob("gemv_waves");
    if (w == 16 && M > 4) w = 8;                // 16 wavefronts leave too few registers for that many accumulators
    const bool forced = w == 4 || w == 8 || w == 16;
    // 16 wavefronts when K is long, or when a workgroup has many work items of a medium K; 8 otherwise
    // (measured on the layer shapes of 2B to 14B models)
    const int64_t t_guess = (nrb + kTargetWorkgroups - 1) / kTargetWorkgroups;
    if (!forced) w = (M <= 4 && (nsi >= 16 || (nsi >= 8 && nsi * unit * t_guess >= 32))) ? 16 : 8;
    // M = 1 with 1, 2, 4 or 8 whole work items per row block: 8 wavefronts, each of which then stays on its
    // own k blocks and keeps their activations in registers (measured 2-4 % faster than 16 wavefronts)
    // (K = 5120, 6144, 7168: 10, 12 or 14 work items per row block get as many wavefronts, for the same reason;
    // 10 and 14 load the four SIMDs unevenly, which costs more than it gains when a workgroup has only one or
    // two row blocks: 5120 x 5120 takes 6.1 us against 5.7)
    if (!forced && M == 1 && nkb % kSuper == 0 && knob("gemv_xreg") != 2) {
        if (8 % nsi == 0) w = 8;
        else if (more_waves && (nsi == 12 || ((nsi == 10 || nsi == 14) && unit * t_guess >= 3))) w = (int)nsi;
    }
    int64_t t = 1;
    bool single_segment = true;
    for (;;) {
        const int64_t cap = kXBudgetBytes / (M * kSuper * kBytesPerBlockX);    // work items whose X fits (>= 5)
        single_segment = nsi <= cap;
        p.seg_items = (int)(single_segment ? nsi : (cap >= w ? cap / w * w : cap));   // a multiple of W if possible
        const int64_t x_bytes = M * p.seg_items * kSuper * kBytesPerBlockX;
        const int64_t red_budget = std::min<int64_t>(kRedBudgetBytes, kLdsLimitBytes - x_bytes);
        int64_t t_max = red_budget / ((int64_t)unit * w * M * kBlockRows * sizeof(float));
        if (t_max < 1) t_max = 1;
        int target = knob("gemv_workgroups");
        if (target <= 0) target = kTargetWorkgroups;
        t = (nrb + target - 1) / target;
        if (t > t_max) t = t_max;
        if (t < 1 || !single_segment) t = 1;   // several activation segments: one row block per workgroup
        // Row blocks (pairs of them with the gated epilogue) are dealt out evenly over the fewest workgroups that
        // keep the largest share t: then nearly all of them end together.  With more workgroups a few would own
        // one more than the rest, and a compute unit on its own cannot draw the bandwidth to catch up: 320 row
        // blocks of K = 13696 take 10.6 us on 160 workgroups of two, 11.8 us on 256 of one or two; 856 pairs 13.0 us
        // on 214 workgroups of four, 13.9 us on 256 of three or four.
        p.grid = (nrb + t - 1) / t;
        // fewer wavefronts when a workgroup has fewer work items than wavefronts
        if (!forced && w > 4 && nsi * unit * t < w) { w /= 2; continue; }
        break;
    }
    if (single_segment_out) *single_segment_out = single_segment;
    p.waves = w;
    p.rb_per_wg = (int)(unit * t);
    p.step_slots = (int)(w / nsi);
    p.step_item = (int)(w % nsi);
    p.rb_base = (int)(nrb / p.grid);
    p.rb_rem = (int)(nrb % p.grid);
    p.lds_bytes = (size_t)M * p.seg_items * kSuper * kBytesPerBlockX + (size_t)unit * t * w * M * kBlockRows * sizeof(float);
    p.own_items = M == 1 && unit == 1 && single_segment && p.grid == nrb && nsi >= w && nsi <= (int64_t)kEarlyX * w;
    return p;
}

// A workgroup owns up to `rb_per_wg` consecutive row blocks; its work items are (row block, group of
// four k blocks) in memory order.  Wavefront w takes items w, w+W, w+2W, ...
// DEQ selects how a 4-bit code becomes a number: kDeqE0M4 is the product path (bit operations only);
// kDeqInt4Convert is the INT4 twin of the paper's section "Evaluation of FP4 quantization" (Table 1):
// same data layout and work decomposition, but every code is extracted as an integer and turned into
// fp16 with a conversion instruction, and the parameter word holds (scale, integer zero point).
// kDeqE0M8 is the 8-bit member of the format family (e0m8_pack.hip): a block holds 64 weights, a lane's
// chunk 16, a 32-bit word four codes that one mask-or (and one more after a rotation) turns into two pairs
// of binade values, so the dot product needs no folding of pair kinds.
// kDeqBf16 is E0M4 on bfloat16: the same packed codes; activations, parameters and the output are bfloat16, a
// code becomes the bfloat16 value 2 + c/8 with one shift and one mask-or (code bits 6..3 of each half), and the
// dot products are v_dot2_f32_bf16.
enum { kDeqE0M4 = 0, kDeqInt4Convert = 1, kDeqE0M8 = 2, kDeqBf16 = 3 };

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
constexpr uint32_t kBf16CodeMask2 = 0x00780078u;       // fraction bits 6..3 of both bfloat16 halves
constexpr uint32_t kBf16Ones2 = 0x3F803F80u;           // (1.0, 1.0)
__device__ inline bf16x2_t as_bf16x2(uint32_t v) { return __builtin_bit_cast(bf16x2_t, v); }
__device__ inline float bf16_lo(uint32_t word) { return __builtin_bit_cast(float, word << 16); }
__device__ inline float bf16_hi(uint32_t word) { return __builtin_bit_cast(float, word & 0xFFFF0000u); }
// fp32 -> bfloat16 bits, round to nearest even (finite values)
__device__ inline uint16_t bf16_bits(float f)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
template <int DEQ>
__device__ inline half_t out_value(float s)
{
    if (DEQ == kDeqBf16) return __builtin_bit_cast(half_t, bf16_bits(s));
    return (half_t)s;
}

// FUSED adds the operators of GemvFusion (e0m4_device.h) to the kernel.
// XREG (M = 1, one segment, wavefront count a multiple of the work items per row block): a wavefront meets
// the same four k blocks in every row block and keeps their activations and chunk sums in registers.
// (They are copied from the staged LDS copy: letting every lane request its 4 x 64 bytes of X from memory
// instead, without staging and its barrier, measured 3-6 % slower: sixteen more load instructions per
// lane queue up ahead of the weights.)
template <int G, int M, int W, int DEQ = kDeqE0M4, bool FUSED = false, bool XREG = false>
__global__ __launch_bounds__(W * 64) void gemv_kernel(const half_t* __restrict__ X, const uint4* __restrict__ packed,
                                                      half_t* __restrict__ Y, uint32_t N32, uint32_t K32, int seg_items,
                                                      int step_slots, int step_item, int rb_base, int rb_rem, int own_items,
                                                      GemvFusion fu)
{
    // (The arguments up to own_items fill the 14 scalar registers that the launch itself can preload, see the
    // build flags: the plain kernel starts without waiting for a load of its arguments.  N <= 2^31, K <= 2^20.)
    const int64_t N = N32, K = K32;
    constexpr int kThreads = W * 64;
    constexpr int PW = block_param_words(G);            // parameter words per k block: 16, 32 or 64
    constexpr int NPL = kSuper * PW / 64;               // dword loads per lane that fetch a work item's parameters
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BLK_K = DEQ == kDeqE0M8 ? 64 : kBlockK;       // weights per block
    constexpr int CHUNK = DEQ == kDeqE0M8 ? 16 : kCodesPerChunk; // weights per lane and block
    const int seg_k = seg_items * kSuper * BLK_K;
    half_t* xs = reinterpret_cast<half_t*>(smem);                               // [M][seg_k]
    // per 32-wide chunk of X: (sum of the chunk, 30 x sum of its elements with k % 8 in 2..5)
    float2* sxs = reinterpret_cast<float2*>(smem + (size_t)M * seg_k * 2);      // [M][seg_k/32]
    float* part = reinterpret_cast<float*>(sxs + (size_t)M * (seg_k / CHUNK));  // [W][M] sums of squares (FUSED only)
    float* red = part + (FUSED ? W * M : 0);                                    // [rb_per_wg][W][M][16]

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int q = lane >> 4, r = lane & 15;
    const uint32_t fmask = frac_mask_vgpr(), fmask_low = frac_mask_low_vgpr();
    const PackedLayout<G> lay(DEQ == kDeqE0M8 ? 2 * K : K);     // 8-bit codes: two 4-bit slots each
    const int nkb = (int)lay.nkb;
    const int nsi = (nkb + kSuper - 1) / kSuper;
    // even deal of row blocks (of pairs of row blocks with the gated epilogue: rb0 is then the first pair,
    // which is also the number of its gate row block)
    const bool gated = FUSED && fu.swiglu;
    const int64_t rb0 = (int64_t)blockIdx.x * rb_base + min((int)blockIdx.x, rb_rem);
    const int n_rb = (rb_base + ((int)blockIdx.x < rb_rem ? 1 : 0)) * (gated ? 2 : 1);
    // Weights are read with buffer loads: a wavefront-uniform resource (base of this workgroup's run
    // of row blocks, far smaller than 2 GiB), a scalar offset per block and a constant lane offset.
    // Every address is clamped into the run by hand; nothing relies on the resource's range check.
    const __amdgpu_buffer_rsrc_t wg_codes = make_rsrc(packed + lay.code_index(rb0, 0));
    const __amdgpu_buffer_rsrc_t wg_params = make_rsrc(reinterpret_cast<const char*>(packed) + 4 * lay.param_index(rb0, 0));
    const uint32_t rb_stride = (uint32_t)nkb * block_bytes(G);                  // bytes from one row block to the next
    const uint32_t lane_code_off = lane * 16;
    // byte offset of row block slot s from the workgroup's first row block
    auto slot_off = [&](uint32_t s_) -> uint32_t {
        if (FUSED && fu.swiglu) return (s_ >> 1) * rb_stride + (s_ & 1) * fu.half_bytes;
        return s_ * rb_stride;
    };
    // Parameters of a work item: its 4*PW words are contiguous; load n gives lane l word 64n + l, and
    // block j of lane (q, r) needs word j*PW + slot(q, r), i.e. load (j*PW)/64, lane (j*PW)%64 + slot.
    const int pslot = lay.param_slot(q, r);
    const int param_words_rb = nkb * PW;                // parameter words of one row block

    auto advance = [&](int& s_, int& i_) {              // W work items ahead
        s_ += step_slots;
        i_ += step_item;
        if (i_ >= nsi) {
            i_ -= nsi;
            ++s_;
        }
    };
    int slot = 0, si = wave;                            // current work item: row block slot, item inside the row block
    while (si >= nsi) {
        si -= nsi;
        ++slot;
    }
    int nslot = slot, nitem = si;                       // the one after
    advance(nslot, nitem);

    // ---- activations
    const int pieces = seg_k / 8;                       // 16-byte pieces per row of X per segment
    auto x_piece = [&](int idx, int kb_first) {
        const int m = M == 1 ? 0 : idx / pieces, pc = M == 1 ? idx : idx % pieces;
        const int64_t k = (int64_t)kb_first * BLK_K + pc * 8;
        half8_t v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (idx < M * pieces && k < K) v = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + k);
        return v;
    };
    // the two sums of one piece (a piece is the k range of one code word: elements 2..5 meet the code
    // pairs that are read at 1/128 scale)
    auto piece_sums = [&](const half8_t& v, float& s, float& sl) {
        if (DEQ == kDeqBf16) {                          // one plain sum of the eight bfloat16 values
            const uint4 u = __builtin_bit_cast(uint4, v);
            s = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(u.x), as_bf16x2(kBf16Ones2), s, false);
            s = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(u.y), as_bf16x2(kBf16Ones2), s, false);
            s = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(u.z), as_bf16x2(kBf16Ones2), s, false);
            s = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(u.w), as_bf16x2(kBf16Ones2), s, false);
            return;
        }
        const half2_t ones = {(half_t)1.f, (half_t)1.f};
        const half2_t x0 = {v[0], v[1]}, x1 = {v[2], v[3]}, x2 = {v[4], v[5]}, x3 = {v[6], v[7]};
        sl = __builtin_amdgcn_fdot2(x1, ones, sl, false);
        sl = __builtin_amdgcn_fdot2(x2, ones, sl, false);
        s = __builtin_amdgcn_fdot2(x0, ones, s, false);
        s = __builtin_amdgcn_fdot2(x3, ones, s, false);
    };
    // rms-norm (FUSED with gamma): 1 / sqrt(mean of squares + eps) of every row of X, set below
    float rs[M];
#pragma unroll
    for (int m = 0; m < M; ++m) rs[m] = 1.f;
    // store one piece and, from every fourth lane, the two sums of its 32-wide chunk
    // the rms-norm weights that go with piece idx (zero beyond K)
    auto g_piece = [&](int idx, int kb_first) {
        const int pc = M == 1 ? idx : idx % pieces;
        const int64_t k = (int64_t)kb_first * BLK_K + pc * 8;
        half8_t gv = {0, 0, 0, 0, 0, 0, 0, 0};
        if (FUSED && fu.gamma && idx < M * pieces && k < K) gv = *reinterpret_cast<const half8_t*>(fu.gamma + k);
        return gv;
    };
    auto x_store = [&](int idx, const half8_t& vin, const half8_t& gv) {
        const int m = M == 1 ? 0 : idx / pieces, pc = M == 1 ? idx : idx % pieces;
        half8_t v = vin;
        if (FUSED && fu.gamma) {                        // normalise on the way in: (x * rs[m]) * gamma[k], one rounding
            float r = rs[0];
#pragma unroll
            for (int mm = 1; mm < M; ++mm) r = mm == m ? rs[mm] : r;
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (half_t)(((float)vin[i] * r) * (float)gv[i]);
        }
        float s = 0.f, sl = 0.f;
        piece_sums(v, s, sl);
        s += sl;
        s += __shfl_xor(s, 1);
        sl += __shfl_xor(sl, 1);
        if (CHUNK == 32) {                              // a chunk is four pieces (two for the 8-bit format)
            s += __shfl_xor(s, 2);
            sl += __shfl_xor(sl, 2);
        }
        if (idx < M * pieces) {
            constexpr int PPC = CHUNK / 8;              // pieces per chunk
            *reinterpret_cast<half8_t*>(&xs[m * seg_k + pc * 8]) = v;
            if ((pc % PPC) == 0) sxs[m * (seg_k / CHUNK) + pc / PPC] = make_float2(s, 30.f * sl);
        }
    };
    // stage pieces start, start + kThreads, ... : loads in batches of four, issued together and then
    // consumed, so that their latencies overlap
    auto stage_from = [&](int start, int kb_first) {
        for (int base = start; base < M * pieces; base += 4 * kThreads) {
            half8_t vb[4], gb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                vb[u] = x_piece(base + u * kThreads, kb_first);
                gb[u] = g_piece(base + u * kThreads, kb_first);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) x_store(base + u * kThreads, vb[u], gb[u]);
        }
    };
    // Two pieces of X per thread are requested before the weights, so that they are not queued behind
    // them (loads return in order; requesting the weights first was measured slower).  What two pieces
    // per thread do not cover (large M * K) is staged right away.
    // Without rms-norm, when a wavefront needs nothing but the activations of its own work items -- XREG
    // (the same four k blocks in every row block), or `own_items` (M = 1, one row block per workgroup, at
    // most kEarlyX items per wavefront) -- it stages exactly those (one piece per lane and item; wavefronts on
    // the same k blocks write the same bytes) and waits for no other wavefront before it starts.
    const bool normed = FUSED && fu.gamma != nullptr;   // then staging waits for the row scales (below)
    // With rms-norm the same holds for XREG when every k block belongs to exactly one wavefront (step_slots == 1):
    // the wavefronts' sums of squares of their own pieces add up to the row's, and only that sum crosses wavefronts.
    const bool own_norm = normed && XREG && M == 1 && step_slots == 1;
    const bool own_x = (!normed && (XREG || own_items != 0)) || own_norm;
    constexpr int kItemPieces = kSuper * BLK_K / 8;     // pieces of one work item's activations: 64 (32 for 8-bit codes)
    auto own_idx = [&](int e) {                         // piece index of this lane for the wavefront's item number e
        const int it = si + e * W;
        return (lane < kItemPieces && it < nsi && (!XREG || e == 0)) ? it * kItemPieces + lane : M * pieces;
    };
    half8_t xearly[kEarlyX];
#pragma unroll
    for (int e = 0; e < kEarlyX; ++e) xearly[e] = x_piece(own_x ? own_idx(e) : t + e * kThreads, 0);
    const half8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    half8_t gearly[kEarlyX];                            // norm weights of the early pieces, requested with them
#pragma unroll
    for (int e = 0; e < kEarlyX; ++e) gearly[e] = normed ? g_piece(own_norm ? own_idx(e) : t + e * kThreads, 0) : zero8;
    // gated or not, result number t of the epilogue is this thread's first: request its residual value now
    float res_early = 0.f;
    if (FUSED && fu.residual) {
        const int units = gated ? n_rb / 2 : n_rb;
        const int u = t / (M * kBlockRows), m = (t / kBlockRows) % M, rr = t % kBlockRows;
        const int64_t n = (rb0 + u) * kBlockRows + rr;
        if (u < units && n < fu.n_out) res_early = (float)fu.residual[(int64_t)m * fu.n_out + n];
    }
    if (!normed && !own_x) stage_from(t + kEarlyX * kThreads, 0);

    // ---- the work item in flight: four code blocks and the parameter words
    uint4 c[kSuper];
    uint32_t pwraw[NPL];
    auto fetch_params = [&](int fs, int fi) {           // past the end the last item is read again
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, i_ = in ? fi : nsi - 1;
        const uint32_t soff = __builtin_amdgcn_readfirstlane(slot_off(s_) + i_ * (kSuper * PW * 4));
        const int last = param_words_rb - 1 - (int)i_ * (kSuper * PW);       // words left in this row block
#pragma unroll
        for (int n = 0; n < NPL; ++n)
            pwraw[n] = __builtin_amdgcn_raw_buffer_load_b32(wg_params, min(n * 64 + lane, last) * 4, (int)soff, 0);
    };
    auto fetch_code = [&](int j, int fs, int fi) {      // k blocks beyond K: the last block again (their X is zero)
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, i_ = in ? fi : nsi - 1;
        const uint32_t kb = min(i_ * kSuper + j, (uint32_t)nkb - 1);
        const uint32_t soff = __builtin_amdgcn_readfirstlane(slot_off(s_) + kb * kBlockCodeBytes);
        const u32x4 cv = __builtin_amdgcn_raw_buffer_load_b128(wg_codes, (int)lane_code_off, (int)soff, 0);
        c[j] = make_uint4(cv.x, cv.y, cv.z, cv.w);
    };
    fetch_params(slot, si);
#pragma unroll
    for (int j = 0; j < kSuper; ++j) fetch_code(j, slot, si);

    // every wavefront clears its own partial sums (it may not visit every row block)
    if (lane < kBlockRows)
        for (int sl = 0; sl < n_rb; ++sl)
#pragma unroll
            for (int m = 0; m < M; ++m) red[((sl * W + wave) * M + m) * kBlockRows + lane] = 0.f;

    if (normed) {
        // Sum of squares of every row of X over the whole of K: from the pieces already in registers when
        // one segment holds whole rows, else (and for what the registers do not cover) from memory.
        float ss[M];
#pragma unroll
        for (int m = 0; m < M; ++m) ss[m] = 0.f;
        auto add_squares = [&](int m, const half8_t& v) {
            const half2_t x0 = {v[0], v[1]}, x1 = {v[2], v[3]}, x2 = {v[4], v[5]}, x3 = {v[6], v[7]};
            float d = __builtin_amdgcn_fdot2(x0, x0, 0.f, false);
            d = __builtin_amdgcn_fdot2(x1, x1, d, false);
            d = __builtin_amdgcn_fdot2(x2, x2, d, false);
            d = __builtin_amdgcn_fdot2(x3, x3, d, false);
#pragma unroll
            for (int mm = 0; mm < M; ++mm) ss[mm] += mm == m ? d : 0.f;
        };
        if (own_norm) {                                 // this wavefront's share: its own piece per lane
            add_squares(0, xearly[0]);
        } else if (seg_items >= nsi) {                  // segment 0 is all of K (pieces beyond K are zero)
#pragma unroll
            for (int e = 0; e < kEarlyX; ++e) {
                const int idx = t + e * kThreads;
                add_squares(M == 1 ? 0 : idx / pieces, xearly[e]);
            }
            for (int idx = t + kEarlyX * kThreads; idx < M * pieces; idx += kThreads)
                add_squares(M == 1 ? 0 : idx / pieces, x_piece(idx, 0));
        } else {
            const int row_pieces = (int)(K / 8);
            for (int idx = t; idx < M * row_pieces; idx += kThreads) {
                const int m = M == 1 ? 0 : idx / row_pieces, pc = M == 1 ? idx : idx % row_pieces;
                add_squares(m, *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + (int64_t)pc * 8));
            }
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float v = ss[m];
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) v += __shfl_xor(v, d);
            if (lane == 0) part[wave * M + m] = v;
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < W; ++w) v += part[w * M + m];
            rs[m] = 1.f / sqrtf(v / (float)K + fu.eps);
        }
        if (!own_norm) stage_from(t + kEarlyX * kThreads, 0);
    }

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

    for (int seg0 = 0; seg0 < nsi; seg0 += seg_items) {
        // stage the segment's activations and the sums of every 32-wide chunk
        if (own_x) {                                    // (single segment) the wavefront's own pieces, read back by itself
#pragma unroll
            for (int e = 0; e < (XREG ? 1 : kEarlyX); ++e) x_store(own_idx(e), xearly[e], gearly[e]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            if (seg0 == 0) {
#pragma unroll
                for (int e = 0; e < kEarlyX; ++e) x_store(t + e * kThreads, xearly[e], gearly[e]);
            } else {
                __syncthreads();                        // everyone is done with the previous segment's activations
                stage_from(t, seg0 * kSuper);
            }
            __syncthreads();
        }
        half8_t xr[XREG ? kSuper : 1][4];
        float2 sxr[XREG ? kSuper : 1];
        if (XREG) {
#pragma unroll
            for (int j = 0; j < kSuper; ++j) {
                const int xoff = (si * kSuper + j) * BLK_K + q * CHUNK;
#pragma unroll
                for (int w = 0; w < CHUNK / 8; ++w) xr[j][w] = *reinterpret_cast<const half8_t*>(&xs[xoff + 8 * w]);
                sxr[j] = sxs[xoff / CHUNK];
            }
        }
        const int seg_end = seg0 + seg_items;
        while (slot < n_rb && si < seg_end) {
            // the item's parameter words, then request the next item's
            uint32_t pwj[kSuper];
#pragma unroll
            for (int j = 0; j < kSuper; ++j) {
                if (G == 32) pwj[j] = pwraw[j];
                else pwj[j] = (uint32_t)__builtin_amdgcn_ds_bpermute((((j * PW) % 64) + pslot) * 4, (int)pwraw[(j * PW) / 64]);
            }
            fetch_params(nslot, nitem);
#pragma unroll
            for (int j = 0; j < kSuper; ++j) {
                const float sc = DEQ == kDeqBf16 ? bf16_lo(pwj[j]) : (float)param_scale(pwj[j]);
                const float bi = DEQ == kDeqBf16 ? bf16_hi(pwj[j]) : (float)param_bias(pwj[j]);
                const uint32_t words[4] = {c[j].x, c[j].y, c[j].z, c[j].w};
                const int xoff = ((si - seg0) * kSuper + j) * BLK_K + q * CHUNK;
                float a[M][2];      // per row of X: sum x*(2 + c/8) over code pairs 0 and 3, sum x*(2 + c/128) over 1 and 2
#pragma unroll
                for (int m = 0; m < M; ++m) a[m][0] = a[m][1] = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    if (DEQ == kDeqE0M8) {              // four weights per word: two mask-or, two dot instructions
                        const half2_t p01 = __builtin_bit_cast(half2_t, (words[w] & kFrac8Mask2) | kExpBits2);
                        const half2_t p23 =
                            __builtin_bit_cast(half2_t, (__builtin_amdgcn_alignbit(words[w], words[w], 8) & kFrac8Mask2) | kExpBits2);
#pragma unroll
                        for (int m = 0; m < M; ++m) {
                            half4_t xv;
                            if (XREG) {
                                const half8_t x8 = xr[XREG ? j : 0][w >> 1];
                                xv = (w & 1) ? half4_t{x8[4], x8[5], x8[6], x8[7]} : half4_t{x8[0], x8[1], x8[2], x8[3]};
                            } else {
                                xv = *reinterpret_cast<const half4_t*>(&xs[m * seg_k + xoff + 4 * w]);
                            }
                            const half2_t x01 = {xv[0], xv[1]}, x23 = {xv[2], xv[3]};
                            a[m][0] = __builtin_amdgcn_fdot2(p01, x01, a[m][0], false);
                            a[m][0] = __builtin_amdgcn_fdot2(p23, x23, a[m][0], false);
                        }
                        continue;
                    }
                    if (DEQ == kDeqBf16) {              // four shifts, four mask-or, four dot instructions per word
                        const uint32_t wd = words[w];
                        const uint32_t b0 = ((wd >> 3) & kBf16CodeMask2) | kExpBits2;
                        const uint32_t b1 = ((wd << 1) & kBf16CodeMask2) | kExpBits2;
                        const uint32_t b2 = ((wd >> 7) & kBf16CodeMask2) | kExpBits2;
                        const uint32_t b3 = (__builtin_amdgcn_alignbit(wd, wd, 11) & kBf16CodeMask2) | kExpBits2;
#pragma unroll
                        for (int m = 0; m < M; ++m) {
                            const half8_t xv = XREG ? xr[XREG ? j : 0][w] : *reinterpret_cast<const half8_t*>(&xs[m * seg_k + xoff + 8 * w]);
                            const uint4 xu = __builtin_bit_cast(uint4, xv);
                            a[m][0] = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(b0), as_bf16x2(xu.x), a[m][0], false);
                            a[m][0] = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(b1), as_bf16x2(xu.y), a[m][0], false);
                            a[m][0] = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(b2), as_bf16x2(xu.z), a[m][0], false);
                            a[m][0] = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(b3), as_bf16x2(xu.w), a[m][0], false);
                        }
                        continue;
                    }
                    half2_t p[4];
                    if (DEQ == kDeqInt4Convert) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)     // integer code -> fp16 by conversion
                            p[i] = half2_t{(half_t)(uint16_t)extract_code(words[w], 2 * i),
                                           (half_t)(uint16_t)extract_code(words[w], 2 * i + 1)};
                    } else {
                        w1_pairs_mixed(words[w], fmask, fmask_low, p);
                    }
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        const half8_t xv = XREG ? xr[XREG ? j : 0][w] : *reinterpret_cast<const half8_t*>(&xs[m * seg_k + xoff + 8 * w]);
                        const half2_t x0 = {xv[0], xv[1]}, x1 = {xv[2], xv[3]}, x2 = {xv[4], xv[5]}, x3 = {xv[6], xv[7]};
                        a[m][0] = __builtin_amdgcn_fdot2(p[0], x0, a[m][0], false);
                        a[m][1] = __builtin_amdgcn_fdot2(p[1], x1, a[m][1], false);
                        a[m][1] = __builtin_amdgcn_fdot2(p[2], x2, a[m][1], false);
                        a[m][0] = __builtin_amdgcn_fdot2(p[3], x3, a[m][0], false);
                    }
                }
                fetch_code(j, nslot, nitem);            // the block's registers are free: request the next item's
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    const float2 sx = XREG ? sxr[XREG ? j : 0] : sxs[m * (seg_k / CHUNK) + xoff / CHUNK];
                    if (DEQ == kDeqE0M8 || DEQ == kDeqBf16)     // y += scale * (sum x*w1 - bias * sum x)
                        acc[m] += sc * (a[m][0] - bi * sx.x);
                    else if (DEQ == kDeqInt4Convert)    // y += scale * (sum x*q - zero * sum x)
                        acc[m] += sc * ((a[m][0] + a[m][1]) - bi * sx.x);
                    else    // sum x*w1 = a0 + 16*a1 - 30*(sum of x over pairs 1 and 2); then the group's affine map
                        acc[m] += sc * ((a[m][0] + 16.f * a[m][1] - sx.y) - bi * sx.x);
                }
            }
            const int prev = slot;
            slot = nslot;
            si = nitem;
            advance(nslot, nitem);
            if (slot != prev) flush(prev);              // the next item belongs to a later row block
        }
    }
    if (slot < n_rb) flush(slot);                       // sums of a row block this wavefront left unfinished (several segments)
    __syncthreads();
    if (FUSED) {
        // one result per (row block or pair of row blocks, row of X, row of the block)
        const int units = gated ? n_rb / 2 : n_rb;
        for (int idx = t; idx < units * M * kBlockRows; idx += kThreads) {
            const int u = idx / (M * kBlockRows), m = (idx / kBlockRows) % M, rr = idx % kBlockRows;
            const int sl = gated ? 2 * u : u;
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < W; ++w) s += red[((sl * W + w) * M + m) * kBlockRows + rr];
            if (gated) {
                float up = 0.f;
#pragma unroll
                for (int w = 0; w < W; ++w) up += red[(((sl + 1) * W + w) * M + m) * kBlockRows + rr];
                s = silu_f32(s) * up;
            }
            const int64_t n = (rb0 + u) * kBlockRows + rr;
            if (n < fu.n_out) {
                if (fu.residual) s += idx == t ? res_early : (float)fu.residual[(int64_t)m * fu.n_out + n];
                Y[(int64_t)m * fu.n_out + n] = (half_t)s;
            }
        }
        return;
    }
    for (int idx = t; idx < n_rb * M * kBlockRows; idx += kThreads) {
        const int sl = idx / (M * kBlockRows), m = (idx / kBlockRows) % M, rr = idx % kBlockRows;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) s += red[((sl * W + w) * M + m) * kBlockRows + rr];
        const int64_t n = (rb0 + sl) * kBlockRows + rr;
        if (n < N) Y[(int64_t)m * N + n] = out_value<DEQ>(s);
    }
}

template <int G, int M, int W, int DEQ = kDeqE0M4, bool FUSED = false, bool XREG = false>
int launch_one(const GemvPlan& p, const void* X, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream,
               const GemvFusion& fu = GemvFusion{})
{
    if constexpr (M == 1 && !XREG) {
        // every wavefront stays on its own k blocks, all of X in one segment, and a work item that exists
        const int64_t nkb = k_blocks(DEQ == kDeqE0M8 ? 2 * K : K);     // (8-bit codes: blocks of 64 weights)
        const int64_t nsi = (nkb + kSuper - 1) / kSuper;
        if (knob("gemv_xreg") != 2 && p.step_item == 0 && p.seg_items >= nsi && W >= nsi &&       // (2: never)
            nkb % kSuper == 0)
            return launch_one<G, M, W, DEQ, FUSED, true>(p, X, packed, N, K, Y, stream, fu);
    }
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    const dim3 grid((unsigned)p.grid), block(W * 64);
    const size_t lds_bytes = p.lds_bytes + (FUSED ? (size_t)W * M * sizeof(float) : 0);
    if (lds_bytes > (size_t)kLdsDefaultBytes) {
        static std::atomic<uint64_t> lds_allowed{0};    // per instantiation
        const int arc = allow_dynamic_lds(reinterpret_cast<const void*>(&gemv_kernel<G, M, W, DEQ, FUSED, XREG>),
                                          kLdsLimitBytes, lds_allowed);
        if (arc != E0M4_OK) return arc;
    }
    hipLaunchKernelGGL((gemv_kernel<G, M, W, DEQ, FUSED, XREG>), grid, block, lds_bytes, stream, x, c, y, (uint32_t)N,
                       (uint32_t)K, p.seg_items, p.step_slots, p.step_item, p.rb_base, p.rb_rem, p.own_items, fu);
    return check_launch();
}

// INT4 twin, M = 1: the same plan and launch shape as the product kernel.
template <int G>
int launch_int4_w(const GemvPlan& p, const void* X, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream)
{
    switch (p.waves) {
        case 4: return launch_one<G, 1, 4, kDeqInt4Convert>(p, X, packed, N, K, Y, stream);
        case 8: return launch_one<G, 1, 8, kDeqInt4Convert>(p, X, packed, N, K, Y, stream);
        default: return launch_one<G, 1, 16, kDeqInt4Convert>(p, X, packed, N, K, Y, stream);
    }
}

template <int G, int M, bool FUSED>
int launch_w(const GemvPlan& p, const void* X, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream,
             const GemvFusion& fu)
{
    if constexpr (M == 1) {                             // one wavefront per work item of a row block, activations in registers
        const bool own = p.step_item == 0 && p.step_slots == 1 && p.seg_items == p.waves;
        if (p.waves == 10 && own) return launch_one<G, 1, 10, kDeqE0M4, FUSED, true>(p, X, packed, N, K, Y, stream, fu);
        if (p.waves == 12 && own) return launch_one<G, 1, 12, kDeqE0M4, FUSED, true>(p, X, packed, N, K, Y, stream, fu);
        if (p.waves == 14 && own) return launch_one<G, 1, 14, kDeqE0M4, FUSED, true>(p, X, packed, N, K, Y, stream, fu);
    }
    if (p.waves != 4 && p.waves != 8 && p.waves != 16) return E0M4_ERR_SHAPE;      // make_plan never asks for this
    switch (p.waves) {
        case 4: return launch_one<G, M, 4, kDeqE0M4, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 8: return launch_one<G, M, 8, kDeqE0M4, FUSED>(p, X, packed, N, K, Y, stream, fu);
        default:
            if constexpr (M <= 4) return launch_one<G, M, 16, kDeqE0M4, FUSED>(p, X, packed, N, K, Y, stream, fu);
            else return E0M4_ERR_SHAPE;                 // make_plan never asks for this
    }
}

template <int G, bool FUSED>
int launch_m(const GemvPlan& p, int64_t M, const void* X, const void* packed, int64_t N, int64_t K, void* Y,
             hipStream_t stream, const GemvFusion& fu = GemvFusion{})
{
    switch (M) {
        case 1: return launch_w<G, 1, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 2: return launch_w<G, 2, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 3: return launch_w<G, 3, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 4: return launch_w<G, 4, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 5: return launch_w<G, 5, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 6: return launch_w<G, 6, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 7: return launch_w<G, 7, FUSED>(p, X, packed, N, K, Y, stream, fu);
        case 8: return launch_w<G, 8, FUSED>(p, X, packed, N, K, Y, stream, fu);
        default: return E0M4_ERR_SHAPE;
    }
}

}  // namespace

int launch_gemv(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                hipStream_t stream)
{
    const GemvPlan p = make_plan(M, N, K, 1, nullptr, true);
    switch (group) {
        case 32: return launch_m<32, false>(p, M, X, packed, N, K, Y, stream);
        case 64: return launch_m<64, false>(p, M, X, packed, N, K, Y, stream);
        case 128: return launch_m<128, false>(p, M, X, packed, N, K, Y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

GemvFusion make_gemv_fusion(const Fusion& f, int64_t N, int64_t K, int group)
{
    GemvFusion fu{};
    fu.gamma = static_cast<const half_t*>(f.gamma);
    fu.residual = static_cast<const half_t*>(f.residual);
    fu.eps = f.eps;
    fu.swiglu = f.swiglu ? 1 : 0;
    fu.half_bytes = (uint32_t)gated_half_bytes(N, K, group);
    fu.n_out = f.swiglu ? N / 2 : N;
    return fu;
}

// The gated epilogue needs a workgroup to own a gate row block together with its up row block, which
// the kernel cannot do when X has to be staged in several segments (it then owns one row block at a
// time); N/2 must be whole row blocks and the two halves less than 2 GiB apart.
bool gemv_fused_supported(const Fusion& f, int64_t M, int64_t N, int64_t K)
{
    if (M < 1 || M > kGemvMaxM) return false;
    if (!f.swiglu) return true;
    if (N % (2 * kBlockRows) != 0) return false;
    bool single = true;
    make_plan(M, N, K, 2, &single);
    return single;
}

int launch_gemv_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group,
                      void* Y, hipStream_t stream)
{
    if (!gemv_fused_supported(f, M, N, K)) return E0M4_ERR_SHAPE;
    const GemvPlan p = make_plan(M, N, K, f.swiglu ? 2 : 1, nullptr, true);
    const int64_t half_bytes = gated_half_bytes(N, K, group);
    if (f.swiglu && half_bytes > kMaxHalfBytes) return E0M4_ERR_SHAPE;
    const GemvFusion fu = make_gemv_fusion(f, N, K, group);
    switch (group) {
        case 32: return launch_m<32, true>(p, M, X, packed, N, K, Y, stream, fu);
        case 64: return launch_m<64, true>(p, M, X, packed, N, K, Y, stream, fu);
        case 128: return launch_m<128, true>(p, M, X, packed, N, K, Y, stream, fu);
        default: return E0M4_ERR_GROUP;
    }
}

// 8-bit format, M <= 8: the packed buffer is a 4-bit layout of 2K codes with groups of 128.  `f`: fused
// operators, or null.
namespace {
template <bool FUSED>
int launch_gemv8_m(const GemvPlan& p, const GemvFusion& fu, const void* X, int64_t M, const void* packed, int64_t N,
                   int64_t K, void* Y, hipStream_t stream)
{
    auto go = [&](auto m_tag) -> int {
        constexpr int MM = decltype(m_tag)::value;
        switch (p.waves) {
            case 4: return launch_one<128, MM, 4, kDeqE0M8, FUSED>(p, X, packed, N, K, Y, stream, fu);
            case 8: return launch_one<128, MM, 8, kDeqE0M8, FUSED>(p, X, packed, N, K, Y, stream, fu);
            default:
                if constexpr (MM <= 4) return launch_one<128, MM, 16, kDeqE0M8, FUSED>(p, X, packed, N, K, Y, stream, fu);
                else return E0M4_ERR_SHAPE;
        }
    };
    switch (M) {
        case 1: return go(std::integral_constant<int, 1>{});
        case 2: return go(std::integral_constant<int, 2>{});
        case 3: return go(std::integral_constant<int, 3>{});
        case 4: return go(std::integral_constant<int, 4>{});
        case 5: return go(std::integral_constant<int, 5>{});
        case 6: return go(std::integral_constant<int, 6>{});
        case 7: return go(std::integral_constant<int, 7>{});
        case 8: return go(std::integral_constant<int, 8>{});
        default: return E0M4_ERR_SHAPE;
    }
}
}  // namespace

int launch_gemv8(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream)
{
    return launch_gemv8_m<false>(make_plan(M, N, 2 * K), GemvFusion{}, X, M, packed, N, K, Y, stream);
}

int launch_gemv8_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                       hipStream_t stream)
{
    if (!gemv_fused_supported(f, M, N, 2 * K)) return E0M4_ERR_SHAPE;
    if (f.swiglu && gated_half_bytes(N, 2 * K, 128) > kMaxHalfBytes) return E0M4_ERR_SHAPE;
    return launch_gemv8_m<true>(make_plan(M, N, 2 * K, f.swiglu ? 2 : 1), make_gemv_fusion(f, N, 2 * K, 128), X, M, packed,
                                N, K, Y, stream);
}

// E0M4 on bfloat16, M <= 8: X, the embedded parameters and Y are bfloat16.
namespace {
template <int G>
int launch_bf16_m(const GemvPlan& p, int64_t M, const void* X, const void* packed, int64_t N, int64_t K, void* Y,
                  hipStream_t stream)
{
    auto go = [&](auto m_tag) -> int {
        constexpr int MM = decltype(m_tag)::value;
        switch (p.waves) {
            case 4: return launch_one<G, MM, 4, kDeqBf16>(p, X, packed, N, K, Y, stream);
            case 8: return launch_one<G, MM, 8, kDeqBf16>(p, X, packed, N, K, Y, stream);
            default:
                if constexpr (MM <= 4) return launch_one<G, MM, 16, kDeqBf16>(p, X, packed, N, K, Y, stream);
                else return E0M4_ERR_SHAPE;
        }
    };
    switch (M) {
        case 1: return go(std::integral_constant<int, 1>{});
        case 2: return go(std::integral_constant<int, 2>{});
        case 3: return go(std::integral_constant<int, 3>{});
        case 4: return go(std::integral_constant<int, 4>{});
        case 5: return go(std::integral_constant<int, 5>{});
        case 6: return go(std::integral_constant<int, 6>{});
        case 7: return go(std::integral_constant<int, 7>{});
        case 8: return go(std::integral_constant<int, 8>{});
        default: return E0M4_ERR_SHAPE;
    }
}
}  // namespace

int launch_gemv_bf16(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     hipStream_t stream)
{
    const GemvPlan p = make_plan(M, N, K);
    switch (group) {
        case 32: return launch_bf16_m<32>(p, M, X, packed, N, K, Y, stream);
        case 64: return launch_bf16_m<64>(p, M, X, packed, N, K, Y, stream);
        case 128: return launch_bf16_m<128>(p, M, X, packed, N, K, Y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

int launch_gemv_int4(const void* X, const void* packed, int64_t N, int64_t K, int group, void* Y, hipStream_t stream)
{
    const GemvPlan p = make_plan(1, N, K);
    switch (group) {
        case 32: return launch_int4_w<32>(p, X, packed, N, K, Y, stream);
        case 64: return launch_int4_w<64>(p, X, packed, N, K, Y, stream);
        case 128: return launch_int4_w<128>(p, X, packed, N, K, Y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

}  // namespace e0m4
