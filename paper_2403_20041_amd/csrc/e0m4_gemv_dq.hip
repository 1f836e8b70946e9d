// Small-batch decode path of e0m4_matmul with the weight operand dequantised in registers: Y[M,N] = X[M,K] *
// dequant(packed)^T for 2 <= M <= 64 and any group size.  Paper: section "Operator and lagging optimizations"
// (vector-matrix product of the decoding stage, bound by memory bandwidth) with the dequantisation of section
// "E0M4 FP4 quantization" fused in registers.
//
// Same work decomposition as the other decode kernels (a workgroup owns whole 16-row blocks over all of K, a work
// item is four consecutive 16 x 128 weight blocks, the next item is in flight while the current one is processed),
// and the dot products run on the matrix cores (v_mfma_f32_16x16x32_f16).  What differs from the group-128 kernel
// of e0m4_gemv_mfma.hip: a lane turns the 32 codes of its chunk into the dequantised weights themselves (shift,
// mask-or, minus bias, times scale in packed fp16: the bits e0m4_dequant produces), with the parameters of the
// sub-group its chunk lies in, so groups of 32 and 64 need no separate sums; and one dequantised operand serves up
// to four tiles of 16 rows of X, so 17 to 64 rows cost one pass over the weights.
//
// Operands.  MFMA number i of a block takes word i of every lane's chunk: lane (n = l%16, q = l/16) supplies the
// weights of row n, k = 32q + 8i .. 32q + 8i + 7, and the activation operand is the 16-byte piece of X at the same
// k of row l%16 of the tile, read from LDS, where X lies row by row (rows 16 bytes longer than a power of two, so
// that the 16 rows of a read fall into different bank groups).
//
// Long rows.  When the M rows of X exceed the LDS, K is walked in phases: a phase stages its part of X, visits
// that part of every row block of the workgroup, and the sums of a row block, added across the wavefronts in a
// fixed order, are accumulated in a small LDS array that is written to Y after the last phase.  Every weight byte
// is still read exactly once.
#include "e0m4_device.h"
#include "e0m4_host.h"

#include <algorithm>

namespace e0m4 {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSuper = 4;                       // weight blocks (of 128 k) per work item
constexpr int kDqWaves = 8;
constexpr int kXBlockBytes = kBlockK * 2;       // one row of X, one block: 256 bytes
constexpr int kRowPadBytes = 16;
constexpr int kLdsLimitBytes = 156 * 1024;      // of the 160 KiB of a compute unit
constexpr int kTargetWorkgroups = 256;          // one workgroup per compute unit
constexpr int kMinPhaseItems = 1;               // work items of X a phase holds at least

struct DqPlan {
    int64_t grid;
    int rb_base, rb_rem;                        // even deal of row blocks
    int kb_phase;                               // k blocks per phase (a multiple of kSuper, or all of them)
    int n_ph;
    size_t lds_bytes;
    uint32_t magic, magic_last;                 // ceil(2^32 / pieces of 8 activations per staged row), per phase kind
};

__device__ inline half2_t dq_pair(half2_t w1, half2_t bias2, half2_t scale2)
{
    return (w1 - bias2) * scale2;               // difference exact, product rounded once
}

template <int G, int MT, int W>
__global__ __launch_bounds__(W * 64) void gemv_dq_kernel(const half_t* __restrict__ X, const uint4* __restrict__ packed,
                                                         half_t* __restrict__ Y, int M, uint32_t N32, uint32_t K32,
                                                         int rb_base, int rb_rem, int kb_phase, int n_ph, uint32_t magic,
                                                         uint32_t magic_last)
{
    constexpr int kThreads = W * 64;
    constexpr int PW = block_param_words(G);            // parameter words per k block: 16, 32 or 64
    constexpr int NPL = kSuper * PW / 64;               // dword loads per lane that fetch a work item's parameters
    constexpr int MR = MT * 16;                         // rows of X the accumulators cover
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int64_t N = N32, K = K32;
    const PackedLayout<G> lay(K);
    const int nkb = (int)lay.nkb;
    const int row_stride = kb_phase * kXBlockBytes + kRowPadBytes;
    unsigned char* xs = smem;                                                   // [M] rows of one phase of X
    float* red = reinterpret_cast<float*>(smem + (size_t)M * row_stride);      // [2][W][MR][16] wavefront sums
    float* accum = red + 2 * W * MR * kBlockRows;                               // [row blocks][MR][16] (several phases)

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n_l = lane & 15, g_l = lane >> 4;         // weight row and chunk of this lane; also (row of X, k-group)
    const uint32_t fmask = frac_mask_vgpr();
    const int64_t rb0 = (int64_t)blockIdx.x * rb_base + min((int)blockIdx.x, rb_rem);
    const int n_rb = rb_base + ((int)blockIdx.x < rb_rem ? 1 : 0);
    // Weights are read with buffer loads: a wavefront-uniform resource (base of this workgroup's run of row blocks,
    // far smaller than 2 GiB), a scalar offset per block and a constant lane offset; every address is clamped into
    // the run by hand.
    const __amdgpu_buffer_rsrc_t wg_codes = make_rsrc(packed + lay.code_index(rb0, 0));
    const __amdgpu_buffer_rsrc_t wg_params = make_rsrc(reinterpret_cast<const char*>(packed) + 4 * lay.param_index(rb0, 0));
    const uint32_t rb_stride = (uint32_t)nkb * block_bytes(G);
    const uint32_t lane_code_off = lane * 16;
    const int param_words_rb = nkb * PW;
    const int pslot = lay.param_slot(g_l, n_l);         // parameter word of (chunk, row) inside a block's words

    // ---- per phase: the k blocks [kb_lo, kb_lo + nkb_ph) of every row block, as nsi work items per row block
    int kb_lo = 0, nkb_ph = min(kb_phase, nkb), nsi = (nkb_ph + kSuper - 1) / kSuper;
    int slot = 0, si = 0, nslot = 0, nitem = 0;         // current work item (row block slot, item) and the one in flight
    auto advance = [&](int& s_, int& i_) {              // W work items ahead
        i_ += W;
        while (i_ >= nsi) {
            i_ -= nsi;
            ++s_;
        }
    };
    uint4 c[kSuper];
    uint32_t pwraw[NPL];
    auto fetch_params = [&](int fs, int fi) {           // past the end the last item is read again
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, i_ = in ? fi : nsi - 1;
        const uint32_t first = (uint32_t)kb_lo * PW + i_ * (kSuper * PW);       // the item's first parameter word
        const uint32_t soff = __builtin_amdgcn_readfirstlane(s_ * rb_stride + first * 4);
        const int last = param_words_rb - 1 - (int)first;
#pragma unroll
        for (int n = 0; n < NPL; ++n)
            pwraw[n] = __builtin_amdgcn_raw_buffer_load_b32(wg_params, min(n * 64 + lane, last) * 4, (int)soff, 0);
    };
    auto fetch_code = [&](int j, int fs, int fi) {      // k blocks beyond the phase: the last block again (left out of the sums)
        const bool in = fs < n_rb;
        const uint32_t s_ = in ? fs : n_rb - 1, i_ = in ? fi : nsi - 1;
        const uint32_t kb = min((uint32_t)kb_lo + i_ * kSuper + j, (uint32_t)nkb - 1);
        const uint32_t soff = __builtin_amdgcn_readfirstlane(s_ * rb_stride + kb * kBlockCodeBytes);
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

    const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
    const half8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int ph = 0; ph < n_ph; ++ph) {
        kb_lo = ph * kb_phase;
        nkb_ph = min(kb_phase, nkb - kb_lo);
        nsi = (nkb_ph + kSuper - 1) / kSuper;
        first_item();                                   // its requests are in flight while X is staged
        if (ph > 0) __syncthreads();                    // every wavefront has finished with the previous part of X
        // stage this phase's part of the M rows: piece idx is (row idx / ph_pieces, piece idx % ph_pieces), the row
        // taken as the high half of idx * ceil(2^32 / ph_pieces) (exact while M * ph_pieces^2 < 2^32)
        {
            const int ph_pieces = nkb_ph * (kXBlockBytes / 16);
            const uint32_t mg = ph == n_ph - 1 ? magic_last : magic;
            constexpr int kBatch = 4;
            for (int base = 0; base < M * ph_pieces; base += kBatch * kThreads) {
                half8_t vb[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int idx = base + u * kThreads + t;
                    const int m = (int)__umulhi((uint32_t)idx, mg), pc = idx - m * ph_pieces;
                    const int64_t k = ((int64_t)kb_lo * (kXBlockBytes / 16) + pc) * 8;
                    vb[u] = zero8;
                    if (idx < M * ph_pieces && k < K) vb[u] = *reinterpret_cast<const half8_t*>(X + (int64_t)m * K + k);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int idx = base + u * kThreads + t;
                    const int m = (int)__umulhi((uint32_t)idx, mg), pc = idx - m * ph_pieces;
                    if (idx < M * ph_pieces) *reinterpret_cast<half8_t*>(xs + (size_t)m * row_stride + pc * 16) = vb[u];
                }
            }
        }
        __syncthreads();
        // activation operand of this lane for tile mt: row min(16 mt + l%16, M - 1) (rows beyond M repeat the last
        // one; their results are never stored), chunk l/16 of a block
        uint32_t x_lane[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) x_lane[mt] = (uint32_t)(min(16 * mt + n_l, M - 1) * row_stride + g_l * 64);

        for (int s_rb = 0; s_rb < n_rb; ++s_rb) {
            floatx4 acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = zero4;
            while (slot == s_rb) {
                uint32_t pwj[kSuper];
#pragma unroll
                for (int j = 0; j < kSuper; ++j) {
                    if (G == 32) pwj[j] = pwraw[j];
                    else pwj[j] = (uint32_t)__builtin_amdgcn_ds_bpermute((((j * PW) % 64) + pslot) * 4, (int)pwraw[(j * PW) / 64]);
                }
                fetch_params(nslot, nitem);
#pragma unroll
                for (int j = 0; j < kSuper; ++j) {
                    const int kb = si * kSuper + j;     // (inside the phase) may lie beyond it in the last item
                    const half_t sc = param_scale(pwj[j]), bi = param_bias(pwj[j]);
                    const half2_t s2 = {sc, sc}, b2 = {bi, bi};
                    const uint32_t words[4] = {c[j].x, c[j].y, c[j].z, c[j].w};
                    half8_t wq[4];
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        half2_t o[4];
                        o[0] = dq_pair(w1_pair<0>(words[w], fmask), b2, s2);
                        o[1] = dq_pair(w1_pair<1>(words[w], fmask), b2, s2);
                        o[2] = dq_pair(w1_pair<2>(words[w], fmask), b2, s2);
                        o[3] = dq_pair(w1_pair<3>(words[w], fmask), b2, s2);
                        wq[w] = *reinterpret_cast<const half8_t*>(o);
                    }
                    fetch_code(j, nslot, nitem);        // the block's registers are free: request the next item's
                    if (kb < nkb_ph) {
                        const unsigned char* xb = xs + (size_t)kb * kXBlockBytes;
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
                                const half8_t xa = *reinterpret_cast<const half8_t*>(xb + x_lane[mt] + w * 16);
                                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa, wq[w], acc[mt], 0, 0, 0);
                            }
                        }
                    }
                }
                slot = nslot;
                si = nitem;
                advance(nslot, nitem);
            }
            // the wavefronts' shares of row block s_rb are added in wavefront order; lane l holds rows 4 (l/16) ..
            // 4 (l/16) + 3 of every tile, weight row l%16
            float* mine = red + ((size_t)((s_rb & 1) * W + wave) * MR + 4 * g_l) * kBlockRows + n_l;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) mine[(16 * mt + r) * kBlockRows] = acc[mt][r];
            __syncthreads();
            for (int idx = t; idx < MR * kBlockRows; idx += kThreads) {
                const int m = idx >> 4, n = idx & 15;
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < W; ++w) s += red[((size_t)((s_rb & 1) * W + w) * MR + m) * kBlockRows + n];
                if (n_ph > 1) {                         // (a cell belongs to one thread, which adds later phases to it)
                    float* cell = accum + ((size_t)s_rb * MR + m) * kBlockRows + n;
                    *cell = ph > 0 ? *cell + s : s;
                } else {
                    const int64_t row = (rb0 + s_rb) * kBlockRows + n;
                    if (m < M && row < N) Y[(int64_t)m * N + row] = (half_t)s;
                }
            }
            // no second barrier: row block s_rb + 1 uses the other half of `red`, and nobody writes this half again
            // before passing the barrier of s_rb + 1, which the readers above reach after reading
        }
    }
    if (n_ph > 1) {                                     // every cell was last written by the thread that reads it here
        for (int s_rb = 0; s_rb < n_rb; ++s_rb)
            for (int idx = t; idx < MR * kBlockRows; idx += kThreads) {
                const int m = idx >> 4, n = idx & 15;
                const int64_t row = (rb0 + s_rb) * kBlockRows + n;
                if (m < M && row < N) Y[(int64_t)m * N + row] = (half_t)accum[((size_t)s_rb * MR + m) * kBlockRows + n];
            }
    }
}

size_t red_bytes(int mt) { return 2 * (size_t)kDqWaves * mt * 16 * kBlockRows * sizeof(float); }

bool make_dq_plan(int64_t M, int64_t N, int64_t K, DqPlan& p)
{
    if (M < 2 || M > 64 || N <= 0 || K <= 0) return false;
    const int mt = (int)((M + 15) / 16);
    const int64_t nrb = row_blocks(N), nkb = k_blocks(K), nsi = (nkb + kSuper - 1) / kSuper;
    int target = knob("gemv_workgroups");
    if (target <= 0) target = kTargetWorkgroups;
    int64_t most = (nrb + std::min<int64_t>(nrb, target) - 1) / std::min<int64_t>(nrb, target);    // row blocks of a workgroup
    // a workgroup's run of row blocks is addressed with 32-bit offsets from its first row block
    const int64_t rb_bytes = nkb * (int64_t)(kBlockCodeBytes + 4 * block_param_words(32));     // (at most, over the group sizes)
    most = std::min<int64_t>(most, std::max<int64_t>(1, ((int64_t)1 << 30) / rb_bytes));
    const size_t red = red_bytes(mt), pad = (size_t)M * kRowPadBytes, per_item = (size_t)M * kSuper * kXBlockBytes;
    const size_t x_all = (size_t)M * nkb * kXBlockBytes + pad;
    if (x_all + red <= (size_t)kLdsLimitBytes) {        // all of X at once
        p.kb_phase = (int)nkb;
        p.n_ph = 1;
        p.lds_bytes = x_all + red;
    } else {
        const size_t per_rb = (size_t)mt * 16 * kBlockRows * sizeof(float);     // accumulated sums of one row block
        const size_t min_x = pad + (size_t)std::min<int64_t>(kMinPhaseItems, nsi) * per_item;
        if (red + min_x + per_rb > (size_t)kLdsLimitBytes) return false;
        most = std::min<int64_t>(most, (int64_t)(((size_t)kLdsLimitBytes - red - min_x) / per_rb));
        const size_t fixed = red + pad + (size_t)most * per_rb;
        const int64_t fit = (int64_t)(((size_t)kLdsLimitBytes - fixed) / per_item);     // work items of X at a time
        const int64_t phases = (nsi + fit - 1) / fit;
        const int64_t nsi_ph = (nsi + phases - 1) / phases;
        p.kb_phase = (int)(nsi_ph * kSuper);
        p.n_ph = (int)((nkb + p.kb_phase - 1) / p.kb_phase);
        p.lds_bytes = fixed + (size_t)nsi_ph * per_item;
    }
    p.grid = (nrb + most - 1) / most;
    p.rb_base = (int)(nrb / p.grid);
    p.rb_rem = (int)(nrb % p.grid);
    const uint64_t pieces = (uint64_t)std::min<int64_t>(p.kb_phase, nkb) * (kXBlockBytes / 16);
    const uint64_t pieces_last = (uint64_t)(nkb - (int64_t)(p.n_ph - 1) * p.kb_phase) * (kXBlockBytes / 16);
    if ((uint64_t)M * pieces * pieces >= (1ull << 32)) return false;            // (never within the LDS limit)
    p.magic = (uint32_t)(((1ull << 32) + pieces - 1) / pieces);
    p.magic_last = (uint32_t)(((1ull << 32) + pieces_last - 1) / pieces_last);
    return p.lds_bytes <= (size_t)kLdsLimitBytes;
}

template <int G, int MT>
int launch_dq(const DqPlan& p, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream)
{
    static std::atomic<uint64_t> lds_allowed{0};
    const int arc = allow_dynamic_lds(reinterpret_cast<const void*>(&gemv_dq_kernel<G, MT, kDqWaves>), kLdsLimitBytes, lds_allowed);
    if (arc != E0M4_OK) return arc;
    hipLaunchKernelGGL((gemv_dq_kernel<G, MT, kDqWaves>), dim3((unsigned)p.grid), dim3(kDqWaves * 64), p.lds_bytes, stream,
                       static_cast<const half_t*>(X), static_cast<const uint4*>(packed), static_cast<half_t*>(Y), (int)M,
                       (uint32_t)N, (uint32_t)K, p.rb_base, p.rb_rem, p.kb_phase, p.n_ph, p.magic, p.magic_last);
    return check_launch();
}

template <int G>
int launch_dq_g(const DqPlan& p, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, hipStream_t stream)
{
    switch ((M + 15) / 16) {
        case 1: return launch_dq<G, 1>(p, X, M, packed, N, K, Y, stream);
        case 2: return launch_dq<G, 2>(p, X, M, packed, N, K, Y, stream);
        case 3: return launch_dq<G, 3>(p, X, M, packed, N, K, Y, stream);
        case 4: return launch_dq<G, 4>(p, X, M, packed, N, K, Y, stream);
        default: return E0M4_ERR_SHAPE;
    }
}

}  // namespace

bool gemv_dq_supported(int64_t M, int64_t N, int64_t K, int group, bool* whole_rows)
{
    if (group != 32 && group != 64 && group != 128) return false;
    DqPlan p;
    if (!make_dq_plan(M, N, K, p)) return false;
    if (whole_rows) *whole_rows = p.n_ph == 1;
    return true;
}

int launch_gemv_dq(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y, hipStream_t stream)
{
    DqPlan p;
    if (!make_dq_plan(M, N, K, p)) return E0M4_ERR_SHAPE;
    switch (group) {
        case 32: return launch_dq_g<32>(p, X, M, packed, N, K, Y, stream);
        case 64: return launch_dq_g<64>(p, X, M, packed, N, K, Y, stream);
        case 128: return launch_dq_g<128>(p, X, M, packed, N, K, Y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

}  // namespace e0m4
