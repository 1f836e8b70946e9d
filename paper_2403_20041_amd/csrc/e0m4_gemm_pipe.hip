// Software-pipelined tile of the prefill GEMM (paper: section "Operator and lagging optimizations",
// matrix-matrix product; dequantisation of section "E0M4 FP4 quantization" fused in registers), built
// for 256 x 256 outputs, for 128 x 256 and 64 x 256 outputs (four wavefronts side by side, two workgroups
// per compute unit) and for 128 x 128 outputs (four wavefronts 2 x 2); pipe_tile() below chooses.  The
// description is that of the large tile.
//
// Eight wavefronts (2 x 4, two per SIMD) share the tile, 128 x 64 outputs and 128 fp32 accumulator
// registers per lane each, which leaves two wavefronts per SIMD at most: little but a wavefront's own
// instruction stream can hide latency.  The stream is therefore laid out by hand, per K slice of 64
// (= 4 MFMA sub-steps of 16):
//   - activations: global -> registers (issued two slices ahead) -> LDS ring of three stages ->
//     16-byte fragments, read one sub-step ahead of their use;
//   - weights: never touch LDS.  Lane (n = l%32, h = l/32) reads the 16-byte chunk of row n with
//     k = 32h..32h+31 of the slice (two slices ahead), and word s of that chunk is dequantised
//     (shift, mask-or exponent, minus bias, times scale; packed fp16, bit-identical to
//     e0m4_dequant) one sub-step ahead of MFMA number s, whose K set is {8s..8s+7} u
//     {32+8s..32+8s+7}; the activation fragment of the same MFMA is piece 4h+s of the row.
//   - one barrier per slice, placed after sub-step 1, separates the LDS write of slice kt+1 from
//     the fragment reads that start in sub-step 3.
// The LDS tile is 128-byte rows whose eight 16-byte pieces are XOR-swizzled with (row / 2) % 8: the
// LDS of gfx950 serves a 16-byte-per-lane read 16 lanes (256 bytes, two rows of the tile) at a time,
// so 16 consecutive rows have to land in 16 different 16-byte bank groups (swizzling with row % 8, the
// right choice for 128-byte-wide LDS, costs 40 % more LDS cycles here, all of them bank conflicts).
#include "e0m4_device.h"
#include "e0m4_host.h"

#include <algorithm>
#include <type_traits>

namespace e0m4 {

namespace {

constexpr int BK = 64;
constexpr int kRowBytes = BK * 2;
constexpr int kStages = 3;
constexpr int kNumXcd = 8;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ inline half2_t dequant_pair(half2_t w1, half2_t bias2, half2_t scale2)
{
    return (w1 - bias2) * scale2;                       // difference exact, product rounded once
}

// bfloat16 member (BF): X, the embedded parameters and Y are bfloat16; the same packed codes.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
template <typename T>
__device__ inline T out_value(float v)                 // one rounding to the output type (nearest even)
{
    return (T)v;
}

// WGM x WGN wavefronts share the tile.  Built as 2 x 4 (two per SIMD, 128 x 64 each): against 2 x 2
// (one per SIMD, 128 x 128 each) that doubles the instruction issue capacity and lets one wavefront's
// waits hide behind the other's MFMAs, for twice the activation fragment traffic; 2 x 2 (accumulators in
// the 256 AGPRs, one wavefront per SIMD, 17 registers spilled) was measured 3-9 % slower on every shape.
//
// FUSED adds the operators of e0m4_matmul_fused that belong to the epilogue (paper: section "Operator and
// lagging optimizations", element-wise operators fused into their neighbours).  With the gated
// epilogue a tile covers 128 output columns: the first operand block of a wavefront holds 32 gate rows
// o .. o+31 and its second the up rows N/2 + o .. N/2 + o+31, so that a lane finds the gate and the up
// value of an output element in the same register of its two accumulator blocks and writes
// silu(gate) * up.  The residual is added before the one rounding.
struct PipeFusion {
    const half_t* residual;
    int swiglu;
    int panel;                                          // row tiles per panel of the tile numbering (0: one panel)
    int split_major;                                    // work items ordered by K split first, then by tile
    int64_t n_half;                                     // N / 2 (gated epilogue)
};

// Even scheduling of the tiles over the compute units ("stream-K").  When the tile count is not a multiple of
// the number of compute units, the last, partly filled round would leave units idle for the length of a whole
// tile.  With `enabled`, the launch has exactly one workgroup per compute unit, and each workgroup runs
//   - `rounds_dp` whole tiles (tile r * grid + position), written out directly, then
//   - its share of the remaining `rem_tiles` tiles: those tiles' K ranges, in pairs of K slices, laid end to end
//     are `rem_tiles * pairs` units, of which the workgroup at position p owns [p * U / grid, (p + 1) * U / grid):
//     at most the tail of one tile and the head of the next.
// A tile that several workgroups share is finished by whichever of them arrives last: every sharer stores its
// fp32 partial sums to a slab of the workspace (slabs of the sharers of a tile are consecutive, in K order) with
// write-through stores, one thread orders them ahead of the counter (release fence) and adds one to the tile's
// counter; the one that brings the counter to the number of sharers reads all slabs back (acquire, device-coherent
// loads), adds them in K order -- a fixed order, whoever does it -- and writes the tile.  Nobody waits for anybody,
// so a workgroup that is never scheduled next to the others cannot stall them.  The counters are zeroed by a small
// kernel before the launch.  The shared-out tiles are numbered row by row (see the kernel).
struct SkArgs {
    int enabled;
    int rounds_dp;                                      // whole tiles per workgroup
    int rem_tiles;                                      // tiles shared out in K ranges, after rounds_dp * grid whole tiles
    int pairs;                                          // K / 128: pairs of K slices per tile
    unsigned int* counters;                             // [rem_tiles], zero on entry
    float* slabs;                                       // [grid + rem_tiles][BM * BN] fp32
};

//
// The tile is BM x BN: 256 x 256 with 2 x 4 wavefronts; 128 x 256 with 1 x 4 wavefronts (the same 128 x 64 per
// wavefront, two independent workgroups per compute unit); 64 x 256 with 1 x 4 wavefronts, where the taller tiles
// would compute many rows that do not exist or leave compute units without a tile; 128 x 128 with 2 x 2 wavefronts
// (forced launches only).
//
// E8 selects the 8-bit format E0M8 (e0m8_pack.hip; G is then 128, the group of its 4-bit slots): a K slice
// of 64 is one block, a lane reads two 16-byte chunks of 16 weights per slice, and MFMA number s takes
// words 2(s%2) and 2(s%2)+1 of chunk s/2, each of which one mask-or (and one more after a rotation) turns
// into four binade values.
template <int G, int WGM, int WGN, bool FUSED, int BM, int BN, bool E8 = false, bool BF = false>
__global__ __launch_bounds__(64 * WGM * WGN, 2) void gemm_pipe_kernel(const half_t* __restrict__ X, int64_t M,
                                                             const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                             half_t* __restrict__ Y, int m_tiles, int n_tiles,
                                                             int splits, float* __restrict__ partial, PipeFusion fu,
                                                             SkArgs sk)
{
    constexpr int kThreads = 64 * WGM * WGN;
    constexpr int kStageBytes = BM * kRowBytes;
    constexpr int TM = BM / (32 * WGM), TN = BN / (32 * WGN);      // 32x32 MFMA blocks per wavefront
    constexpr int RP = kThreads / 8;                    // rows covered by one activation loader pass
    constexpr int PA = BM / RP;                         // activation loader passes
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // Work items are (tile, K split) pairs, the splits of a tile adjacent -- or, with split_major, all tiles of one
    // split before those of the next, so that the workgroups running together on an XCD are on the same K range of
    // neighbouring tiles and share operands in its L2; each XCD takes a contiguous run.
    // (even scheduling exists in the instance the launcher uses it with; elsewhere the segment loop below folds away)
    static_assert(!BF || (!FUSED && !E8), "the bfloat16 member has the plain 4-bit kernel only");
    constexpr bool kSk = !FUSED && !E8 && !BF && BM == 256 && BN == 256;
    const bool sk_on = kSk && sk.enabled;
    const int total = m_tiles * n_tiles * splits;
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    const int item = (blockIdx.x % kNumXcd) * per_xcd + blockIdx.x / kNumXcd;
    if (!sk_on && item >= total) return;
    const int KT_all = (int)(K / BK);
    // Even scheduling: this workgroup's position (consecutive positions on one XCD: they share weight rows in
    // its L2), its range of units among the shared-out tiles, and the one or two K ranges that makes.
    // (Quotients are computed on the vector unit: every one of them goes through readfirstlane, or the segment
    // loop below, its trip count included, counts as divergent and every buffer load turns into a per-lane loop.
    // All of this fits 32 bits: at most 255 shared-out tiles of at most 8192 pairs, times 256 positions.)
    const uint32_t sk_grid = gridDim.x;
    const uint32_t sk_pos = (blockIdx.x % kNumXcd) * (sk_grid / kNumXcd) + blockIdx.x / kNumXcd;
    const uint32_t sk_pairs = (uint32_t)sk.pairs;
    const uint32_t sk_units = (uint32_t)sk.rem_tiles * sk_pairs;
    // (fewer units than workgroups, which only a forced launch has: the first sk_units positions take one each, so
    // that the sharers of a tile are always consecutive positions with a share each)
    const uint32_t sk_div = sk_units < sk_grid ? (sk_units > 0 ? sk_units : 1u) : sk_grid;
    auto sk_begin = [&](uint32_t pos) -> uint32_t {     // first unit of the workgroup at `pos`
        return (uint32_t)__builtin_amdgcn_readfirstlane((int)(sk_units * (pos < sk_div ? pos : sk_div) / sk_div));
    };
    const uint32_t sk_u0 = sk_on ? sk_begin(sk_pos) : 0u, sk_u1 = sk_on ? sk_begin(sk_pos + 1) : 0u;
    const uint32_t sk_t0 = sk_u1 > sk_u0 ? (uint32_t)__builtin_amdgcn_readfirstlane((int)(sk_u0 / sk_pairs)) : 0u;  // its first tile
    int sk_segs = 0;
    if (sk_u1 > sk_u0) sk_segs = sk_u1 > (sk_t0 + 1) * sk_pairs ? 2 : 1;
    const int n_segments = sk_on ? sk.rounds_dp + sk_segs : 1;
    // the position whose range holds `unit`
    auto sk_pos_of = [&](uint32_t unit) -> int {
        uint32_t g = (uint32_t)__builtin_amdgcn_readfirstlane((int)(unit * sk_div / sk_units));
        while (sk_begin(g + 1) <= unit) ++g;
        while (sk_begin(g) > unit) --g;
        return (int)g;
    };
    // the work item of a launch without even scheduling
    const int all_tiles = m_tiles * n_tiles;
    const int plain_tile = __builtin_amdgcn_readfirstlane(fu.split_major ? item % all_tiles : item / splits);
    const int plain_split = __builtin_amdgcn_readfirstlane(fu.split_major ? item / all_tiles : item % splits);
    const int plain_kb = __builtin_amdgcn_readfirstlane(2 * (int)((int64_t)(KT_all / 2) * plain_split / splits));
    const int plain_ke = __builtin_amdgcn_readfirstlane(2 * (int)((int64_t)(KT_all / 2) * (plain_split + 1) / splits));
  for (int seg = 0; seg < n_segments; ++seg) {
    if (seg > 0) __syncthreads();                       // every wavefront has left the previous segment's LDS stages
    // what this segment computes: a tile, a range of its K slices, and where the sums go
    //   out_mode 0: the whole K range, results to Y (with the fused epilogue, if any)
    //   out_mode 1: one of `splits` K ranges, fp32 sums to slab `split` of the [splits][M][N] workspace
    //   out_mode 2: a shared-out K range (see SkArgs), fp32 sums to this sharer's slab; the last sharer finishes the tile
    int seg_tile, seg_kb, seg_ke, out_mode, seg_split = 0, sk_rt = 0, sk_first = 0, sk_sharers = 1;
    if (!sk_on) {
        seg_tile = plain_tile;
        seg_split = plain_split;
        seg_kb = plain_kb;
        seg_ke = plain_ke;
        out_mode = splits > 1 ? 1 : 0;
    } else if (seg < sk.rounds_dp) {
        seg_tile = seg * (int)sk_grid + (int)sk_pos;
        seg_kb = 0;
        seg_ke = KT_all;
        out_mode = 0;
    } else {
        sk_rt = (int)sk_t0 + (seg - sk.rounds_dp);      // the range's first tile, then its second
        const uint32_t t_lo = (uint32_t)sk_rt * sk_pairs, t_hi = t_lo + sk_pairs;
        const uint32_t lo = sk_u0 > t_lo ? sk_u0 : t_lo, hi = sk_u1 < t_hi ? sk_u1 : t_hi;
        // Which tile is shared-out tile number sk_rt: the shared tiles are the last rem_tiles of the column-by-column
        // numbering (the tail of column c0 from row tile m_start on, then whole columns); they are taken row by row
        // instead, so that the workgroups of one XCD, whose ranges are consecutive, are on tiles of the same rows of
        // X at nearly the same K (consecutive tiles start 'units per workgroup' apart): the activations, four
        // times the bytes of the weights, are then shared through that XCD's L2.
        const uint32_t first_shared = (uint32_t)sk.rounds_dp * sk_grid, mt = (uint32_t)m_tiles;
        const uint32_t c0 = first_shared / mt, m_start = first_shared - c0 * mt;
        const uint32_t w_full = (uint32_t)n_tiles - 1 - c0;         // columns after c0: shared in every row tile
        const uint32_t head = m_start * w_full;                     // shared tiles of the row tiles above m_start
        uint32_t tm, tn;
        if ((uint32_t)sk_rt < head) {
            tm = (uint32_t)sk_rt / w_full;
            tn = c0 + 1 + ((uint32_t)sk_rt - tm * w_full);
        } else {
            const uint32_t r = (uint32_t)sk_rt - head, q = r / (w_full + 1);
            tm = m_start + q;
            tn = c0 + (r - q * (w_full + 1));
        }
        seg_tile = (int)(tn * mt + tm);
        seg_kb = 2 * (int)(lo - t_lo);
        seg_ke = 2 * (int)(hi - t_lo);
        sk_first = sk_pos_of(t_lo);
        sk_sharers = sk_pos_of(t_hi - 1) - sk_first + 1;
        out_mode = sk_sharers > 1 ? 2 : 0;
    }
    // (quotients and remainders are computed on the vector unit; move them to scalar registers, or
    // everything derived from them, the K loop counter included, is treated as divergent and every
    // buffer load below turns into a per-lane loop)
    const int tile = __builtin_amdgcn_readfirstlane(seg_tile);
    const int split = __builtin_amdgcn_readfirstlane(seg_split);
    out_mode = __builtin_amdgcn_readfirstlane(out_mode);
    // (Not with even scheduling, whose shared-out tiles have a numbering of their own: measured, panels under it gain
    // or lose 2 %, 4 % lost on 2048 x 5120 x 13696.)
    // Tiles are numbered down the rows of a panel of `panel` row tiles, column after column, panel after panel: the
    // workgroups that run together on an XCD (consecutive numbers) then cover a block of panel x (their number / panel)
    // tiles and share both operands through its L2, instead of one or two whole columns of tiles.
    int tile_m = tile % m_tiles, tile_n = tile / m_tiles;
    if (!sk_on && fu.panel > 0 && fu.panel < m_tiles) {
        const int per_panel = fu.panel * n_tiles, pn = tile / per_panel;
        const int rows_p = min(fu.panel, m_tiles - pn * fu.panel), t_in = tile - pn * per_panel;
        tile_m = pn * fu.panel + t_in % rows_p;
        tile_n = t_in / rows_p;
    }
    const int64_t m0 = (int64_t)__builtin_amdgcn_readfirstlane(tile_m) * BM;
    const bool gated = FUSED && fu.swiglu;
    // first column of the tile: of the weight rows, or of the output (= of the gate rows) when gated
    const int64_t n0 = (int64_t)__builtin_amdgcn_readfirstlane(tile_n) * (gated ? BN / 2 : BN);

    // (the thread number is made opaque to the optimiser in every segment: what is derived from it -- loader
    // offsets, epilogue rows and masks -- is then computed where it is used, not ahead of the segment loop, where it
    // would hold registers through the K loop)
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t fmask = frac_mask_vgpr();
    const PackedLayout<G> lay(E8 ? 2 * K : K);
    const int64_t nrb = row_blocks(N);
    const int wm = (wave / WGN) * (BM / WGM), wn = (wave % WGN) * (BN / WGN);
    const int KT = KT_all;                              // K % 128 == 0 is required by the launcher: KT is even
    // this segment's K slices [kt_begin, kt_end): whole pairs of slices
    const int kt_begin = __builtin_amdgcn_readfirstlane(seg_kb);
    const int kt_end = __builtin_amdgcn_readfirstlane(seg_ke);

    // ---- activation loader: 8 lanes cover one 128-byte row slice; pass p handles row RP*p + t/8.
    // Rows beyond M are clamped (their products are never stored).
    // Global reads are buffer loads: a wavefront-uniform resource (base of this tile's data, in
    // scalar registers), a scalar offset that advances with the K slice, and a 32-bit per-lane
    // offset that never changes -- no vector address arithmetic inside the K loop.
    const int a_row = t >> 3, a_piece = t & 7;
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(X + m0 * K);
    uint32_t a_pass_off[PA];
#pragma unroll
    for (int p = 0; p < PA; ++p)
        a_pass_off[p] = (uint32_t)((min((int64_t)(a_row + RP * p), M - 1 - m0) * K + a_piece * 8) * 2);
    // LDS write position of this thread's piece (pass p adds RP rows)
    const uint32_t a_lds_off = (uint32_t)(a_row * kRowBytes + ((a_piece ^ ((a_row >> 1) & 7)) << 4));

    // ---- weight loader: operand block j of this wavefront covers rows n0 + wn + 32j .. +31
    const int b_h = lane >> 5, b_r = lane & 15;
    const int64_t rb_tile = n0 / kBlockRows;            // first row block of the tile (exists: n0 < N)
    const __amdgpu_buffer_rsrc_t b_code_rsrc = make_rsrc(packed + lay.code_index(rb_tile, 0));
    const __amdgpu_buffer_rsrc_t b_param_rsrc =
        make_rsrc(reinterpret_cast<const uint32_t*>(packed) + lay.param_index(rb_tile, 0));
    const uint32_t rb_stride = (uint32_t)lay.nkb * block_bytes(G);
    uint32_t b_code_off[TN], b_param_off[TN];           // row blocks beyond N are clamped (never stored)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int64_t rb = min(rb_tile + wn / kBlockRows + 2 * j + ((lane >> 4) & 1), nrb - 1) - rb_tile;
        if (gated) {                                    // block 0: gate rows, block 1: the up rows, N/2 further
            const int64_t nrbh = fu.n_half / kBlockRows;
            rb = min(rb_tile + (wave % WGN) * 2 + ((lane >> 4) & 1), nrbh - 1) - rb_tile + j * nrbh;
        }
        // 4-bit: chunk b_h of the slice; 8-bit: chunks 2 b_h and 2 b_h + 1 of the block (the second 256 bytes on)
        b_code_off[j] = (uint32_t)rb * rb_stride + (uint32_t)((E8 ? 2 * b_h : b_h) * kBlockRows + b_r) * 16;
        b_param_off[j] = (uint32_t)rb * rb_stride + (uint32_t)b_r * 4 + (G == 32 ? b_h * 64 : 0);
    }

    // ---- fragment read position: row wm + 32i + l%32 (32i rows = immediate 4096 i), piece 4h + s
    uint32_t frag_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        frag_off[s] = (uint32_t)((wm + (lane & 31)) * kRowBytes + (((4 * b_h + s) ^ ((lane >> 1) & 7)) << 4));

    u32x4 a_reg[PA];
    constexpr int NCH = E8 ? 2 : 1;                     // 16-byte chunks per lane, slice and operand block
    u32x4 bset[2][TN][NCH];
    uint32_t pwset[2][TN];
    half8_t fa[2][TM], fb[2][TN];

    auto load_a = [&](int kt) {
        const uint32_t k0 = (uint32_t)min(kt, KT - 1) * BK;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            a_reg[p] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)a_pass_off[p], (int)(k0 * 2), 0);
    };
    auto load_b = [&](int kt, int set) {
        const uint32_t k0 = (uint32_t)min(kt, KT - 1) * BK;
        // chunk (k0/32) of the row block's codes starts (k0/32)*256 bytes in; the parameter words of
        // group k0/G start (k0/G)*64 bytes into the row block's parameters
        // (8-bit: the slice is block k0/64 of 1 KiB with 16 parameter words)
        const int code_soff = E8 ? (int)((k0 / BK) * kBlockCodeBytes) : (int)((k0 / kCodesPerChunk) * (kBlockRows * 16));
        const int param_soff = E8 ? (int)((k0 / BK) * (kBlockRows * 4)) : (int)((k0 / G) * (kBlockRows * 4));
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int c = 0; c < NCH; ++c)
                bset[set][j][c] = __builtin_amdgcn_raw_buffer_load_b128(b_code_rsrc, (int)b_code_off[j] + c * kBlockRows * 16,
                                                                        code_soff, 0);
            pwset[set][j] = __builtin_amdgcn_raw_buffer_load_b32(b_param_rsrc, (int)b_param_off[j], param_soff, 0);
        }
    };
    auto store_a = [&](uint32_t stage_off) {
#pragma unroll
        for (int p = 0; p < PA; ++p)
            *reinterpret_cast<u32x4*>(smem + stage_off + a_lds_off + p * RP * kRowBytes) = a_reg[p];
    };
    auto read_frags = [&](uint32_t stage_off, int s, half8_t (&dst)[TM]) {
        const unsigned char* base = smem + stage_off + frag_off[s];
#pragma unroll
        for (int i = 0; i < TM; ++i) dst[i] = *reinterpret_cast<const half8_t*>(base + i * 32 * kRowBytes);
    };
    auto dequant_frags = [&](int set, int s, half8_t (&dst)[TN]) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const half_t sc = param_scale(pwset[set][j]), bi = param_bias(pwset[set][j]);
            const half2_t s2 = {sc, sc}, b2 = {bi, bi};
            half2_t o[4];
            if (E8) {
                const uint32_t m8 = fmask | (fmask >> 4);       // 0x03FC03FC: eight fraction bits of both halves
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const uint32_t w8 = bset[set][j][(s >> 1) * (NCH - 1)][2 * (s & 1) + h2];
                    const uint32_t lo = (w8 & m8) | kExpBits2;
                    const uint32_t hi = (__builtin_amdgcn_alignbit(w8, w8, 8) & m8) | kExpBits2;
                    o[2 * h2] = dequant_pair(__builtin_bit_cast(half2_t, lo), b2, s2);
                    o[2 * h2 + 1] = dequant_pair(__builtin_bit_cast(half2_t, hi), b2, s2);
                }
                dst[j] = *reinterpret_cast<const half8_t*>(o);
                continue;
            }
            const uint32_t word = bset[set][j][0][s];
            if (BF) {
                // bfloat16 member: the parameter word holds bfloat16 scale and bias; w1 * scale - bias * scale in one
                // fp32 fused multiply-add per weight (both products and their difference are exact: 5, 4 and 8
                // significant bits), then the one rounding to bfloat16 -- the bits e0m4_bf16_dequant produces
                const float sf = __builtin_bit_cast(float, pwset[set][j] << 16);
                const float nb = -__builtin_bit_cast(float, pwset[set][j] & 0xFFFF0000u) * sf;
                const half2_t q[4] = {w1_pair<0>(word, fmask), w1_pair<1>(word, fmask), w1_pair<2>(word, fmask),
                                      w1_pair<3>(word, fmask)};
                bf16x2_t ob[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const floatx2 f = {__builtin_fmaf((float)q[p][0], sf, nb), __builtin_fmaf((float)q[p][1], sf, nb)};
                    ob[p] = __builtin_convertvector(f, bf16x2_t);
                }
                dst[j] = *reinterpret_cast<const half8_t*>(ob);
                continue;
            }
            o[0] = dequant_pair(w1_pair<0>(word, fmask), b2, s2);
            o[1] = dequant_pair(w1_pair<1>(word, fmask), b2, s2);
            o[2] = dequant_pair(w1_pair<2>(word, fmask), b2, s2);
            o[3] = dequant_pair(w1_pair<3>(word, fmask), b2, s2);
            dst[j] = *reinterpret_cast<const half8_t*>(o);
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto mfma_block = [&](const half8_t (&a)[TM], const half8_t (&b)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = BF ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[i]),
                                                                         __builtin_bit_cast(bf16x8_t, b[j]), acc[i][j], 0, 0, 0)
                               : __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    };

    // Instruction order inside one sub-step: after every MFMA a few of the vector instructions that
    // prepare the next sub-step's operands, so that a single wavefront keeps the matrix pipe busy
    // (an MFMA of this shape occupies it for 32 cycles, its issue only for 4).
    auto interleave = [&](auto dsw, auto vmem) {
        constexpr int kMfma = TM * TN;
#pragma unroll
        for (int i = 0; i < kMfma; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // one MFMA
            if (i < TM) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS fragment read
            __builtin_amdgcn_sched_group_barrier(0x002, kMfma >= 8 ? 5 : 9, 0);     // vector ALU
            if (i < decltype(dsw)::value) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);    // LDS write
            if (i < decltype(vmem)::value) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // global load
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using IPA = std::integral_constant<int, PA>;
    using ITN2 = std::integral_constant<int, (1 + NCH) * TN>;      // loads issued by load_b

    // One K slice.  On entry: stage `cur` holds slice kt; fa[0], fb[0] hold its sub-step 0 operands;
    // bset[set] holds its codes; bset[set^1] and a_reg are in flight for slice kt+1.
    auto step = [&](int kt, int set, uint32_t cur, uint32_t nxt) {
        // sub-step 0: operands of sub-step 1; publish slice kt+1's activations and, the staging
        // registers being free again, request those of slice kt+2 at once
        read_frags(cur, 1, fa[1]);
        dequant_frags(set, 1, fb[1]);
        store_a(nxt);
        load_a(kt + 2);
        mfma_block(fa[0], fb[0]);
        interleave(IPA{}, IPA{});
        __builtin_amdgcn_sched_barrier(0);
        // sub-step 1: operands of sub-step 2
        read_frags(cur, 2, fa[0]);
        dequant_frags(set, 2, fb[0]);
        mfma_block(fa[1], fb[1]);
        interleave(I0{}, I0{});
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();                // slice kt+1 is complete in stage `nxt`
        __builtin_amdgcn_sched_barrier(0);
        // sub-step 2: operands of sub-step 3 (last use of this slice's codes)
        read_frags(cur, 3, fa[1]);
        dequant_frags(set, 3, fb[1]);
        mfma_block(fa[0], fb[0]);
        interleave(I0{}, I0{});
        __builtin_amdgcn_sched_barrier(0);
        // sub-step 3: operands of the next slice's sub-step 0; this slice's code registers are free,
        // so the codes of slice kt+2 are requested into them
        load_b(kt + 2, set);
        read_frags(nxt, 0, fa[0]);
        dequant_frags(set ^ 1, 0, fb[0]);
        mfma_block(fa[1], fb[1]);
        interleave(I0{}, ITN2{});
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- prologue
    load_a(kt_begin);
    load_b(kt_begin, 0);
    load_b(kt_begin + 1, 1);
    store_a(0);
    load_a(kt_begin + 1);
    __syncthreads();
    read_frags(0, 0, fa[0]);
    dequant_frags(0, 0, fb[0]);

    uint32_t s0 = 0, s1 = kStageBytes, s2 = 2 * kStageBytes;      // ring: current, next, the one after
    for (int kt = kt_begin; kt < kt_end; kt += 2) {
        step(kt, 0, s0, s1);
        step(kt + 1, 1, s1, s2);
        const uint32_t tmp = s0;                        // advance the ring by two slices
        s0 = s2;
        s2 = s1;
        s1 = tmp;
    }

    // accumulator layout of a 32x32 block: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
    // (n32 is made opaque to the optimiser here, after the K loop: otherwise the products of n32 with the row
    // numbers of the epilogue, invariant across the segment loop, are computed before it and held in registers
    // through the K loop: a hundred registers more, and spills in the large tile)
    uint32_t n32 = (uint32_t)N;
    asm volatile("" : "+s"(n32));
    const int rows_left = (int)min((int64_t)BM, M - m0), cols_left = (int)min((int64_t)BN, N - n0);
    const int row0 = wm + 4 * (lane >> 5), col0 = wn + (lane & 31);
    const uint32_t off0 = (uint32_t)row0 * n32 + (uint32_t)col0;
    auto store_tile = [&](auto* __restrict__ dst) {     // dst: element (m0, n0) of a row-major [M, N] array
        using out_t = std::remove_reference_t<decltype(*dst)>;
        if (rows_left >= BM && cols_left >= BN) {       // a whole tile (uniform): stores without per-element masks
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                        dst[off0 + (uint32_t)dr * n32 + 32 * j] = out_value<out_t>(acc[i][j][r]);
                    }
            return;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (col0 + 32 * j < cols_left) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                        if (row0 + dr < rows_left) dst[off0 + (uint32_t)dr * n32 + 32 * j] = out_value<out_t>(acc[i][j][r]);
                    }
            }
        }
    };
    // A shared-out K range (even scheduling): this sharer's sums go to its slab, in the order the registers hold
    // them (16 bytes per lane and store, a wavefront's stores contiguous); the sharer that arrives last adds all
    // slabs of the tile in K order and goes on to write the tile like an unshared one.
    if (kSk && out_mode == 2) {
        constexpr uint32_t kSlabStep = kThreads * 16;   // bytes between consecutive register quads of a lane
        constexpr int kCoherent = 17;                   // sc0 | sc1: written through to memory, read from memory
        uint32_t lane_off = (uint32_t)t * 16;
        asm volatile("" : "+v"(lane_off));              // (opaque, like n32: the slab offsets stay here)
        const __amdgpu_buffer_rsrc_t my_slab = make_rsrc(sk.slabs + (size_t)((int)sk_pos + sk_rt) * (size_t)(BM * BN));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const floatx4 f = {acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, f), my_slab,
                                                           (int)(lane_off + ((i * TN + j) * 4 + q4) * kSlabStep), 0, kCoherent);
                }
        // The slab is in memory before the counter moves: every thread waits for its own stores, and after the
        // barrier one thread orders them, at device scope, ahead of its addition to the counter.  (One fence per
        // workgroup: a device-scope release writes back the XCD's whole L2, and two thousand of those, one per
        // wavefront, took longer than the tiles they shared out.)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                // (also: every wavefront has left the K loop's LDS stages)
        if (t == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            const unsigned int before = __hip_atomic_fetch_add(sk.counters + sk_rt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *reinterpret_cast<volatile int*>(smem) = before + 1 == (unsigned int)sk_sharers ? 1 : 0;
        }
        __syncthreads();
        const int last = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(smem));
        if (!last) continue;
        // (acquire at device scope: nothing this XCD's caches may still hold of these slabs from an earlier launch is
        // used; the loads below are device-coherent besides)
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        // The last sharer: the tile's slabs (its own among them) added in K order, a quarter of the registers at a
        // time -- the accumulators are not needed any more, and this way the code shares nothing with the other
        // epilogues.  The loads are device-coherent: the other sharers ran on other XCDs, whose L2 this one cannot see.
        half_t* __restrict__ yt = Y + m0 * N + n0;
        // (one of the wavefront's TM row blocks at a time: two at a time measured twice as slow)
        constexpr int kAtOnce = 1;
#pragma unroll 1
        for (int i0 = 0; i0 < TM; i0 += kAtOnce) {
            floatx4 sum[kAtOnce * TN * 4];
#pragma unroll
            for (int v = 0; v < kAtOnce * TN * 4; ++v) sum[v] = floatx4{0.f, 0.f, 0.f, 0.f};
            const int quad0 = __builtin_amdgcn_readfirstlane(i0 * TN * 4 * (int)kSlabStep);
            for (int sh = 0; sh < sk_sharers; ++sh) {
                const __amdgpu_buffer_rsrc_t slab = make_rsrc(sk.slabs + (size_t)(sk_first + sk_rt + sh) * (size_t)(BM * BN));
#pragma unroll
                for (int v = 0; v < kAtOnce * TN * 4; ++v) {
                    const u32x4 d = __builtin_amdgcn_raw_buffer_load_b128(slab, (int)(lane_off + v * kSlabStep), quad0, kCoherent);
                    sum[v] += __builtin_bit_cast(floatx4, d);
                }
            }
#pragma unroll
            for (int a = 0; a < kAtOnce; ++a)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int dr = 32 * (i0 + a) + 8 * q4 + e;
                            if (col0 + 32 * j < cols_left && row0 + dr < rows_left)
                                yt[off0 + (uint32_t)dr * n32 + 32 * j] = (half_t)sum[(a * TN + j) * 4 + q4][e];
                        }
        }
        continue;
    }
    // Split K in a fixed number of ranges: this work item's fp32 partial sums go to slab `split` of the workspace
    // (row-major [splits][M][N]); a second kernel adds the slabs in split order and rounds to fp16.
    if (FUSED) {
        static_assert(!FUSED || TN == 2, "the gated epilogue pairs the two operand blocks of a wavefront");
        if (gated) {
            const int ocols_left = (int)min((int64_t)(BN / 2), fu.n_half - n0);
            const int ocol = (wave % WGN) * 32 + (lane & 31);
            if (ocol < ocols_left) {
                if (out_mode == 1) {                    // partial sums keep the [M, N] layout of the weight rows
                    float* __restrict__ pg = partial + ((size_t)split * (size_t)M + (size_t)m0) * (size_t)N + (size_t)n0;
                    float* __restrict__ pu = pg + fu.n_half;
                    const uint32_t o0 = (uint32_t)row0 * n32 + (uint32_t)ocol;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                            if (row0 + dr < rows_left) {
                                pg[o0 + (uint32_t)dr * n32] = acc[i][0][r];
                                pu[o0 + (uint32_t)dr * n32] = acc[i][1][r];
                            }
                        }
                } else {
                    uint32_t nh32 = (uint32_t)fu.n_half;
                    asm volatile("" : "+s"(nh32));             // (opaque, like n32)
                    half_t* __restrict__ yt = Y + m0 * fu.n_half + n0;
                    const half_t* __restrict__ rt = fu.residual ? fu.residual + m0 * fu.n_half + n0 : nullptr;
                    const uint32_t o0 = (uint32_t)row0 * nh32 + (uint32_t)ocol;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                            if (row0 + dr < rows_left) {
                                float v = silu_f32(acc[i][0][r]) * acc[i][1][r];
                                if (rt) v += (float)rt[o0 + (uint32_t)dr * nh32];
                                yt[o0 + (uint32_t)dr * nh32] = (half_t)v;
                            }
                        }
                }
            }
            continue;
        }
        if (out_mode != 1 && fu.residual) {
            const half_t* __restrict__ rt = fu.residual + m0 * N + n0;
            half_t* __restrict__ yt = Y + m0 * N + n0;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (col0 + 32 * j < cols_left) {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                            const uint32_t o = off0 + (uint32_t)dr * n32 + 32 * j;
                            if (row0 + dr < rows_left) yt[o] = (half_t)(acc[i][j][r] + (float)rt[o]);
                        }
                }
            }
            continue;
        }
    }
    if (out_mode == 1)
        store_tile(partial + ((size_t)split * (size_t)M + (size_t)m0) * (size_t)N + (size_t)n0);
    else
        if (BF) store_tile(reinterpret_cast<__bf16*>(Y) + m0 * N + n0);
        else store_tile(Y + m0 * N + n0);
  }
}

// The same with the fused epilogue: element i of the output is (m, j) with j < n_out; its sums are at
// [m, j] of the slabs (and, gated, [m, n_half + j]), whose rows are N long.
// V consecutive elements per thread (V = 4 needs n_out, N and N/2 to be multiples of 4).
template <int V>
__global__ __launch_bounds__(256) void splitk_reduce_fused_kernel(const float* __restrict__ partial, int splits,
                                                                  int64_t M, int64_t N, int64_t n_out,
                                                                  half_t* __restrict__ Y, PipeFusion fu)
{
    typedef float fvec __attribute__((ext_vector_type(V)));
    typedef _Float16 hvec __attribute__((ext_vector_type(V)));
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= M * n_out) return;
    const int64_t m = i / n_out, j = i - m * n_out;
    const size_t slab = (size_t)M * (size_t)N;
    const float* __restrict__ src = partial + (size_t)m * (size_t)N + (size_t)j;
    fvec v = *reinterpret_cast<const fvec*>(src);
    for (int s = 1; s < splits; ++s) v += *reinterpret_cast<const fvec*>(src + (size_t)s * slab);
    if (fu.swiglu) {
        fvec up = *reinterpret_cast<const fvec*>(src + fu.n_half);
        for (int s = 1; s < splits; ++s) up += *reinterpret_cast<const fvec*>(src + (size_t)s * slab + fu.n_half);
#pragma unroll
        for (int e = 0; e < V; ++e) v[e] = silu_f32(v[e]) * up[e];
    }
    if (fu.residual) {
        const hvec r = *reinterpret_cast<const hvec*>(fu.residual + i);
#pragma unroll
        for (int e = 0; e < V; ++e) v[e] += (float)r[e];
    }
    *reinterpret_cast<hvec*>(Y + i) = __builtin_convertvector(v, hvec);
}

// Y[i] = fp16(sum over splits, in split order, of partial[s][i]); V elements per thread.
template <int V>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int64_t count,
                                                            half_t* __restrict__ Y)
{
    typedef float fvec __attribute__((ext_vector_type(V)));
    typedef _Float16 hvec __attribute__((ext_vector_type(V)));
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= count) return;
    fvec sum = *reinterpret_cast<const fvec*>(partial + i);
    for (int s = 1; s < splits; ++s) sum += *reinterpret_cast<const fvec*>(partial + (size_t)s * count + i);
    *reinterpret_cast<hvec*>(Y + i) = __builtin_convertvector(sum, hvec);
}

// K splits: none when the tiles alone give every compute unit work, else the number the estimate below puts ahead,
// up to kMaxSplits, each split keeping at least kMinPairsPerSplit pairs of K slices.
constexpr int kComputeUnits = 256;
constexpr int kMinPairsPerSplit = 4;
constexpr int kMaxSplits = 8;

// The tile a problem gets (gemm_variant 2, 3, 4, 5 force the 256 x 256, 128 x 128, 64 x 256 and 128 x 256 tile) and
// whether the large tile runs with even scheduling (SkArgs; gemm_sk 1 forces it whenever the last round is partly
// filled, 2 forbids it) are decided by an estimate of the launch's duration.  Up to 64 rows only the 64 x 256 tile
// (four wavefronts side by side, every weight dequantised once per workgroup) makes sense; the 128 x 128 tile never
// won.  The 128 x 256 tile has the large tile's wavefront (128 x 64, 3.75 vector instructions per MFMA) in workgroups
// of four, two to a compute unit, that start and finish independently: it pads fewer rows than the large tile,
// dequantises half as often as the flat one and leaves a shorter tail (354 x 13056 x 10368: 111 us against 138 and
// 146; 2048 x 27392 x 4096: 397 against 421 with even scheduling).
//
// The estimate counts rounds: the work items (tiles times K splits) run `cap` at a time (one 256 x 256 tile per
// compute unit, two of the others), a full round takes  pairs-of-K-slices * a(1) + b  and the last, partly filled
// one  pairs * a(fill) + b  with a() piecewise linear in the fill -- a compute unit is slower the more of them run
// (one round of 160 large tiles with K = 5120 takes 112 us, one of 256 tiles 152 us, whether the workgroups read
// different tiles or all the same one: it is not the memory side), which is why filling idle units buys much less
// than their number suggests; a() has a step at half fill, where the first compute units get a second workgroup.
// A K split adds its reduction kernel (a fixed part and one per MB of partial sums), and the number of splits is the
// one with the shortest estimate; even scheduling runs its whole rounds like whole tiles and the shared-out rest on
// every unit at the full rate, and adds the slabs' cost, of which the part per sharer of a tile is serial (the last
// arriver reads them all).
// The constants are a least-squares fit (logarithm of the ratio to the measurement, rms 5.8 %) to 1301 timings of 321
// problems -- M = 65 .. 8192, N = 1024 .. 256000, K = 1024 .. 16384, groups of 32, 64 and 128, random and layer shapes
// of 2B to 14B models -- each timed with the three tiles and with even scheduling, 18 of them also with one to eight K
// splits per tile, on weights out of cache.  Choosing by the estimate costs 0.8 % over always choosing the measured
// best (geometric mean; 0.6 - 0.9 % with the fit made on two thirds and tested on the rest; 3.6 % on the 18 problems
// with their 15 candidates each; the timings themselves repeat within about 3 %).  tune_gemm_estimate.py of the Python
// package times and fits in this way.
struct PipeTile {
    int bm, bn;
    int slots;                                          // (128 x 128 tile) work items wanted before K is split no further
};
constexpr PipeTile kFlatTile{64, 256, 2 * kComputeUnits}, kMidTile{128, 128, kComputeUnits + kComputeUnits / 2},
    kBigTile{256, 256, kComputeUnits}, kHalfTile{128, 256, 2 * kComputeUnits};
constexpr int kFlatOnlyMaxM = 64;

struct TileCost {
    double lo[4];                                       // us per pair of K slices at fill 0, 1/8, 1/4, 1/2 of a round ...
    double hi[3];                                       // ... and just above 1/2, at 3/4 and 1
    double b;                                           // us per round: prologue and epilogue of a work item
    int cap;                                            // work items per round
};
constexpr TileCost kFlatCost{{0.809, 1.173, 1.302, 1.456}, {1.601, 2.034, 1.971}, 4.39, 2 * kComputeUnits};
constexpr TileCost kHalfCost{{1.427, 1.531, 1.573, 1.894}, {2.592, 3.118, 3.411}, 5.92, 2 * kComputeUnits};
constexpr TileCost kBigCost{{2.052, 2.302, 2.454, 2.523}, {2.445, 2.908, 3.461}, 9.34, kComputeUnits};
constexpr double kReduceUs = 4.87, kReduceUsPerMB = 0.176;      // reduction kernel of a K split
constexpr double kSkUs = 34.7, kSkUsPerSharer = 0.68;           // even scheduling: slabs, and the serial part per sharer
constexpr int kSplitMajorMinPairs = 16;
constexpr int kSkMinTiles = 128;                        // fewer tiles: the fixed K split (the fit holds no such launch)

double rounds_us(const TileCost& c, int64_t items, double pairs_per_item)
{
    const int64_t full = items / c.cap, rem = items % c.cap;
    double t = (double)full * (pairs_per_item * c.hi[2] + c.b);
    if (rem > 0) {
        const double fill = (double)rem / (double)c.cap;
        double a;
        if (fill <= 0.125) a = c.lo[0] + (c.lo[1] - c.lo[0]) * fill * 8.0;
        else if (fill <= 0.25) a = c.lo[1] + (c.lo[2] - c.lo[1]) * (fill - 0.125) * 8.0;
        else if (fill <= 0.5) a = c.lo[2] + (c.lo[3] - c.lo[2]) * (fill - 0.25) * 4.0;
        else if (fill <= 0.75) a = c.hi[0] + (c.hi[1] - c.hi[0]) * (fill - 0.5) * 4.0;
        else a = c.hi[1] + (c.hi[2] - c.hi[1]) * (fill - 0.75) * 4.0;
        t += pairs_per_item * a + c.b;
    }
    return t;
}

// `tiles` whole tiles (splits = 1), or each in `splits` K ranges followed by the reduction kernel
double split_launch_us(const TileCost& c, int64_t tiles, int splits, int64_t M, int64_t N, int64_t K)
{
    double us = rounds_us(c, tiles * splits, (double)(K / (2 * BK)) / splits);
    if (splits > 1) us += kReduceUs + kReduceUsPerMB * (double)splits * (double)M * (double)N * 4e-6;
    return us;
}

const TileCost* cost_of(const PipeTile& t)
{
    return t.bm == 64 ? &kFlatCost : t.bm == 256 ? &kBigCost : t.bn == 256 ? &kHalfCost : nullptr;
}

// The number of K splits of a launch with the tile `t` (gemm_splits forces one).  Which number pays depends on the
// tile count as much as on K: 1024 x 4096 x 4096 on 128 tiles of 128 x 256 takes 56 us unsplit, 44.6 in two splits
// (one work item per compute unit) and 53 in four; 256 x 4096 x 13696 on 32 such tiles 177, 95, 55 and 41 us in one,
// two, four and eight.
int choose_splits(const PipeTile& t, int64_t tiles, int64_t M, int64_t N, int64_t K)
{
    const int forced = knob("gemm_splits");
    const int64_t pairs = K / (2 * BK);
    if (forced > 0) return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(forced, pairs), kMaxSplits));   // tests: down to one pair per split
    // every compute unit already has a tile: the partial sums and their reduction cost more than a second
    // workgroup per unit gains
    if (tiles >= kComputeUnits || tiles <= 0) return 1;
    const int max_splits = (int)std::max<int64_t>(1, std::min<int64_t>(pairs / kMinPairsPerSplit, kMaxSplits));
    const TileCost* c = cost_of(t);
    if (c == nullptr)                                   // (the 128 x 128 tile, forced launches only: as many as fill its slots)
        return (int)std::max<int64_t>(1, std::min<int64_t>(t.slots / tiles, max_splits));
    int best = 1;
    double best_us = split_launch_us(*c, tiles, 1, M, N, K);
    for (int sp = 2; sp <= max_splits; ++sp) {
        const double us = split_launch_us(*c, tiles, sp, M, N, K);
        if (us < best_us) {
            best_us = us;
            best = sp;
        }
    }
    return best;
}

// whole tiles, or the K split that the estimate puts ahead, with its reduction kernel
double tile_launch_us(const PipeTile& t, const TileCost& c, int64_t M, int64_t N, int64_t K, bool whole_tiles)
{
    const int64_t tiles = ((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
    return split_launch_us(c, tiles, whole_tiles ? 1 : choose_splits(t, tiles, M, N, K), M, N, K);
}

// even scheduling of `tiles` large tiles, of which `rem` are shared out
double sk_launch_us(int64_t tiles, int64_t rem, int64_t pairs)
{
    const double sharers = std::min<double>((double)kComputeUnits / (double)rem + 1.0, (double)pairs);
    const double whole_rounds = (double)(tiles / kComputeUnits) * ((double)pairs * kBigCost.hi[2] + kBigCost.b);
    return whole_rounds + (double)rem * (double)pairs / kComputeUnits * kBigCost.hi[2] + kBigCost.b + kSkUs +
           kSkUsPerSharer * sharers;
}

constexpr size_t kSkCounterBytes = 1024;                // 255 counters at most, then the slabs (16-byte aligned)
struct SkPlan {
    bool on;
    int rounds_dp, rem_tiles, pairs;
    size_t workspace_bytes;
    double us;                                          // estimated duration of the launch when on
};

// With M = 2048, G = 128: N = 27392, K = 5120 (856 tiles) 547 -> 525 us; N = 5120, K = 13696 (160 tiles) 293 -> 275 us;
// but N = 5120, K = 5120 (160 tiles) 113 -> 133 us and N = 15360, K = 5120 (480 tiles) 286 -> 316 us.  (Shared tiles
// taken row by row, see the kernel; column by column the first two were 525 and 284.)
SkPlan sk_plan(int64_t tiles, int64_t K, int bm, int bn, bool allowed)
{
    SkPlan p{false, 0, 0, 0, 0, 0.0};
    const int forced = knob("gemm_sk");
    if (!allowed || forced == 2 || bm != 256 || bn != 256 || tiles <= 0) return p;
    p.rounds_dp = (int)(tiles / kComputeUnits);
    p.rem_tiles = (int)(tiles % kComputeUnits);
    p.pairs = (int)(K / (2 * BK));
    if (p.rem_tiles == 0 || tiles > 0x3fffffffLL || p.pairs > 8192) return p;      // (the kernel's unit arithmetic is 32-bit)
    p.us = sk_launch_us(tiles, p.rem_tiles, p.pairs);
    if (forced != 1) {
        if (tiles < kSkMinTiles) return p;
        if (p.us >= rounds_us(kBigCost, tiles, (double)p.pairs)) return p;
    }
    p.on = true;
    p.workspace_bytes = kSkCounterBytes + (size_t)(kComputeUnits + p.rem_tiles) * (size_t)bm * bn * sizeof(float);
    return p;
}

// Up to 64 rows the flat tile; above, the tile with the shortest estimate.
// (`sk_allowed`: the launch may use even scheduling; `whole_tiles`: it has no workspace, so neither that nor a K split)
PipeTile pipe_tile(int64_t M, int64_t N, int64_t K, bool sk_allowed, bool whole_tiles = false)
{
    const int v = knob("gemm_variant");
    if (v == 4) return kFlatTile;
    if (v == 3) return kMidTile;
    if (v == 2) return kBigTile;
    if (v == 5) return kHalfTile;
    if (M <= kFlatOnlyMaxM || N <= 0 || K < 2 * BK) return kFlatTile;
    const double flat_us = tile_launch_us(kFlatTile, kFlatCost, M, N, K, whole_tiles);
    const double half_us = tile_launch_us(kHalfTile, kHalfCost, M, N, K, whole_tiles);
    double big_us = tile_launch_us(kBigTile, kBigCost, M, N, K, whole_tiles);
    const SkPlan skp = sk_plan(((M + 255) / 256) * ((N + 255) / 256), K, 256, 256, sk_allowed && !whole_tiles);
    if (skp.on) big_us = std::min(big_us, skp.us);
    if (half_us < flat_us && half_us <= big_us) return kHalfTile;
    return flat_us <= big_us ? kFlatTile : kBigTile;
}

PipeTile tile_of(int bm, int bn) { return bm == 64 ? kFlatTile : bm == 256 ? kBigTile : bn == 256 ? kHalfTile : kMidTile; }

size_t partial_bytes(int splits, int64_t M, int64_t N) { return (size_t)splits * (size_t)M * (size_t)N * sizeof(float); }

__global__ void zero_u32_kernel(unsigned int* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

int64_t pipe_tiles(const PipeTile& t, int64_t M, int64_t N, bool swiglu)
{
    const int64_t n_tiles = swiglu ? (N / 2 + t.bn / 2 - 1) / (t.bn / 2) : (N + t.bn - 1) / t.bn;
    return ((M + t.bm - 1) / t.bm) * n_tiles;
}

// (`whole_tiles`: neither a K split nor the even scheduling, hence no workspace)
template <int G, int WGM, int WGN, bool FUSED, int BM, int BN, bool E8 = false, bool BF = false>
int launch_pipe(const half_t* x, int64_t M, const uint4* c, int64_t N, int64_t K, half_t* y, void* workspace,
                size_t workspace_bytes, hipStream_t stream, const Fusion& f, bool whole_tiles = false)
{
    PipeFusion fu;
    fu.residual = static_cast<const half_t*>(f.residual);
    fu.swiglu = f.swiglu ? 1 : 0;
    // Panels of four row tiles (two of the large tile): 2 to 7 % faster than whole columns of tiles from M = 2048 on (2048 x 27392 x 5120 on
    // 128 x 256 tiles: 504 -> 488 us, 2048 x 32768 x 2048: 269 -> 251; on 64 x 256 tiles 601 -> 569 and 318 -> 285; on
    // the large tile 550 -> 541 and 270 -> 254); heights of 2 to 6 tiles of 128 rows measured alike.
    // gemm_panel forces a height, -1 whole columns.
    const int panel_knob = knob("gemm_panel");
    fu.panel = panel_knob > 0 ? panel_knob : panel_knob < 0 ? 0 : BM == 256 ? 2 : 4;
    fu.split_major = 0;
    fu.n_half = N / 2;
    const PipeTile shape = tile_of(BM, BN);
    const int64_t m_tiles = (M + BM - 1) / BM;
    const int64_t tiles = pipe_tiles(shape, M, N, f.swiglu), n_tiles = tiles / m_tiles;
    const SkPlan skp = sk_plan(tiles, K, BM, BN, !FUSED && !E8 && !BF && !whole_tiles);
    const int splits = skp.on || whole_tiles ? 1 : choose_splits(shape, tiles, M, N, K);
    if (tiles * splits > 0x3fffffffLL) return E0M4_ERR_SHAPE;
    // Long K ranges gain from the order by split (1024 x 4096 x 13696 in four splits 122 -> 116 us, 512 x 2048 x 16384
    // in eight 46.9 -> 44.6), short ones lose (128 x 4608 x 4096 in eight splits of four pairs 19.6 -> 21.6, 1024 x 4608
    // x 4096 in three of ten or eleven 56.9 -> 58.5); gemm_split_order 1 forces the order by tile, 2 the order by split.
    const int order_knob = knob("gemm_split_order");
    fu.split_major = splits > 1 && (order_knob == 2 || (order_knob == 0 && K / (2 * BK) / splits >= kSplitMajorMinPairs)) ? 1 : 0;
    const int total = (int)(tiles * splits);
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    float* partial = nullptr;
    if (splits > 1) {
        if (workspace == nullptr || workspace_bytes < partial_bytes(splits, M, N)) return E0M4_ERR_WORKSPACE;
        partial = static_cast<float*>(workspace);
    }
    SkArgs sk{0, 0, 0, 0, nullptr, nullptr};
    unsigned grid = (unsigned)(per_xcd * kNumXcd);
    if (skp.on) {
        if (workspace == nullptr || workspace_bytes < skp.workspace_bytes) return E0M4_ERR_WORKSPACE;
        sk.enabled = 1;
        sk.rounds_dp = skp.rounds_dp;
        sk.rem_tiles = skp.rem_tiles;
        sk.pairs = skp.pairs;
        sk.counters = static_cast<unsigned int*>(workspace);
        sk.slabs = reinterpret_cast<float*>(static_cast<char*>(workspace) + kSkCounterBytes);
        grid = kComputeUnits;
        hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(256), 0, stream, sk.counters, skp.rem_tiles);
        const int zrc = check_launch();
        if (zrc != E0M4_OK) return zrc;
    }
    constexpr size_t lds = (size_t)kStages * BM * kRowBytes;       // 96 KiB for the large tile: above the default limit
    static std::atomic<uint64_t> lds_allowed{0};
    const int arc = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_pipe_kernel<G, WGM, WGN, FUSED, BM, BN, E8, BF>),
                                      (int)lds, lds_allowed);
    if (arc != E0M4_OK) return arc;
    hipLaunchKernelGGL((gemm_pipe_kernel<G, WGM, WGN, FUSED, BM, BN, E8, BF>), dim3(grid), dim3(64 * WGM * WGN), lds, stream, x,
                       M, c, N, K, y, (int)m_tiles, (int)n_tiles, splits, partial, fu, sk);
    int rc = check_launch();
    if (rc != E0M4_OK || splits == 1) return rc;
    if (FUSED) {
        const int64_t n_out = f.swiglu ? N / 2 : N;
        if (n_out % 4 == 0 && N % 8 == 0)
            hipLaunchKernelGGL(splitk_reduce_fused_kernel<4>, dim3((unsigned)((M * n_out / 4 + 255) / 256)), dim3(256), 0,
                               stream, partial, splits, M, N, n_out, y, fu);
        else
            hipLaunchKernelGGL(splitk_reduce_fused_kernel<1>, dim3((unsigned)((M * n_out + 255) / 256)), dim3(256), 0,
                               stream, partial, splits, M, N, n_out, y, fu);
        return check_launch();
    }
    const int64_t count = M * N;
    if (count % 4 == 0)                                 // slabs stay 16-byte aligned
        hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, stream,
                           partial, splits, count, y);
    else
        hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream,
                           partial, splits, count, y);
    return check_launch();
}

}  // namespace

bool gemm_pipe_supported(int64_t K) { return K >= 128 && (K % (2 * BK)) == 0; }

// (`fused`: the call comes from a fused matmul or the 8-bit format, whose kernels keep whole tiles or the fixed K split)
size_t gemm_pipe_workspace_bytes(int64_t M, int64_t N, int64_t K, bool swiglu, bool fused)
{
    const PipeTile shape = pipe_tile(M, N, K, !fused && !swiglu);
    const int64_t tiles = pipe_tiles(shape, M, N, swiglu);
    if (tiles == 0 || !gemm_pipe_supported(K)) return 0;
    const SkPlan skp = sk_plan(tiles, K, shape.bm, shape.bn, !fused && !swiglu);
    if (skp.on) return skp.workspace_bytes;
    const int splits = choose_splits(shape, tiles, M, N, K);
    return splits > 1 ? partial_bytes(splits, M, N) : 0;
}

namespace {

// the kernel instance of a tile
template <int G, bool FUSED, bool E8 = false, bool BF = false>
int launch_pipe_as(const PipeTile& t, const half_t* x, int64_t M, const uint4* c, int64_t N, int64_t K, half_t* y,
                   void* workspace, size_t workspace_bytes, hipStream_t stream, const Fusion& f, bool whole_tiles = false)
{
    if (t.bm == 64)
        return launch_pipe<G, 1, 4, FUSED, 64, 256, E8, BF>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f, whole_tiles);
    if (t.bm == 128 && t.bn == 256)
        return launch_pipe<G, 1, 4, FUSED, 128, 256, E8, BF>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f, whole_tiles);
    if (t.bm == 128)
        return launch_pipe<G, 2, 2, FUSED, 128, 128, E8, BF>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f, whole_tiles);
    return launch_pipe<G, 2, 4, FUSED, 256, 256, E8, BF>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f, whole_tiles);
}

template <int G, bool FUSED>
int launch_pipe_tile(const half_t* x, int64_t M, const uint4* c, int64_t N, int64_t K, half_t* y, void* workspace,
                     size_t workspace_bytes, hipStream_t stream, const Fusion& f)
{
    return launch_pipe_as<G, FUSED>(pipe_tile(M, N, K, !FUSED), x, M, c, N, K, y, workspace, workspace_bytes, stream, f);
}

}  // namespace

// 8-bit format: same tiles, K splits and workspace as the 4-bit problem of the same M, N, K.
int launch_gemm_pipe8(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y, void* workspace,
                      size_t workspace_bytes, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    return launch_pipe_as<128, false, true>(pipe_tile(M, N, K, false), x, M, c, N, K, y, workspace, workspace_bytes, stream,
                                            Fusion{});
}

int launch_gemm_pipe8_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, void* Y,
                            void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    if (f.swiglu && (N % (2 * kBlockRows) != 0 || gated_half_bytes(N, 2 * K, 128) > kMaxHalfBytes)) return E0M4_ERR_SHAPE;
    return launch_pipe_as<128, true, true>(pipe_tile(M, N, K, false), x, M, c, N, K, y, workspace, workspace_bytes, stream, f);
}

int launch_gemm_pipe(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    switch (group) {
        case 32: return launch_pipe_tile<32, false>(x, M, c, N, K, y, workspace, workspace_bytes, stream, Fusion{});
        case 64: return launch_pipe_tile<64, false>(x, M, c, N, K, y, workspace, workspace_bytes, stream, Fusion{});
        case 128: return launch_pipe_tile<128, false>(x, M, c, N, K, y, workspace, workspace_bytes, stream, Fusion{});
        default: return E0M4_ERR_GROUP;
    }
}

namespace {
// Whole tiles only (no workspace to split K into); the tile by the same estimate as for fp16, whose timings those of
// this member follow.  M = 1024: 4608 x 4096 (72 large tiles) 70 us flat against 90 large, 27392 x 4096 (428) 214
// large against 253 flat, 4096 x 13696 (64) 154 flat against 253 large; 2048 x 5120 x 5120 (160) 111 large against 132.
template <int G>
int launch_pipe_bf16(const half_t* x, int64_t M, const uint4* c, int64_t N, int64_t K, half_t* y, hipStream_t stream)
{
    return launch_pipe_as<G, false, false, true>(pipe_tile(M, N, K, false, true), x, M, c, N, K, y, nullptr, 0, stream,
                                                 Fusion{}, true);
}
}  // namespace

// bfloat16 member (X, parameters and Y bfloat16): whole tiles only, so no workspace.  At least as fast as the caller's
// 128 x 128-tile kernel on every measured shape (1.3 - 2.2 x at M = 512 ... 2048, 1.8 x at M = 64 and 128).
bool gemm_pipe_bf16_pays(int64_t M, int64_t N, int64_t K)
{
    (void)M;
    return gemm_pipe_supported(K) && N <= (int64_t)1 << 24;
}

int launch_gemm_pipe_bf16(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                          hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    switch (group) {
        case 32: return launch_pipe_bf16<32>(x, M, c, N, K, y, stream);
        case 64: return launch_pipe_bf16<64>(x, M, c, N, K, y, stream);
        case 128: return launch_pipe_bf16<128>(x, M, c, N, K, y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

// With the epilogue operators of e0m4_matmul_fused (rms-norm is applied to X before this call).  The
// gated epilogue needs N/2 to be whole pairs of row blocks and the halves less than 2 GiB apart.
int launch_gemm_pipe_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group,
                           void* Y, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    if (f.swiglu) {
        if (N % (2 * kBlockRows) != 0 || gated_half_bytes(N, K, group) > kMaxHalfBytes) return E0M4_ERR_SHAPE;
    }
    switch (group) {
        case 32: return launch_pipe_tile<32, true>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f);
        case 64: return launch_pipe_tile<64, true>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f);
        case 128: return launch_pipe_tile<128, true>(x, M, c, N, K, y, workspace, workspace_bytes, stream, f);
        default: return E0M4_ERR_GROUP;
    }
}

}  // namespace e0m4
