// Prefill path of e0m4_matmul: Y[M,N] = X[M,K] * dequant(packed)^T on the matrix
// cores.  Paper: section "Operator and lagging optimizations" (matrix-matrix
// product of the prefill stage, bound by compute) with the dequantisation of
// section "E0M4 FP4 quantization" fused into the tile loader.
//
// This file holds the dispatch between the two GEMM kernels and the small-tile
// kernel, used for problems that give the pipelined kernel too few work items
// and for K that is not a multiple of 128 (the pipelined kernel, with its three
// tile shapes, is in e0m4_gemm_pipe.hip).
//
// A workgroup (4 wavefronts, 2 x 2) owns a BM x BN tile of Y and walks K in
// slices of 64.  Per slice the activations go global -> registers -> LDS
// unchanged; the weight codes go global -> registers -> (shift, mask-or with
// the exponent, minus bias, times scale: packed fp16, one rounding, the same
// bits e0m4_dequant produces) -> LDS.  Both tiles are K-contiguous, so every
// MFMA operand is one 16-byte LDS read per lane; rows are 128 bytes and the
// eight 16-byte pieces of a row are XOR-swizzled with half the row number,
// which keeps those reads (32 rows at one k offset) and the loader's writes
// free of bank conflicts without padding.  Two LDS stages: the next slice is loaded
// into registers while the current one feeds v_mfma_f32_32x32x16_f16, written
// to the other stage, and one barrier per slice separates the two.
// Workgroups are numbered so that each XCD (own L2) works on a contiguous run of
// tiles that share weight rows.
#include "e0m4_device.h"
#include "e0m4_host.h"

namespace e0m4 {

namespace {

constexpr int BK = 64;
constexpr int kThreads = 256;
constexpr int kRowBytes = BK * 2;                       // one tile row in LDS
constexpr int kNumXcd = 8;

__device__ inline half2_t dequant_pair(half2_t w1, half2_t bias2, half2_t scale2)
{
    return (w1 - bias2) * scale2;                       // difference exact, product rounded once
}

// byte offset of 16-byte piece `piece` (0..7) of row `row` inside a swizzled tile
// (swizzled with (row / 2) % 8: the LDS of gfx950 serves 16-byte reads 16 lanes, i.e. 256 bytes or two
// tile rows, at a time, so 16 consecutive rows must fall into 16 different 16-byte bank groups)
__device__ inline int tile_off(int row, int piece) { return row * kRowBytes + ((piece ^ ((row >> 1) & 7)) << 4); }

// Epilogue operators of e0m4_matmul_fused (FUSED).  Gated: the tile covers BN/2 output columns; of the
// two 32-row operand blocks of a wavefront the first holds gate rows o .. o+31 and the second the up rows
// N/2 + o .. N/2 + o+31, and the lane that holds both values of an output element writes silu(gate) * up.
struct TileFusion {
    const half_t* residual;
    int swiglu;
    int64_t n_half;                                     // N / 2 (gated epilogue)
};

// BF: E0M4 on bfloat16 (X, the embedded parameters and Y are bfloat16; the same packed codes).  A code's value
// 2 + c/8 is taken from the fp16 pattern, the affine map runs in fp32 (difference and product exact) and is
// rounded once to bfloat16, the bits e0m4_bf16_dequant produces; the MFMA is the bfloat16 one.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
__device__ inline uint32_t bf16_pair_bits(float lo, float hi)     // two fp32 -> two bfloat16, round to nearest even
{
    const uint32_t a = __builtin_bit_cast(uint32_t, lo), b = __builtin_bit_cast(uint32_t, hi);
    return ((a + 0x7FFFu + ((a >> 16) & 1u)) >> 16) | ((b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u);
}

template <int G, int BM, int BN, bool FUSED, bool BF = false>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const half_t* __restrict__ X, int64_t M,
                                                        const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                        half_t* __restrict__ Y, int m_tiles, int n_tiles, TileFusion fu)
{
    constexpr int TM = BM / 64, TN = BN / 64;           // 32x32 MFMA blocks per wavefront along m and n
    constexpr int PA = BM / 32, PB = BN / 128;          // loader passes
    constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes, STAGE = A_BYTES + B_BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // XCD-aware numbering: workgroup w runs on XCD w % 8; give each XCD a contiguous run of tiles
    const int total = m_tiles * n_tiles;
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    const int tile = (blockIdx.x % kNumXcd) * per_xcd + blockIdx.x / kNumXcd;
    if (tile >= total) return;
    const bool gated = FUSED && fu.swiglu;
    // n0: first weight row of the tile, or first output column (= gate row) when gated
    const int64_t m0 = (int64_t)(tile % m_tiles) * BM, n0 = (int64_t)(tile / m_tiles) * (gated ? BN / 2 : BN);

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const uint32_t fmask = frac_mask_vgpr();
    const PackedLayout<G> lay(K);
    const int64_t nrb = row_blocks(N);

    // A loader: 8 lanes cover one 128-byte row slice; pass p handles rows 32p + t/8
    const int a_row = t >> 3, a_piece = t & 7;
    // B loader: 32 consecutive threads read the 512 contiguous bytes of one half block (16 rows x 64 k)
    const int b_hb = t >> 5, b_q = (t >> 4) & 1, b_r = t & 15;

    uint4 a_reg[PA];
    uint4 b_reg[PB];
    uint32_t pw_reg[PB];

    // Per-thread base addresses, computed once; inside the K loop only uniform offsets are added.
    // Rows outside M and row blocks outside N are clamped to the last valid one (their products
    // are never stored), so the loads need no per-element predicate.
    const int64_t a_m = min(m0 + a_row, M - 1);
    const char* a_base = reinterpret_cast<const char*>(X + a_m * K + a_piece * 8);
    uint32_t a_pass_off[PA];                            // byte offset of pass p's row from pass 0's row
#pragma unroll
    for (int p = 0; p < PA; ++p)
        a_pass_off[p] = (uint32_t)((min(m0 + a_row + 32 * p, M - 1) - a_m) * K * 2);
    const int64_t rb_first = n0 / kBlockRows + b_hb;
    int64_t rb_c = min(rb_first, nrb - 1);
    if (gated) {
        // tile row block b_hb belongs to wavefront column b_hb / 4, operand block (b_hb / 2) % 2 (0: gate,
        // 1: up), and is row block b_hb % 2 of that operand block's 32 rows
        static_assert(!FUSED || (BN == 128 && PB == 1), "gated epilogue: one loader pass, two wavefront columns");
        const int64_t nrbh = fu.n_half / kBlockRows;
        rb_c = ((b_hb >> 1) & 1) * nrbh + min(n0 / kBlockRows + 2 * (b_hb >> 2) + (b_hb & 1), nrbh - 1);
    }
    const char* b_code_base = reinterpret_cast<const char*>(packed + lay.code_index(rb_c, 0) + b_q * kBlockRows + b_r);
    const char* b_param_base = reinterpret_cast<const char*>(packed) + 4 * (lay.param_index(rb_c, 0) + b_r) +
                               (G == 32 ? b_q * 64 : 0);
    uint32_t b_pass_off[PB];
#pragma unroll
    for (int p = 0; p < PB; ++p)
        b_pass_off[p] = gated ? 0u : (uint32_t)((min(rb_first + 8 * p, nrb - 1) - rb_c) * lay.nkb * block_bytes(G));
    const bool k_tail = (K % BK) != 0;                  // only then can a 16-byte piece of X lie beyond K

    auto load_global = [&](int kt) {
        const uint32_t k0 = (uint32_t)kt * BK;
        const bool a_ok = !k_tail || (int64_t)k0 + a_piece * 8 < K;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            a_reg[p] = make_uint4(0, 0, 0, 0);
            if (a_ok) a_reg[p] = *reinterpret_cast<const uint4*>(a_base + (a_pass_off[p] + k0 * 2));
        }
        // chunk q of k block kb starts (k0/32) * 256 bytes into the row block's codes; the parameter
        // words of (kb, sub-group) follow the same order
        const uint32_t code_off = (k0 / kCodesPerChunk) * (kBlockRows * 16);
        const uint32_t param_off = (k0 / G) * (kBlockRows * 4);
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            b_reg[p] = *reinterpret_cast<const uint4*>(b_code_base + (b_pass_off[p] + code_off));
            pw_reg[p] = *reinterpret_cast<const uint32_t*>(b_param_base + (b_pass_off[p] + param_off));
        }
    };

    auto store_lds = [&](unsigned char* stage) {
#pragma unroll
        for (int p = 0; p < PA; ++p)
            *reinterpret_cast<uint4*>(stage + tile_off(a_row + 32 * p, a_piece)) = a_reg[p];
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const half_t sc = param_scale(pw_reg[p]), bi = param_bias(pw_reg[p]);
            const half2_t s2 = {sc, sc}, b2 = {bi, bi};
            const uint32_t words[4] = {b_reg[p].x, b_reg[p].y, b_reg[p].z, b_reg[p].w};
            const int row = (b_hb + 8 * p) * kBlockRows + b_r;
            if (BF) {
                const float sf = __builtin_bit_cast(float, pw_reg[p] << 16);
                const float bf = __builtin_bit_cast(float, pw_reg[p] & 0xFFFF0000u);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const half2_t q[4] = {w1_pair<0>(words[w], fmask), w1_pair<1>(words[w], fmask),
                                          w1_pair<2>(words[w], fmask), w1_pair<3>(words[w], fmask)};
                    uint4 o;
                    o.x = bf16_pair_bits(((float)q[0][0] - bf) * sf, ((float)q[0][1] - bf) * sf);
                    o.y = bf16_pair_bits(((float)q[1][0] - bf) * sf, ((float)q[1][1] - bf) * sf);
                    o.z = bf16_pair_bits(((float)q[2][0] - bf) * sf, ((float)q[2][1] - bf) * sf);
                    o.w = bf16_pair_bits(((float)q[3][0] - bf) * sf, ((float)q[3][1] - bf) * sf);
                    *reinterpret_cast<uint4*>(stage + A_BYTES + tile_off(row, b_q * 4 + w)) = o;
                }
                continue;
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                half2_t o[4];
                o[0] = dequant_pair(w1_pair<0>(words[w], fmask), b2, s2);
                o[1] = dequant_pair(w1_pair<1>(words[w], fmask), b2, s2);
                o[2] = dequant_pair(w1_pair<2>(words[w], fmask), b2, s2);
                o[3] = dequant_pair(w1_pair<3>(words[w], fmask), b2, s2);
                *reinterpret_cast<uint4*>(stage + A_BYTES + tile_off(row, b_q * 4 + w)) = *reinterpret_cast<const uint4*>(o);
            }
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // wavefront tile origin inside the block tile, and this lane's fragment row / k piece
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
    const int frag_row = lane & 31, frag_piece = lane >> 5;

    auto compute = [&](const unsigned char* stage) {
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            half8_t a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[i] = *reinterpret_cast<const half8_t*>(stage + tile_off(wm + 32 * i + frag_row, 2 * s + frag_piece));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[j] = *reinterpret_cast<const half8_t*>(stage + A_BYTES + tile_off(wn + 32 * j + frag_row, 2 * s + frag_piece));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (BF)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[i]),
                                                                            __builtin_bit_cast(bf16x8_t, b[j]), acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
                }
        }
    };

    const int KT = (int)((K + BK - 1) / BK);
    load_global(0);
    store_lds(smem);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        unsigned char* cur = smem + (kt & 1) * STAGE;
        unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
        if (kt + 1 < KT) load_global(kt + 1);
        compute(cur);
        if (kt + 1 < KT) store_lds(nxt);
        __syncthreads();
    }

    // accumulator layout of a 32x32 block: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
    // (tile-local offsets fit 32 bits: at most 256 rows of N elements)
    half_t* __restrict__ Yt = Y + m0 * N + n0;
    const uint32_t n32 = (uint32_t)N;
    const int rows_left = (int)min((int64_t)BM, M - m0), cols_left = (int)min((int64_t)BN, N - n0);
    const int row0 = wm + 4 * (lane >> 5), col0 = wn + (lane & 31);
    const uint32_t off0 = (uint32_t)row0 * n32 + (uint32_t)col0;
    if (FUSED) {
        if (gated) {
            const int ocols_left = (int)min((int64_t)(BN / 2), fu.n_half - n0);
            const int ocol = (wave & 1) * 32 + (lane & 31);
            const uint32_t nh32 = (uint32_t)fu.n_half;
            half_t* __restrict__ yt = Y + m0 * fu.n_half + n0;
            const half_t* __restrict__ rt = fu.residual ? fu.residual + m0 * fu.n_half + n0 : nullptr;
            const uint32_t o0 = (uint32_t)row0 * nh32 + (uint32_t)ocol;
            if (ocol < ocols_left) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                        if (row0 + dr < rows_left) {
                            float v = silu_f32(acc[i][0][r]) * acc[i][TN - 1][r];
                            if (rt) v += (float)rt[o0 + (uint32_t)dr * nh32];
                            yt[o0 + (uint32_t)dr * nh32] = (half_t)v;
                        }
                    }
            }
            return;
        }
        if (fu.residual) {
            const half_t* __restrict__ rt = fu.residual + m0 * N + n0;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (col0 + 32 * j < cols_left) {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = 32 * i + 8 * (r >> 2) + (r & 3);
                            const uint32_t o = off0 + (uint32_t)dr * n32 + 32 * j;
                            if (row0 + dr < rows_left) Yt[o] = (half_t)(acc[i][j][r] + (float)rt[o]);
                        }
                }
            }
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        if (col0 + 32 * j < cols_left) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * i + 8 * (r >> 2) + (r & 3);       // compile-time row step
                    if (row0 + dr < rows_left) {
                        const float v = acc[i][j][r];
                        Yt[off0 + (uint32_t)dr * n32 + 32 * j] =
                            BF ? __builtin_bit_cast(half_t, (uint16_t)bf16_pair_bits(v, 0.f)) : (half_t)v;
                    }
                }
        }
    }
}

template <int G, int BM, int BN, bool FUSED, bool BF = false>
int launch_tile(const half_t* x, int64_t M, const uint4* c, int64_t N, int64_t K, half_t* y, hipStream_t stream,
                const Fusion& f = Fusion{})
{
    TileFusion fu;
    fu.residual = static_cast<const half_t*>(f.residual);
    fu.swiglu = f.swiglu ? 1 : 0;
    fu.n_half = N / 2;
    const int64_t m_tiles = (M + BM - 1) / BM;
    const int64_t n_tiles = f.swiglu ? (N / 2 + BN / 2 - 1) / (BN / 2) : (N + BN - 1) / BN;
    if (m_tiles * n_tiles > 0x3fffffffLL) return E0M4_ERR_SHAPE;
    const int total = (int)(m_tiles * n_tiles);
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    constexpr size_t lds = 2 * (size_t)(BM + BN) * kRowBytes;
    static std::atomic<uint64_t> lds_allowed{0};        // LDS above the default 64 KiB limit must be requested
    const int arc = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_kernel<G, BM, BN, FUSED, BF>), (int)lds, lds_allowed);
    if (arc != E0M4_OK) return arc;
    hipLaunchKernelGGL((gemm_kernel<G, BM, BN, FUSED, BF>), dim3((unsigned)(per_xcd * kNumXcd)), dim3(kThreads), lds, stream,
                       x, M, c, N, K, y, (int)m_tiles, (int)n_tiles, fu);
    return check_launch();
}

// The pipelined kernel runs whenever it can (K a multiple of 128): with its three tiles and the K split it was
// never slower than the kernel of this file on any measured shape, and up to 2.7x faster on small ones
// (M = 17..96, 2048 x 2048: 12 us against 31).  gemm_variant 1 forces the kernel of this file.
bool use_pipe(int64_t M, int64_t N, int64_t K, bool swiglu = false)
{
    (void)M; (void)N; (void)swiglu;
    return gemm_pipe_supported(K) && knob("gemm_variant") != 1;
}

}  // namespace

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, bool swiglu, bool fused)
{
    return use_pipe(M, N, K, swiglu) ? gemm_pipe_workspace_bytes(M, N, K, swiglu, fused) : 0;
}

int launch_gemm(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    if (use_pipe(M, N, K)) return launch_gemm_pipe(X, M, packed, N, K, group, Y, workspace, workspace_bytes, stream);
    switch (group) {
        case 32: return launch_tile<32, 128, 128, false>(x, M, c, N, K, y, stream);
        case 64: return launch_tile<64, 128, 128, false>(x, M, c, N, K, y, stream);
        case 128: return launch_tile<128, 128, 128, false>(x, M, c, N, K, y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

// E0M4 on bfloat16, any M: the pipelined kernel in whole tiles when K is a multiple of 128, else the small-tile kernel
// with the bfloat16 operand path; no K split, no workspace.  (gemm_variant 1 forces the small-tile kernel, 2 to 4 the
// pipelined kernel with that tile.)
int launch_gemm_bf16(const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group, void* Y,
                     hipStream_t stream)
{
    if (knob("gemm_variant") != 1 && gemm_pipe_bf16_pays(M, N, K))
        return launch_gemm_pipe_bf16(X, M, packed, N, K, group, Y, stream);
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    switch (group) {
        case 32: return launch_tile<32, 128, 128, false, true>(x, M, c, N, K, y, stream);
        case 64: return launch_tile<64, 128, 128, false, true>(x, M, c, N, K, y, stream);
        case 128: return launch_tile<128, 128, 128, false, true>(x, M, c, N, K, y, stream);
        default: return E0M4_ERR_GROUP;
    }
}

// With the epilogue operators of e0m4_matmul_fused; X is already normalised if rms-norm was asked for.
int launch_gemm_fused(const Fusion& f, const void* X, int64_t M, const void* packed, int64_t N, int64_t K, int group,
                      void* Y, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const half_t* x = static_cast<const half_t*>(X);
    const uint4* c = static_cast<const uint4*>(packed);
    half_t* y = static_cast<half_t*>(Y);
    if (f.swiglu) {
        if (N % (2 * kBlockRows) != 0 || gated_half_bytes(N, K, group) > kMaxHalfBytes) return E0M4_ERR_SHAPE;
    }
    if (use_pipe(M, N, K, f.swiglu))
        return launch_gemm_pipe_fused(f, X, M, packed, N, K, group, Y, workspace, workspace_bytes, stream);
    switch (group) {
        case 32: return launch_tile<32, 128, 128, true>(x, M, c, N, K, y, stream, f);
        case 64: return launch_tile<64, 128, 128, true>(x, M, c, N, K, y, stream, f);
        case 128: return launch_tile<128, 128, 128, true>(x, M, c, N, K, y, stream, f);
        default: return E0M4_ERR_GROUP;
    }
}

}  // namespace e0m4
