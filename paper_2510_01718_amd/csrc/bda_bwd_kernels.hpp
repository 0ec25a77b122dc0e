// Gradient kernels of the BD K/V projection (Section "BDA Training Evaluation": C is a learnable
// parameter and gradients flow through steps 2-3 of Algorithm "BD Attention Inference").
//
// With out[t, n] = c[t, off_g + (n - col0_g) % d_h] + sum_i c[t, Bbar_g(i)] C[i, n] and G = dL/d out:
//
//   latent gradient  gc[t, l] = sum_g sum_{n in group g} G[t, n] Wfull_g[l, n]
//                    Wfull_g[l, n] = C[rank_g(l), n]             for l outside the window of g
//                                  = [l - off_g == (n - col0_g) % d_h]   for l inside it
//   weight gradient  gC[i, n] = sum_t c[t, Bbar_g(i)] G[t, n]
//
// Both are GEMMs of the forward's size with other operand layouts.  The latent gradient contracts
// over the output columns n, along which both G and C are contiguous, so both tiles go from global
// memory to LDS as they are; the window rows of Wfull are an identity pattern that is never
// loaded: where a 32-column MFMA tile of gc meets the window, the staged G fragment is multiplied
// by a constant 0/1 fragment, which sums the heads' gradients in float32 inside the accumulator.
// The weight gradient contracts over the tokens t, along which neither c nor G is contiguous, so
// both tiles keep their memory layout in LDS and the fragments come from transposing LDS reads.
//
// Both contract over thousands of elements into few output tiles (T x d_c and (d_c - d_h) x N are
// small next to T x N), so a launch has about one workgroup per compute unit and each workgroup a
// long, latency-bound loop.  Two measures keep enough loads in flight:
//   * a workgroup is 8 waves = 2 halves of 2 x 2 waves; the halves take alternate contraction chunks
//     of 64 of the SAME output tile through LDS tiles of their own, and their float32 accumulators
//     are added through LDS at the end (a fixed order: results do not depend on timing);
//   * every half keeps three or four chunks in flight: chunk k + depth is being fetched into
//     registers while chunk k is multiplied from LDS and the chunks between wait in registers.
// Each wave owns TT x TN MFMA tiles of 32 x 32 (v_mfma_f32_32x32x16); the operand whose index is
// contiguous in the OUTPUT is the MFMA's row operand, so that each lane stores four consecutive
// elements.
#pragma once
#include <type_traits>

#include "bda_gemm_kernels.hpp"

namespace bda {

struct BwdArgs {
    const void* c;    // T x d_c latent
    const void* g;    // T x N upstream gradient
    const void* C;    // K x N coefficients (latent gradient only)
    void* out;        // gc (T x d_c) or gC (K x N)
    int64_t ldc, ldg, ldC, ldo;          // in elements
    int64_t T;
    int d_c, d_h, K;                     // K = d_c - d_h
    int n_groups;
    int m_tiles, n_tiles;                // tile grid: rows x columns of the output
    int tile_start[kMaxGroups + 1];      // weight gradient: first column tile of each group
    int64_t col_start[kMaxGroups + 1];   // first output column of each group
    int a_off[kMaxGroups];               // basis window start of each group
};

template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

// Register sets of the software pipeline: chunk k + depth is being fetched while chunk k is
// multiplied (LDS holds chunks k and k + 1).  As many as the register file allows at two waves per
// SIMD.
template <int TT, int TN>
constexpr int bwd_depth() { return TT * TN >= 4 ? 3 : 4; }

// 0/1 fragment (MFMA row operand, one k-step of 16): row i = l31 has a one at k' = i - d.
template <typename X>
__device__ __forceinline__ u32x4 shifted_identity_frag(int d, int l31, int lhi)
{
    u32x4 f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int k0 = d + 8 * lhi + 2 * w;
        f[w] = (k0 == l31 ? IdentityFrag<X>::one : 0u) | (k0 + 1 == l31 ? IdentityFrag<X>::one << 16 : 0u);
    }
    return f;
}

// Tiles are dealt to the dies in contiguous runs (workgroup b runs on die b % 8), so that tiles
// that are neighbours in the run order -- they share one operand -- meet in the same L2.
__device__ __forceinline__ int bwd_tile_of_block(int total)
{
    const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    const int tile = (blockIdx.x % kNumXcd) * per_xcd + slot;
    return (slot < per_xcd && tile < total) ? tile : -1;
}

template <typename X, typename OutT, int TT, int TN>
__device__ __forceinline__ void bwd_epilogue(const f32x16 (&acc)[TN][TT], __amdgpu_buffer_rsrc_t rD, int64_t ldo,
                                             int cols_left, int wt, int wn, int l31, int lhi)
{
    const uint32_t ep_lane = (uint32_t)(wt * (32 * TT) + l31) * (uint32_t)(ldo * sizeof(OutT)) +
                             (uint32_t)(wn * (32 * TN) + lhi * 4) * (uint32_t)sizeof(OutT);
    const uint32_t ep_row_step = 32u * (uint32_t)(ldo * sizeof(OutT));
#pragma unroll
    for (int ti = 0; ti < TT; ++ti) {
        const uint32_t row_off = ep_lane + (uint32_t)ti * ep_row_step;
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int c0 = ni * 32 + rg * 8;
                if (wn * (32 * TN) + c0 >= cols_left) continue;   // uniform per wave: widths are multiples of 8
                const uint32_t off = row_off + (uint32_t)c0 * (uint32_t)sizeof(OutT);
                if constexpr (sizeof(OutT) == 4) {
                    const float e0 = acc[ni][ti][rg * 4 + 0], e1 = acc[ni][ti][rg * 4 + 1];
                    const float e2 = acc[ni][ti][rg * 4 + 2], e3 = acc[ni][ti][rg * 4 + 3];
                    const f32x4 vf = {e0, e1, e2, e3};
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vf), rD, off, 0, 0);
                } else {
                    u32x2 v;
                    v[0] = X::pack2(acc[ni][ti][rg * 4 + 0], acc[ni][ti][rg * 4 + 1]);
                    v[1] = X::pack2(acc[ni][ti][rg * 4 + 2], acc[ni][ti][rg * 4 + 3]);
                    __builtin_amdgcn_raw_buffer_store_b64(v, rD, off, 0, 0);
                }
            }
        }
    }
}

// LDS of one workgroup: [half 0: tok 0 | tok 1 | wgt 0 | wgt 1][half 1: the same]; after the main
// loop the same memory carries half 1's accumulators to half 0.
template <int TT, int TN>
struct BwdLds {
    static constexpr int BT = 64 * TT, BN = 64 * TN;
    static constexpr int TOK_STAGE = BT * kRowBytes, WGT_STAGE = BN * kRowBytes;
    static constexpr int WGT_BASE = 2 * TOK_STAGE;
    static constexpr int HALF = 2 * (TOK_STAGE + WGT_STAGE);
    static constexpr int BYTES = 2 * HALF;
    static_assert(4 * TT * TN * 16 * 64 * 4 <= BYTES, "accumulator exchange must fit the staging memory");
};

// One staged chunk: 4 k-steps of TT x TN MFMAs; `extra(ks, ft)` may add MFMAs that reuse the column
// operand's fragments.
template <typename X, int TT, int TN, typename Extra>
__device__ __forceinline__ void bwd_mma_chunk(const unsigned char* tok_s, const unsigned char* wgt_s,
                                              f32x16 (&acc)[TN][TT], Extra&& extra)
{
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        u32x4 fw[TN], ft[TT];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) fw[ni] = *(const u32x4*)(wgt_s + ni * 32 * kRowBytes + ks * 32);
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) ft[ti] = *(const u32x4*)(tok_s + ti * 32 * kRowBytes + ks * 32);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(fw[ni], ft[ti], acc[ni][ti]);
        extra(ks, ft);
    }
}

// Adds half 1's accumulators to half 0's through LDS (all 8 waves call this after the last chunk).
template <int TT, int TN>
__device__ __forceinline__ void bwd_reduce_halves(unsigned char* smem, f32x16 (&acc)[TN][TT], int half, int w4, int lane)
{
    __syncthreads();   // every wave is done reading the staged tiles
    float* x = (float*)smem + (w4 * (TT * TN * 16)) * 64 + lane;
    if (half == 1) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti)
#pragma unroll
                for (int r = 0; r < 16; ++r) x[((ni * TT + ti) * 16 + r) * 64] = acc[ni][ti][r];
    }
    __syncthreads();
    if (half == 0) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ni][ti][r] += x[((ni * TT + ti) * 16 + r) * 64];
    }
}

// ---------------------------------------------------------------------------------------------
// Latent gradient.  Output tile: (64 TT) tokens x (64 TN) latent columns.  Column operand ("tok")
// = G rows, row operand ("wgt") = rows of Wfull, one per latent column of the tile.
// ---------------------------------------------------------------------------------------------
template <typename X, typename OutT, int TT, int TN>
__global__ __launch_bounds__(512) void bwd_latent_kernel(const BwdArgs p)
{
    using L = BwdLds<TT, TN>;
    constexpr int BT = L::BT, BN = L::BN;
    constexpr int TOK_LOADS = BT / 32, WGT_LOADS = BN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tile = bwd_tile_of_block(p.m_tiles * p.n_tiles);
    if (tile < 0) return;
    const int mt = tile / p.n_tiles, nt = tile % p.n_tiles;   // the column tiles of one token tile share its G rows

    const int tid = threadIdx.x & 255;                        // thread within its half
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = wave >> 2, w4 = wave & 3;
    const int wt = w4 >> 1, wn = w4 & 1;
    const int l31 = lane & 31, lhi = lane >> 5;
    const int tq = tid & 7, trow = tid >> 3;
    unsigned char* const lds = smem + half * L::HALF;

    const int64_t t0 = (int64_t)mt * BT;
    const int64_t rows_left = p.T - t0;
    const int l0 = nt * BN;
    const int cols_left = p.d_c - l0 > BN ? BN : p.d_c - l0;
    const int64_t N = p.col_start[p.n_groups];

    const __amdgpu_buffer_rsrc_t rG = make_rsrc((const char*)p.g + t0 * p.ldg * 2, ((rows_left - 1) * p.ldg + N) * 2);
    const __amdgpu_buffer_rsrc_t rC = make_rsrc(p.C, ((int64_t)(p.K - 1) * p.ldC + N) * 2);
    const __amdgpu_buffer_rsrc_t rD = make_rsrc((char*)p.out + (t0 * p.ldo + l0) * (int64_t)sizeof(OutT),
                                                ((rows_left - 1) * p.ldo + cols_left) * (int64_t)sizeof(OutT));
    const uint32_t g_row_bytes = (uint32_t)(p.ldg * 2), c_row_bytes = (uint32_t)(p.ldC * 2);

    int n_chunks = 0;
    for (int g = 0; g < p.n_groups; ++g) n_chunks += (int)((p.col_start[g + 1] - p.col_start[g] + 63) >> 6);
    const int n_it = (n_chunks + 1) >> 1;                     // chunks of this half: 2 it + half

    // Cursor over this half's chunks (every second chunk of 64 output columns; chunks never
    // straddle groups).  All scalar; the group tables are read again only when a group ends.
    struct Cursor {
        int g, q, cnt;      // group, chunk within the group, chunks of the group
        int start, end;     // output columns of the group
        int off;            // basis window start of the group
        int jc;             // (64 q) % d_h: window column of the chunk's first output column
        bool valid;
    };
    auto enter_group = [&](Cursor& k) {
        k.start = (int)p.col_start[k.g];
        k.end = (int)p.col_start[k.g + 1];
        k.cnt = (k.end - k.start + 63) >> 6;
        k.off = p.a_off[k.g];
    };
    auto settle = [&](Cursor& k) {        // moves on while q lies beyond the group's chunks
        bool crossed = false;
        while (k.valid && k.q >= k.cnt) {
            k.q -= k.cnt;
            if (++k.g >= p.n_groups) k.valid = false;
            else enter_group(k);
            crossed = true;
        }
        if (crossed) k.jc = 64 * k.q;
        while (k.jc >= p.d_h) k.jc -= p.d_h;
    };
    auto advance = [&](Cursor& k) {
        if (!k.valid) return;
        k.q += 2;
        k.jc += 128;
        settle(k);
    };
    Cursor cur;                           // chunk being multiplied
    cur.g = 0;
    cur.q = half;
    cur.jc = 64 * half;
    cur.valid = true;
    enter_group(cur);
    settle(cur);
    Cursor ld = cur;                      // chunk being fetched: D iterations ahead

    // per-lane pieces of the load offsets that do not depend on the chunk; the rows of C that the
    // tile's latent columns map to depend on the group's window and are redone when the fetch
    // cursor enters another group.
    uint32_t tok_base[TOK_LOADS], wgt_base[WGT_LOADS];
#pragma unroll
    for (int i = 0; i < TOK_LOADS; ++i) tok_base[i] = (uint32_t)(trow + 32 * i) * g_row_bytes + (uint32_t)(tq * 16);
    int base_group = -1;
    auto set_wgt_base = [&](int off) {
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) {
            const int l = l0 + trow + 32 * i;                                 // latent column of this LDS row
            const int row = l < off ? l : l - p.d_h;                          // its row of C
            const bool ok = l < p.d_c && (l < off || l >= off + p.d_h);
            wgt_base[i] = ok ? (uint32_t)row * c_row_bytes + (uint32_t)(tq * 16) : kBadOffset;
        }
    };

    constexpr int D = bwd_depth<TT, TN>();
    u32x4 tok_reg[D][TOK_LOADS], wgt_reg[D][WGT_LOADS];
    auto load_chunk = [&](auto set, const Cursor& k) {
        constexpr int S = decltype(set)::value;
        if (k.g != base_group) {          // uniform; first chunk and group changes only
            set_wgt_base(k.off);
            base_group = k.g;
        }
        const int nc = k.start + 64 * k.q;
        const int rem = k.valid ? k.end - nc : 0;             // columns of the group from nc on
        const bool col_ok = tq * 8 < rem;
        const uint32_t chunk_bytes = (uint32_t)nc * 2u;
#pragma unroll
        for (int i = 0; i < TOK_LOADS; ++i) {
            uint32_t voff = col_ok ? tok_base[i] + chunk_bytes : kBadOffset;
            asm volatile("" : "+v"(voff));                    // one load, not one per branch
            tok_reg[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rG, voff, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) {
            uint32_t voff = (col_ok && wgt_base[i] != kBadOffset) ? wgt_base[i] + chunk_bytes : kBadOffset;
            asm volatile("" : "+v"(voff));
            wgt_reg[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rC, voff, 0, 0);
        }
    };
    auto store_chunk = [&](auto set, auto stage) {
        constexpr int S = decltype(set)::value, LS = decltype(stage)::value;
        unsigned char* tok_s = lds + LS * L::TOK_STAGE;
        unsigned char* wgt_s = lds + L::WGT_BASE + LS * L::WGT_STAGE;
#pragma unroll
        for (int i = 0; i < TOK_LOADS; ++i) *(u32x4*)(tok_s + lds_off(trow + 32 * i, tq)) = tok_reg[S][i];
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) *(u32x4*)(wgt_s + lds_off(trow + 32 * i, tq)) = wgt_reg[S][i];
    };

    f32x16 acc[TN][TT];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int ti = 0; ti < TT; ++ti)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ni][ti][r] = 0.0f;

    const int tok_rd = (wt * (32 * TT) + l31) * kRowBytes + lhi * 16;
    const int wgt_rd = L::WGT_BASE + (wn * (32 * TN) + l31) * kRowBytes + lhi * 16;
    const int colm0 = l0 + wn * (32 * TN);           // first latent column of this wave's MFMA tiles

    // iteration k multiplies this half's chunk k (`cur`) from LDS stage k % 2, fetches chunk k + D
    // (`ld`) into register set k % D and moves chunk k + 1 from register set (k + 1) % D to LDS
    auto iteration = [&](auto set, auto stage) {
        constexpr int S = decltype(set)::value, LS = decltype(stage)::value;
        load_chunk(set, ld);
        advance(ld);
        if (cur.valid) {
            const int off = cur.off, jc = cur.jc;
            bwd_mma_chunk<X, TT, TN>(lds + tok_rd + LS * L::TOK_STAGE, lds + wgt_rd + LS * L::WGT_STAGE, acc,
                                     [&](int ks, const u32x4 (&ft)[TT]) {
                // window rows of Wfull: output columns nc + 16 ks + k' feed latent column off + jk + k'
                int jk = jc + 16 * ks;
                if (jk >= p.d_h) jk -= p.d_h;
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    const int d = off + jk - (colm0 + 32 * ni);
                    if (d > -16 && d < 32) {   // uniform over the wave
                        const u32x4 f = shifted_identity_frag<X>(d, l31, lhi);
#pragma unroll
                        for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(f, ft[ti], acc[ni][ti]);
                    }
                }
            });
        }
        advance(cur);
        store_chunk(std::integral_constant<int, (S + 1) % D>{}, std::integral_constant<int, 1 - LS>{});
        __syncthreads();
    };

    // prologue: chunks 0 .. D - 1 into the register sets, chunk 0 on to LDS
    static_for<D>([&](auto r) {
        load_chunk(r, ld);
        advance(ld);
    });
    store_chunk(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    __syncthreads();
    constexpr int U = D % 2 == 0 ? D : 2 * D;     // iterations until register set and LDS stage repeat
    for (int it = 0; it < n_it; it += U)
        static_for<U>([&](auto i) {
            constexpr int I = decltype(i)::value;
            iteration(std::integral_constant<int, I % D>{}, std::integral_constant<int, I % 2>{});
        });
    bwd_reduce_halves<TT, TN>(smem, acc, half, w4, lane);
    if (half == 0) bwd_epilogue<X, OutT, TT, TN>(acc, rD, p.ldo, cols_left, wt, wn, l31, lhi);
}

// ---------------------------------------------------------------------------------------------
// Weight gradient.  Output tile: (64 TT) rows of C x (64 TN) columns.  Column operand ("tok") =
// latent columns Bbar(i) of c, row operand ("wgt") = columns of G.  The contraction index (token)
// is the slow index of both in memory, so both tiles are copied to LDS as they are -- one LDS row
// per token, coalesced on both sides -- and the fragments are read with the transposing LDS read
// (ds_read_b64_tr_b16): each lane names four consecutive columns of one token row and receives
// four consecutive tokens of one column.  Rows are not padded; the 16-byte pieces of a row are XOR-
// swizzled by the row number so that the four token rows one such read touches (64 bytes each) fall
// into different quarters of the 256-byte bank line, while a row's pieces stay within the row (the
// copies into LDS write whole rows).
// ---------------------------------------------------------------------------------------------
template <int TT, int TN>
struct BwdWeightLds {
    static constexpr int BT = 64 * TT, BN = 64 * TN;
    static constexpr int TOK_PITCH = BT * 2, WGT_PITCH = BN * 2;             // bytes per token row
    // piece p of row r sits at p ^ swz(r): 128-byte rows pair up in a bank line, so the pair number
    // picks the half; 256-byte rows fill one, so the row number picks the quarter
    static __device__ __forceinline__ int swz(int pitch, int r) { return pitch == 128 ? ((r >> 1) & 1) * 4 : (r & 3) * 4; }
    static constexpr int TOK_STAGE = 64 * TOK_PITCH, WGT_STAGE = 64 * WGT_PITCH;
    static constexpr int WGT_BASE = 2 * TOK_STAGE;
    static constexpr int HALF = 2 * (TOK_STAGE + WGT_STAGE);
    static constexpr int BYTES = 2 * HALF;
    static_assert(4 * TT * TN * 16 * 64 * 4 <= BYTES, "accumulator exchange must fit the staging memory");
};

template <typename X, typename OutT, int TT, int TN>
__global__ __launch_bounds__(512) void bwd_weight_kernel(const BwdArgs p)
{
    using L = BwdWeightLds<TT, TN>;
    constexpr int BT = L::BT, BN = L::BN;
    constexpr int TOK_PER_ROW = BT / 8, WGT_PER_ROW = BN / 8;       // 16-byte pieces per token row
    constexpr int TOK_LOADS = 64 * TOK_PER_ROW / 256, WGT_LOADS = 64 * WGT_PER_ROW / 256;
    constexpr int TOK_ROWS_PER_PASS = 256 / TOK_PER_ROW, WGT_ROWS_PER_PASS = 256 / WGT_PER_ROW;
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    typedef __attribute__((address_space(3))) unsigned char* lds_u8;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tile = bwd_tile_of_block(p.m_tiles * p.n_tiles);
    if (tile < 0) return;
    const int nt = tile / p.m_tiles, mt = tile % p.m_tiles;   // the row tiles of one column tile share its G columns

    const int tid = threadIdx.x & 255;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = wave >> 2, w4 = wave & 3;
    const int wt = w4 >> 1, wn = w4 & 1;
    const int l31 = lane & 31, lhi = lane >> 5;
    unsigned char* const lds = smem + half * L::HALF;

    int g = 0;
    while (g + 1 < p.n_groups && nt >= p.tile_start[g + 1]) ++g;
    const int64_t n0 = p.col_start[g] + (int64_t)(nt - p.tile_start[g]) * BN;
    const int cols_left = (int)((p.col_start[g + 1] - n0) > BN ? BN : (p.col_start[g + 1] - n0));
    const int i0 = mt * BT;
    const int rows_left = p.K - i0;
    const int a_off = p.a_off[g];
    const int64_t T = p.T;
    const char* const c_base = (const char*)p.c;
    const char* const g_base = (const char*)p.g + n0 * 2;
    const int64_t c_pitch = p.ldc * 2, g_pitch = p.ldg * 2;
    const int d_c_bytes = p.d_c * 2;

    const __amdgpu_buffer_rsrc_t rD = make_rsrc((char*)p.out + ((int64_t)i0 * p.ldo + n0) * (int64_t)sizeof(OutT),
                                                ((int64_t)(rows_left - 1) * p.ldo + cols_left) * (int64_t)sizeof(OutT));

    // this thread's pieces: tok piece (row tid / TOK_PER_ROW + pass * TOK_ROWS_PER_PASS, 16-byte piece
    // tid % TOK_PER_ROW), the same for wgt; offsets relative to the chunk's first token
    uint32_t tok_voff, wgt_voff, tok_lds, wgt_lds;
    {
        const int piece = tid % TOK_PER_ROW, row = tid / TOK_PER_ROW;
        const int ia = i0 + piece * 8;                              // row of C
        const int col = ia < a_off ? ia : ia + p.d_h;               // its latent column
        tok_voff = piece * 8 < rows_left ? (uint32_t)row * (uint32_t)c_pitch + (uint32_t)col * 2u : kBadOffset;
        tok_lds = (uint32_t)(row * L::TOK_PITCH + ((piece ^ L::swz(L::TOK_PITCH, row)) * 16));
    }
    {
        const int piece = tid % WGT_PER_ROW, row = tid / WGT_PER_ROW;
        wgt_voff = piece * 8 < cols_left ? (uint32_t)row * (uint32_t)g_pitch + (uint32_t)piece * 16u : kBadOffset;
        wgt_lds = (uint32_t)(row * L::WGT_PITCH + ((piece ^ L::swz(L::WGT_PITCH, row)) * 16));
    }
    const uint32_t tok_pass = (uint32_t)TOK_ROWS_PER_PASS * (uint32_t)c_pitch;
    const uint32_t wgt_pass = (uint32_t)WGT_ROWS_PER_PASS * (uint32_t)g_pitch;
    const int n_chunks = (int)((T + 63) >> 6);
    const int n_it = (n_chunks + 1) >> 1;

    constexpr int D = bwd_depth<TT, TN>();
    u32x4 tok_reg[D][TOK_LOADS], wgt_reg[D][WGT_LOADS];
    // Fetch state of this half: its chunks are 128 tokens apart.  The descriptors move along with a
    // running base and end with the chunk's last token, so token rows past T (and whole chunks past
    // the last one) read as zero.  Everything below is scalar and incremental.
    uint32_t tok_v[TOK_LOADS], wgt_v[WGT_LOADS];      // per-lane offsets inside a chunk (or kBadOffset)
#pragma unroll
    for (int i = 0; i < TOK_LOADS; ++i) tok_v[i] = tok_voff == kBadOffset ? kBadOffset : tok_voff + (uint32_t)i * tok_pass;
#pragma unroll
    for (int i = 0; i < WGT_LOADS; ++i) wgt_v[i] = wgt_voff == kBadOffset ? kBadOffset : wgt_voff + (uint32_t)i * wgt_pass;
    const int n_full = (int)(T >> 6), tail_rows = (int)(T & 63);
    const uint32_t c_full = 63u * (uint32_t)c_pitch + (uint32_t)d_c_bytes;
    const uint32_t c_tail = tail_rows ? (uint32_t)(tail_rows - 1) * (uint32_t)c_pitch + (uint32_t)d_c_bytes : 0u;
    const uint32_t g_full = 63u * (uint32_t)g_pitch + (uint32_t)cols_left * 2u;
    const uint32_t g_tail = tail_rows ? (uint32_t)(tail_rows - 1) * (uint32_t)g_pitch + (uint32_t)cols_left * 2u : 0u;
    const char* c_ptr = c_base + (int64_t)half * 64 * c_pitch;
    const char* g_ptr = g_base + (int64_t)half * 64 * g_pitch;
    const int64_t c_step = 128 * c_pitch, g_step = 128 * g_pitch;
    int ld_chunk = half;
    auto load_chunk = [&](auto set) {
        constexpr int S = decltype(set)::value;
        const bool full = ld_chunk < n_full, last = ld_chunk == n_full;
        const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(c_ptr), 0, (int)(full ? c_full : last ? c_tail : 0u), 0x00020000);
        const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char*>(g_ptr), 0, (int)(full ? g_full : last ? g_tail : 0u), 0x00020000);
#pragma unroll
        for (int i = 0; i < TOK_LOADS; ++i) tok_reg[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rA, tok_v[i], 0, 0);
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) wgt_reg[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rB, wgt_v[i], 0, 0);
        c_ptr += c_step;
        g_ptr += g_step;
        ld_chunk += 2;
    };
    auto store_chunk = [&](auto set, auto stage) {
        constexpr int S = decltype(set)::value, LS = decltype(stage)::value;
        unsigned char* tok_s = lds + LS * L::TOK_STAGE + tok_lds;
        unsigned char* wgt_s = lds + L::WGT_BASE + LS * L::WGT_STAGE + wgt_lds;
#pragma unroll
        for (int i = 0; i < TOK_LOADS; ++i) *(u32x4*)(tok_s + i * TOK_ROWS_PER_PASS * L::TOK_PITCH) = tok_reg[S][i];
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) *(u32x4*)(wgt_s + i * WGT_ROWS_PER_PASS * L::WGT_PITCH) = wgt_reg[S][i];
    };

    f32x16 acc[TN][TT];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int ti = 0; ti < TT; ++ti)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ni][ti][r] = 0.0f;

    // transposing reads: lane (16-lane group q = lane / 16, s = lane % 16) names token row
    // 8 (q / 2) + s / 4 (+ 16 ks, + 4 for the upper half of the fragment) and columns
    // 16 (q % 2) + 4 (s % 4) .. + 3 of an MFMA tile's 32; it receives tokens 8 lhi .. 8 lhi + 7 of
    // column l31 -- the MFMA operand layout
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8)lds;
    const int c_s = lane & 15, c_q = lane >> 4;
    const int fr_row = 8 * (c_q >> 1) + (c_s >> 2), fr_col = 16 * (c_q & 1) + 4 * (c_s & 3);
    // (the rows a lane reads differ by multiples of 4, and the passes of a copy by 16 or 32 rows, so
    // the swizzle is a constant of the lane on both sides)
    uint32_t a_tok[TT], a_wgt[TN];
#pragma unroll
    for (int ti = 0; ti < TT; ++ti) {
        const int cb = (wt * (32 * TT) + 32 * ti + fr_col) * 2;
        a_tok[ti] = lds0 + (uint32_t)(fr_row * L::TOK_PITCH + (((cb >> 4) ^ L::swz(L::TOK_PITCH, fr_row)) << 4) + (cb & 15));
    }
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
        const int cb = (wn * (32 * TN) + 32 * ni + fr_col) * 2;
        a_wgt[ni] = lds0 + (uint32_t)(L::WGT_BASE + fr_row * L::WGT_PITCH + (((cb >> 4) ^ L::swz(L::WGT_PITCH, fr_row)) << 4) + (cb & 15));
    }
    auto frag = [&](uint32_t addr, int pitch) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(uintptr_t)addr);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(uintptr_t)(addr + 4 * pitch));
        const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
        return (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
    };

    auto iteration = [&](auto set, auto stage, int it) {
        constexpr int S = decltype(set)::value, LS = decltype(stage)::value;
        load_chunk(set);
        if (2 * it + half < n_chunks) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4 fw[TN], ft[TT];
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    fw[ni] = frag(a_wgt[ni] + LS * L::WGT_STAGE + 16 * ks * L::WGT_PITCH, L::WGT_PITCH);
#pragma unroll
                for (int ti = 0; ti < TT; ++ti)
                    ft[ti] = frag(a_tok[ti] + LS * L::TOK_STAGE + 16 * ks * L::TOK_PITCH, L::TOK_PITCH);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                    for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(fw[ni], ft[ti], acc[ni][ti]);
            }
        }
        store_chunk(std::integral_constant<int, (S + 1) % D>{}, std::integral_constant<int, 1 - LS>{});
        __syncthreads();
    };

    static_for<D>([&](auto r) { load_chunk(r); });
    store_chunk(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    __syncthreads();
    constexpr int U = D % 2 == 0 ? D : 2 * D;     // iterations until register set and LDS stage repeat
    for (int it = 0; it < n_it; it += U)
        static_for<U>([&](auto i) {
            constexpr int I = decltype(i)::value;
            iteration(std::integral_constant<int, I % D>{}, std::integral_constant<int, I % 2>{}, it + I);
        });
    bwd_reduce_halves<TT, TN>(smem, acc, half, w4, lane);
    if (half == 0) bwd_epilogue<X, OutT, TT, TN>(acc, rD, p.ldo, cols_left, wt, wn, l31, lhi);
}

// ---------------------------------------------------------------------------------------------
// General kernels: any element type, shape or alignment.  64 x 64 output tile per workgroup of 256
// threads (4 x 4 outputs each), contraction in steps of 16, scalar guarded loads, float32 FMAs.
// ---------------------------------------------------------------------------------------------
template <typename InT, typename OutT>
__global__ __launch_bounds__(256) void bwd_latent_general_kernel(const BwdArgs p)
{
    __shared__ float Gs[16][64 + 1];
    __shared__ float Ws[16][64 + 1];
    const InT* __restrict__ Gg = (const InT*)p.g;
    const InT* __restrict__ Cg = (const InT*)p.C;
    OutT* __restrict__ Dg = (OutT*)p.out;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int l0 = blockIdx.x * 64;
    const int64_t t0 = (int64_t)blockIdx.y * 64;
    const int64_t N = p.col_start[p.n_groups];

    float acc[4][4] = {};
    for (int64_t n0 = 0; n0 < N; n0 += 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            {
                const int kk = idx & 15, r = idx >> 4;
                const int64_t n = n0 + kk, t = t0 + r;
                Gs[kk][r] = (n < N && t < p.T) ? load_as_f32(Gg + t * p.ldg + n) : 0.0f;
            }
            {
                const int kk = idx & 15, r = idx >> 4;     // r: latent column of the tile
                const int64_t n = n0 + kk;
                const int l = l0 + r;
                float v = 0.0f;
                if (n < N && l < p.d_c) {
                    int g = 0;
                    while (g + 1 < p.n_groups && n >= p.col_start[g + 1]) ++g;
                    const int off = p.a_off[g];
                    if (l >= off && l < off + p.d_h) v = (l - off == (int)((n - p.col_start[g]) % p.d_h)) ? 1.0f : 0.0f;
                    else v = load_as_f32(Cg + (int64_t)(l < off ? l : l - p.d_h) * p.ldC + n);
                }
                Ws[kk][r] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Gs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t t = t0 + ty * 4 + i;
            const int l = l0 + tx * 4 + j;
            if (t < p.T && l < p.d_c) store_from_f32(Dg + t * p.ldo + l, acc[i][j]);
        }
}

template <typename InT, typename OutT>
__global__ __launch_bounds__(256) void bwd_weight_general_kernel(const BwdArgs p)
{
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const InT* __restrict__ Cg = (const InT*)p.c;
    const InT* __restrict__ Gg = (const InT*)p.g;
    OutT* __restrict__ Dg = (OutT*)p.out;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    // column tiles are laid out per group so that a tile never straddles two basis windows
    const int nt = blockIdx.x;
    int g = 0;
    while (g + 1 < p.n_groups && nt >= p.tile_start[g + 1]) ++g;
    const int64_t n0 = p.col_start[g] + (int64_t)(nt - p.tile_start[g]) * 64;
    const int64_t n_end = p.col_start[g + 1];
    const int i0 = blockIdx.y * 64;
    const int a_off = p.a_off[g];

    float acc[4][4] = {};
    for (int64_t t0 = 0; t0 < p.T; t0 += 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            const int r = idx & 63, kk = idx >> 6;
            const int64_t t = t0 + kk;
            {
                const int i = i0 + r;
                As[kk][r] = (t < p.T && i < p.K) ? load_as_f32(Cg + t * p.ldc + (i < a_off ? i : i + p.d_h)) : 0.0f;
            }
            {
                const int64_t n = n0 + r;
                Bs[kk][r] = (t < p.T && n < n_end) ? load_as_f32(Gg + t * p.ldg + n) : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = i0 + ty * 4 + i;
            const int64_t n = n0 + tx * 4 + j;
            if (r < p.K && n < n_end) store_from_f32(Dg + (int64_t)r * p.ldo + n, acc[i][j]);
        }
}

}  // namespace bda
