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
// both tiles are transposed in registers (8 x 8 blocks of 16-bit values) on their way to LDS.
//
// Same skeleton as gemm_mfma_kernel: 256 threads = 2 x 2 waves, each wave owns TT x TN MFMA tiles
// of 32 x 32 (v_mfma_f32_32x32x16), contraction in chunks of 64 through a double-buffered LDS tile,
// the next chunk's global loads in flight during the MFMAs; the operand whose index is contiguous
// in the OUTPUT is the MFMA's row operand, so that each lane stores four consecutive elements.
#pragma once
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
                    v[0] = (uint32_t)X::from_f32(acc[ni][ti][rg * 4 + 0]) |
                           ((uint32_t)X::from_f32(acc[ni][ti][rg * 4 + 1]) << 16);
                    v[1] = (uint32_t)X::from_f32(acc[ni][ti][rg * 4 + 2]) |
                           ((uint32_t)X::from_f32(acc[ni][ti][rg * 4 + 3]) << 16);
                    __builtin_amdgcn_raw_buffer_store_b64(v, rD, off, 0, 0);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Latent gradient.  Output tile: (64 TT) tokens x (64 TN) latent columns.  Column operand ("tok")
// = G rows, row operand ("wgt") = rows of Wfull, one per latent column of the tile.
// ---------------------------------------------------------------------------------------------
template <typename X, typename OutT, int TT, int TN>
__global__ __launch_bounds__(256) void bwd_latent_kernel(const BwdArgs p)
{
    constexpr int BT = 64 * TT, BN = 64 * TN;
    constexpr int TOK_STAGE = BT * kRowBytes, WGT_STAGE = BN * kRowBytes;
    constexpr int WGT_BASE = 2 * TOK_STAGE;
    constexpr int TOK_LOADS = BT / 32, WGT_LOADS = BN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tile = bwd_tile_of_block(p.m_tiles * p.n_tiles);
    if (tile < 0) return;
    const int mt = tile / p.n_tiles, nt = tile % p.n_tiles;   // the column tiles of one token tile share its G rows

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lhi = lane >> 5;
    const int tq = tid & 7, trow = tid >> 3;

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

    u32x4 tok_reg[TOK_LOADS], wgt_reg[WGT_LOADS];

    // chunk cursor: (group, first column); chunks never straddle groups
    auto advance = [&](int& g, int64_t& nc) {
        nc += 64;
        if (nc >= p.col_start[g + 1]) {
            ++g;
            nc = p.col_start[g < p.n_groups ? g : p.n_groups];
        }
    };
    auto load_chunk = [&](int g, int64_t nc) {
        const int64_t col = nc + tq * 8;
        const bool col_ok = col < p.col_start[g + 1];
        const uint32_t col_bytes = (uint32_t)col * 2u;
#pragma unroll
        for (int i = 0; i < TOK_LOADS; ++i) {
            const uint32_t voff = col_ok ? (uint32_t)(trow + 32 * i) * g_row_bytes + col_bytes : kBadOffset;
            tok_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(rG, voff, 0, 0);
        }
        const int off = p.a_off[g];
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) {
            const int l = l0 + trow + 32 * i;                                 // latent column of this LDS row
            const int row = l < off ? l : l - p.d_h;                          // its row of C
            const bool ok = col_ok && l < p.d_c && (l < off || l >= off + p.d_h);
            wgt_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(rC, ok ? (uint32_t)row * c_row_bytes + col_bytes : kBadOffset, 0, 0);
        }
    };
    auto store_chunk = [&](int stage) {
        unsigned char* tok_s = smem + stage * TOK_STAGE;
        unsigned char* wgt_s = smem + WGT_BASE + stage * WGT_STAGE;
#pragma unroll
        for (int i = 0; i < TOK_LOADS; ++i) *(u32x4*)(tok_s + lds_off(trow + 32 * i, tq)) = tok_reg[i];
#pragma unroll
        for (int i = 0; i < WGT_LOADS; ++i) *(u32x4*)(wgt_s + lds_off(trow + 32 * i, tq)) = wgt_reg[i];
    };

    f32x16 acc[TN][TT];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int ti = 0; ti < TT; ++ti)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ni][ti][r] = 0.0f;

    int n_chunks = 0;
    for (int g = 0; g < p.n_groups; ++g) n_chunks += (int)((p.col_start[g + 1] - p.col_start[g] + 63) >> 6);

    const int tok_rd = (wt * (32 * TT) + l31) * kRowBytes + lhi * 16;
    const int wgt_rd = WGT_BASE + (wn * (32 * TN) + l31) * kRowBytes + lhi * 16;
    const int colm0 = l0 + wn * (32 * TN);           // first latent column of this wave's MFMA tiles

    int g_cur = 0, g_nxt = 0;
    int64_t nc_cur = 0, nc_nxt = 0;
    load_chunk(0, 0);
    store_chunk(0);
    advance(g_nxt, nc_nxt);
    __syncthreads();
    for (int kc = 0; kc < n_chunks; ++kc) {
        const bool more = kc + 1 < n_chunks;
        if (more) load_chunk(g_nxt, nc_nxt);
        const unsigned char* tok_s = smem + tok_rd + (kc & 1) * TOK_STAGE;
        const unsigned char* wgt_s = smem + wgt_rd + (kc & 1) * WGT_STAGE;
        const int off = p.a_off[g_cur];
        const int jc = (int)((nc_cur - p.col_start[g_cur]) % p.d_h);   // window column of the chunk's first output column
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
        }
        if (more) store_chunk((kc + 1) & 1);
        g_cur = g_nxt;
        nc_cur = nc_nxt;
        if (more) advance(g_nxt, nc_nxt);
        __syncthreads();
    }
    bwd_epilogue<X, OutT, TT, TN>(acc, rD, p.ldo, cols_left, wt, wn, l31, lhi);
}

// ---------------------------------------------------------------------------------------------
// Weight gradient.  Output tile: (64 TT) rows of C x (64 TN) columns.  Column operand ("tok") =
// latent columns Bbar(i) of c, row operand ("wgt") = columns of G; both are read as 8 (tokens) x 8
// blocks and transposed in registers.
// ---------------------------------------------------------------------------------------------
template <typename X, typename OutT, int TT, int TN>
__global__ __launch_bounds__(256) void bwd_weight_kernel(const BwdArgs p)
{
    constexpr int BT = 64 * TT, BN = 64 * TN;
    constexpr int TOK_STAGE = BT * kRowBytes, WGT_STAGE = BN * kRowBytes;
    constexpr int WGT_BASE = 2 * TOK_STAGE;
    constexpr int TOK_BLOCKS = (BT + 255) / 256, WGT_BLOCKS = (BN + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tile = bwd_tile_of_block(p.m_tiles * p.n_tiles);
    if (tile < 0) return;
    const int nt = tile / p.m_tiles, mt = tile % p.m_tiles;   // the row tiles of one column tile share its G columns

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lhi = lane >> 5;
    // small tiles: the two operands are fetched by different halves of the workgroup
    const int tid_w = (BT <= 128 && BN <= 128) ? (tid ^ 128) : tid;
    const int kq_t = tid & 7, blk_t = tid >> 3;       // "tok": 8-token block within the chunk, 8-row block of the tile
    const int kq_w = tid_w & 7, blk_w = tid_w >> 3;

    int g = 0;
    while (g + 1 < p.n_groups && nt >= p.tile_start[g + 1]) ++g;
    const int64_t n0 = p.col_start[g] + (int64_t)(nt - p.tile_start[g]) * BN;
    const int cols_left = (int)((p.col_start[g + 1] - n0) > BN ? BN : (p.col_start[g + 1] - n0));
    const int i0 = mt * BT;
    const int rows_left = p.K - i0;
    const int a_off = p.a_off[g];

    const __amdgpu_buffer_rsrc_t rD = make_rsrc((char*)p.out + ((int64_t)i0 * p.ldo + n0) * (int64_t)sizeof(OutT),
                                                ((int64_t)(rows_left - 1) * p.ldo + cols_left) * (int64_t)sizeof(OutT));
    const uint32_t c_row_bytes = (uint32_t)(p.ldc * 2), g_row_bytes = (uint32_t)(p.ldg * 2);

    // block offsets inside a chunk of 64 tokens (the chunk's first token is the descriptor's base)
    uint32_t tok_voff[TOK_BLOCKS], wgt_voff[WGT_BLOCKS];
#pragma unroll
    for (int b = 0; b < TOK_BLOCKS; ++b) {
        const int i = (blk_t + 32 * b) * 8;                       // row of C, relative to the tile
        const int ia = i0 + i;
        const int col = ia < a_off ? ia : ia + p.d_h;             // its latent column
        tok_voff[b] = (i < BT && i < rows_left) ? (uint32_t)(kq_t * 8) * c_row_bytes + (uint32_t)col * 2u : kBadOffset;
    }
#pragma unroll
    for (int b = 0; b < WGT_BLOCKS; ++b) {
        const int n = (blk_w + 32 * b) * 8;
        wgt_voff[b] = (n < BN && n < cols_left) ? (uint32_t)(kq_w * 8) * g_row_bytes + (uint32_t)n * 2u : kBadOffset;
    }

    u32x4 tok_reg[TOK_BLOCKS][8], wgt_reg[WGT_BLOCKS][8];
    auto load_chunk = [&](int kc) {
        // descriptors end with the last token, so token rows past T read as zero
        const int64_t t = (int64_t)kc * 64;
        const int64_t rows = p.T - t > 64 ? 64 : p.T - t;
        const __amdgpu_buffer_rsrc_t rA = make_rsrc((const char*)p.c + t * p.ldc * 2, ((rows - 1) * p.ldc + p.d_c) * 2);
        const __amdgpu_buffer_rsrc_t rB = make_rsrc((const char*)p.g + (t * p.ldg + n0) * 2, ((rows - 1) * p.ldg + cols_left) * 2);
#pragma unroll
        for (int b = 0; b < TOK_BLOCKS; ++b)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                tok_reg[b][e] = __builtin_amdgcn_raw_buffer_load_b128(rA, tok_voff[b] == kBadOffset ? kBadOffset : tok_voff[b] + (uint32_t)e * c_row_bytes, 0, 0);
#pragma unroll
        for (int b = 0; b < WGT_BLOCKS; ++b)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                wgt_reg[b][e] = __builtin_amdgcn_raw_buffer_load_b128(rB, wgt_voff[b] == kBadOffset ? kBadOffset : wgt_voff[b] + (uint32_t)e * g_row_bytes, 0, 0);
    };
    auto store_chunk = [&](int stage) {
        unsigned char* tok_s = smem + stage * TOK_STAGE;
        unsigned char* wgt_s = smem + WGT_BASE + stage * WGT_STAGE;
#pragma unroll
        for (int b = 0; b < TOK_BLOCKS; ++b) {
            const int r = (blk_t + 32 * b) * 8;
            if (r < BT) {
                u32x4 tr[8];
                transpose8x8_b16(tok_reg[b], tr);
#pragma unroll
                for (int j = 0; j < 8; ++j) *(u32x4*)(tok_s + lds_off(r + j, kq_t)) = tr[j];
            }
        }
#pragma unroll
        for (int b = 0; b < WGT_BLOCKS; ++b) {
            const int r = (blk_w + 32 * b) * 8;
            if (r < BN) {
                u32x4 tr[8];
                transpose8x8_b16(wgt_reg[b], tr);
#pragma unroll
                for (int j = 0; j < 8; ++j) *(u32x4*)(wgt_s + lds_off(r + j, kq_w)) = tr[j];
            }
        }
    };

    f32x16 acc[TN][TT];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int ti = 0; ti < TT; ++ti)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ni][ti][r] = 0.0f;

    const int n_chunks = (int)((p.T + 63) >> 6);
    const int tok_rd = (wt * (32 * TT) + l31) * kRowBytes + lhi * 16;
    const int wgt_rd = WGT_BASE + (wn * (32 * TN) + l31) * kRowBytes + lhi * 16;
    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int kc = 0; kc < n_chunks; ++kc) {
        const bool more = kc + 1 < n_chunks;
        if (more) load_chunk(kc + 1);
        const unsigned char* tok_s = smem + tok_rd + (kc & 1) * TOK_STAGE;
        const unsigned char* wgt_s = smem + wgt_rd + (kc & 1) * WGT_STAGE;
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
        }
        if (more) store_chunk((kc + 1) & 1);
        __syncthreads();
    }
    bwd_epilogue<X, OutT, TT, TN>(acc, rD, p.ldo, cols_left, wt, wn, l31, lhi);
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
