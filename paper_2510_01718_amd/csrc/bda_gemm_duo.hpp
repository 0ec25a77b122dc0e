// Two-workgroups-per-compute-unit streaming MFMA GEMM for gfx950: the large-T kernel of libbda for
// launches with many 128 x 256 tiles per compute unit.
//
//   D[t, n] = ident(t, n) + sum_{k < K} A[t, acol_g(k)] * B[k, n]        (see bda_gemm_kernels.hpp)
//
// Same LDS images, swizzles, identity-slice-as-MFMA and rounding as the lean streaming kernel
// (bda_gemm_plain.hpp, whose preconditions it shares; identity slices for head widths 64 and 128).
// What differs is how the compute unit is shared:
//
//   * A workgroup is four waves (one per SIMD) and takes 128 tokens x 256 columns; each wave owns all
//     128 tokens of 64 columns (the 128 accumulator registers of the lean kernel's waves).  It needs
//     80 KiB of LDS and at most 256 registers per lane, so two workgroups share a compute unit.  Each
//     SIMD then holds two waves that belong to different workgroups: they share no barrier, so while
//     one workgroup converts and stores a finished tile, waits at its stage barrier or waits for a
//     late load, the other keeps the MFMA pipes busy.  (In the lean kernel both waves of a SIMD sit
//     in the same workgroup: its barriers, its load waits and its result stores stop the whole
//     compute unit.)
//   * Stages of 32 along the contraction (8 KiB of token rows + 16 KiB of weight rows) in a ring of
//     three slots; the loads of stage g + 2 are requested when stage g starts, so a load has two
//     stage times to land.  One barrier per stage, between its two k-steps: it tells that stage
//     g + 1 has landed in every wave's part of the slot and that slot g is free for stage g + 3.
//     Every wave requests six loads per stage (two token pieces, four weight pieces), also where a
//     stage has less to fetch (identity stages, stages past the last tile): the vmcnt arithmetic
//     stays the same everywhere.
//   * Identity slice: two more stages per tile.  Stage s holds window columns [32 s, 32 s + 32) in
//     its token part and, for 128-wide heads, [64 + 32 s, ...) in the first half of its weight part;
//     a wave multiplies the piece that belongs to its 64 columns by a constant identity fragment
//     into its s-th 32-column block.
//   * Results leave through a 2 KiB staging tile per wave (one 32 x 32 block at a time), so that
//     four lanes store one 64-byte segment of a row.  The stores stay in flight while the next
//     tile's first stage runs.
//   * Tile order: the eight dies split the tile grid into dn column ranges x dm token ranges
//     (dn dm = 8); a die's 64 workgroups walk its range token tile by token tile, so its L2 keeps
//     its column range of the weights (3 MiB for the V3 shape) and streams the latent once.
#pragma once
#include <type_traits>

#include "bda_gemm_plain.hpp"

namespace bda {

struct DuoArgs {
    const void* A;
    const void* B;
    void* D;
    int64_t lda, ldb, ldd;           // in elements
    int64_t M;                       // tokens
    int K;                           // contraction length (a multiple of 32, at least 64)
    int n_groups;
    int d_h, a_skip;                 // as in GemmArgs (d_h: 64 or 128 when there is an identity slice)
    int rounds;                      // tiles every workgroup walks through (some may lie outside its die's range)
    int die_c0[kNumXcd], die_cx[kNumXcd];   // column-tile range of die x: [c0, c0 + cx)
    int die_m0[kNumXcd], die_mx[kNumXcd];   // token-tile range of die x
    uint64_t die_magic[kNumXcd];     // ceil(2^40 / max(cx, 1))
    int tile_start[kMaxGroups + 1];
    int64_t col_start[kMaxGroups + 1];
    int a_off[kMaxGroups];
};

constexpr int kDuoThreads = 256;
constexpr int kDuoSlotsPerXcd = 64;                      // workgroups per die: two per compute unit
constexpr int kDuoTokBytes = 128 * 64;                   // 128 tokens x 32 k
constexpr int kDuoStageBytes = kDuoTokBytes + 32 * 512;  // + 32 k x 256 columns
constexpr int kDuoSlots = 3;
constexpr int kDuoStaging = kDuoSlots * kDuoStageBytes;  // 4 waves x 2 KiB
constexpr int kDuoLdsBytes = kDuoStaging + 4 * 2048;     // 80 KiB: half of a compute unit's LDS

// lane number, recomputed where it is needed so that it does not occupy a register in between
__device__ __forceinline__ int duo_lane_id()
{
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

// IDENT: the launch has an identity slice (then d_h is 64 or 128 and every tile has two identity
// stages).  Compile-time, so that no accumulator crosses a branch or a loop that depends on it.
template <typename X, typename OutT, bool IDENT>
__global__ __launch_bounds__(kDuoThreads, 2) void gemm_duo_kernel(const DuoArgs p)
{
    constexpr int SK = 32, BT = 128, BN = 256, TT = 4, TN = 2, NS = kDuoSlots;
    constexpr int RB = SK * 2;                         // bytes per token row in LDS
    constexpr int TOK_BYTES = kDuoTokBytes;
    constexpr int STAGE_BYTES = kDuoStageBytes;
    constexpr int n_id = IDENT ? 2 : 0;
    constexpr int LOADS = 6;                           // per wave and stage
    constexpr int STORES = TT * TN * (sizeof(OutT) == 4 ? 4 : 2);   // per wave and tile
    static_assert(LOADS + STORES < 64, "vmcnt is six bits");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) unsigned char* lds_u8;
    typedef __attribute__((address_space(3))) const u32x4* lds_u32x4;
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // = the wave's 64-column block of the tile
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8)smem;

    const int xcd = blockIdx.x % kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    // The scalar kernel arguments are fetched here in one batch and made opaque, so that they live in
    // registers: otherwise each use inside the loops re-fetches its argument from memory (a scalar
    // load and a wait of a few hundred cycles each, and the wait also drains the LDS reads in flight).
    struct {
        const void *A, *B; void* D;
        int64_t lda, ldb, ldd, M, cs1;
        uint64_t cmagic;
        int K, n_groups, d_h, a_skip, rounds, c0, cx, m0, mx, ts1, aoff0, aoff1;
    } q = {p.A, p.B, p.D, p.lda, p.ldb, p.ldd, p.M, p.col_start[1], p.die_magic[xcd],
           p.K, p.n_groups, p.d_h, p.a_skip, p.rounds, p.die_c0[xcd], p.die_cx[xcd], p.die_m0[xcd], p.die_mx[xcd],
           p.tile_start[1], p.a_off[0], p.a_off[1]};
    asm volatile("" : "+s"(q.A), "+s"(q.B), "+s"(q.D), "+s"(q.lda), "+s"(q.ldb), "+s"(q.ldd), "+s"(q.M), "+s"(q.cs1), "+s"(q.cmagic));
    asm volatile("" : "+s"(q.K), "+s"(q.n_groups), "+s"(q.d_h), "+s"(q.a_skip), "+s"(q.rounds), "+s"(q.c0), "+s"(q.cx), "+s"(q.m0),
                 "+s"(q.mx), "+s"(q.ts1), "+s"(q.aoff0), "+s"(q.aoff1));
    const int nk = q.K / SK;
    const int S = nk + n_id;
    const int rounds = q.rounds;
    const int die_tiles = q.cx * q.mx;

    // tile `r` of this workgroup: the die's tiles are numbered token tile by token tile across its
    // column range, and the workgroup takes numbers slot, slot + 64, ...
    // (the first two groups' tables are in registers; launches with more groups read the rest from the arguments)
    struct Tile { bool valid; int mt, ct, a_off; int64_t n0; };
    auto tile_of = [&](int r) -> Tile {
        Tile t;
        const int u = slot + kDuoSlotsPerXcd * r;
        t.valid = r < rounds && u < die_tiles;
        const int qt = t.valid ? (int)(((uint64_t)(uint32_t)u * q.cmagic) >> 40) : 0;
        t.mt = q.m0 + qt;
        t.ct = q.c0 + (t.valid ? u - qt * q.cx : 0);
        int g = (q.n_groups >= 2 && t.ct >= q.ts1) ? 1 : 0;
        int g_tile0 = g ? q.ts1 : 0;
        int64_t g_col0 = g ? q.cs1 : 0;
        t.a_off = g ? q.aoff1 : q.aoff0;
        if (q.n_groups > 2 && g == 1) {
            while (g + 1 < q.n_groups && t.ct >= p.tile_start[g + 1]) ++g;
            g_tile0 = p.tile_start[g];
            g_col0 = p.col_start[g];
            t.a_off = p.a_off[g];
        }
        t.n0 = g_col0 + (int64_t)(t.ct - g_tile0) * BN;
        return t;
    };

    // ---- loads: the stage after next, six DMA loads per wave -------------------------------------------
    const uint32_t tok_row_bytes = (uint32_t)(q.lda * 2), wgt_row_bytes = (uint32_t)(q.ldb * 2);
    // token load j (0, 1): LDS rows 32 wave + 16 j + lane / 4, position lane % 4 <- piece (lane % 4) ^ swizzle(row)
    const int l_piece = (lane & 3) ^ tok_swz<SK>((lane >> 2) & 15);
    const uint32_t tok_v = (uint32_t)(32 * wave + (lane >> 2)) * tok_row_bytes + (uint32_t)l_piece * 16u;
    const uint32_t tok_step = 16u * tok_row_bytes;
    // weight load i (0 .. 3): LDS k row 8 wave + 2 i + lane / 32, position lane % 32 <- piece (lane % 32) ^ swizzle(k)
    const uint32_t wgtE = (uint32_t)(8 * wave + (lane >> 5)) * wgt_row_bytes + (uint32_t)((lane & 31) ^ wgt_swz(lane >> 5)) * 16u;
    const uint32_t wgtO = (uint32_t)(8 * wave + 2 + (lane >> 5)) * wgt_row_bytes + (uint32_t)((lane & 31) ^ wgt_swz(2 + (lane >> 5))) * 16u;
    const uint32_t wgt_step = 4u * wgt_row_bytes;
    const uint32_t skip_bytes = (uint32_t)q.a_skip * 2u;
    const bool wide_heads = q.d_h > 64;
    const uint32_t tok_lds_w = (uint32_t)wave * 2048u;                       // this wave's part of a slot's token rows
    const uint32_t wgt_lds_w = (uint32_t)TOK_BYTES + (uint32_t)wave * 4096u;  // ... and of its weight rows

    int lr = 0, lk = 0;                                // tile and stage of the next stage to request
    uint32_t l_slot = lds0;                            // ... and its slot
    u32x4 rA, rB, rNone;
    int l_aoff = 0;
    auto load_tile = [&]() {
        const Tile t = tile_of(lr);
        const int64_t t0 = (int64_t)t.mt * BT;
        const int64_t rows_left = t.valid ? q.M - t0 : 0;
        l_aoff = t.a_off;
        rA = make_rsrc_words((const char*)q.A + (t.valid ? t0 : 0) * q.lda * 2,
                             rows_left > 0 ? ((rows_left - 1) * q.lda + q.K + q.a_skip) * 2 : 0);
        rB = make_rsrc_words((const char*)q.B + (t.valid ? t.n0 : 0) * 2,
                             t.valid ? ((int64_t)(q.K - 1) * q.ldb + BN) * 2 : 0);
        rNone = rA;
        rNone[2] = 0;                                  // nothing to fetch: every lane out of range, zeros land
    };
    auto request_stage = [&]() {
        if (lk < nk) {
            const int k0 = lk * SK;
            const uint32_t ts = __builtin_amdgcn_readfirstlane((uint32_t)(k0 + (k0 >= l_aoff ? q.a_skip : 0)) * 2u);
            uint32_t v = tok_v;
            const int e = l_aoff & (SK - 1);
            if (e != 0 && lk == l_aoff / SK && l_piece * 8 >= e) v += skip_bytes;   // the stage that holds the window's start: later pieces skip the window
            lds_dma1s(rA, l_slot + tok_lds_w, v, ts);
            lds_dma1s(rA, l_slot + tok_lds_w + 1024u, v + tok_step, ts);
            const uint32_t ws = __builtin_amdgcn_readfirstlane((uint32_t)k0 * wgt_row_bytes);
            lds_dma1s(rB, l_slot + wgt_lds_w, wgtE, ws);
            lds_dma1s(rB, l_slot + wgt_lds_w + 1024u, wgtO, ws);
            lds_dma1s(rB, l_slot + wgt_lds_w + 2048u, wgtE + wgt_step, ws);
            lds_dma1s(rB, l_slot + wgt_lds_w + 3072u, wgtO + wgt_step, ws);
        } else {
            // identity stage s = lk - nk: window columns [32 s, 32 s + 32) as token rows in the token part (for
            // the waves whose 64 columns start a head) and [64 + 32 s, ...) in the first half of the weight part
            // (for those that start in the middle of a 128-wide head); two loads that fetch nothing keep the count
            const int sidx = lk - nk;
            const uint32_t sa = __builtin_amdgcn_readfirstlane((uint32_t)(l_aoff + 32 * sidx) * 2u);
            const uint32_t sb = sa + 128u;
            const u32x4 rW = wide_heads ? rA : rNone;
            lds_dma1s(rA, l_slot + tok_lds_w, tok_v, sa);
            lds_dma1s(rA, l_slot + tok_lds_w + 1024u, tok_v + tok_step, sa);
            lds_dma1s(rW, l_slot + (uint32_t)TOK_BYTES + tok_lds_w, tok_v, sb);
            lds_dma1s(rW, l_slot + (uint32_t)TOK_BYTES + tok_lds_w + 1024u, tok_v + tok_step, sb);
            lds_dma1s(rNone, l_slot + (uint32_t)(2 * TOK_BYTES) + tok_lds_w, tok_v, 0u);
            lds_dma1s(rNone, l_slot + (uint32_t)(2 * TOK_BYTES) + tok_lds_w + 1024u, tok_v, 0u);
        }
        l_slot = (l_slot == lds0 + (uint32_t)((NS - 1) * STAGE_BYTES)) ? lds0 : l_slot + (uint32_t)STAGE_BYTES;
        if (++lk == S) {
            lk = 0;
            ++lr;
            load_tile();                               // (past the last tile: descriptors that fetch nothing)
        }
    };

    // ---- fragments ----------------------------------------------------------------------------------
    const int l31 = lane & 31, lhi = lane >> 5;
    f32x16 acc[TN][TT];
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    u32x4 fw0[TN], ft0[TT], fw1[TN], ft1[TT];
    auto clear_acc = [&]() {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = zero16;
    };
    // LDS addresses of this lane's fragments in the slot being read (absolute addresses)
    uint32_t a_tok = lds0 + (uint32_t)(l31 * RB + ((lhi ^ tok_swz<SK>(l31 & 15)) << 4));
    uint32_t a_wgt[TN];
    {
        const int c_s = lane & 15, c_gq = lane >> 4;
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const int col = wave * (32 * TN) + ni * 32 + 16 * (c_gq & 1) + 4 * (c_s & 3);
            const int pc = (col >> 3) ^ wgt_swz(c_s >> 2);
            a_wgt[ni] = lds0 + (uint32_t)(TOK_BYTES + (8 * lhi + (c_s >> 2)) * 512 + (pc << 4) + ((col & 4) << 1));
        }
    }
    int c_slot = 0;                                    // slot the fragment addresses point into
    auto next_slot = [&]() {
        const uint32_t d = c_slot == NS - 1 ? 0u - (uint32_t)((NS - 1) * STAGE_BYTES) : (uint32_t)STAGE_BYTES;
        c_slot = c_slot == NS - 1 ? 0 : c_slot + 1;
        a_tok += d;
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) a_wgt[ni] += d;
    };
    auto read_w = [&](int ks, u32x4 (&fw)[TN]) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(uintptr_t)(a_wgt[ni] + (16 * ks) * 512));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(uintptr_t)(a_wgt[ni] + (16 * ks + 4) * 512));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            fw[ni] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
        }
    };
    auto read_t = [&](int ks, u32x4 (&ft)[TT], uint32_t part_off) {
        const uint32_t a = (a_tok ^ (uint32_t)(ks << 5)) + part_off;
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) ft[ti] = *(lds_u32x4)(uintptr_t)(a + ti * (32 * RB));
    };
    // identity fragments (row operand): lane (row i = l31, half lhi) holds k' = 16 v + 8 lhi + e
    auto make_idf = [&](u32x4 (&idf)[2]) {
        const int ln = duo_lane_id();
        const int r31 = ln & 31, rhi = ln >> 5;
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int k0 = 16 * v + 8 * rhi + 2 * w;
                idf[v][w] = (k0 == r31 ? IdentityFrag<X>::one : 0u) | (k0 + 1 == r31 ? IdentityFrag<X>::one << 16 : 0u);
            }
    };

    // What follows a stage: a regular stage (weights and tokens to read) or an identity stage (one
    // piece of token rows).
    enum Next { NEXT_REGULAR = 0, NEXT_IDENTITY = 1 };
    // the stage's barrier: the next stage has landed (this wave's loads of it: everything older than
    // the newest LOADS, and than the result stores where those are the newest), in every wave
    auto stage_barrier = [&](bool relaxed) {
        if (relaxed) wait_vmcnt<LOADS + STORES>(); else wait_vmcnt<LOADS>();
        __syncthreads();
    };

    // One regular stage (two k-steps of 16).  On entry fw0 / ft0 hold the fragments of its first k-step.
    auto stage_regular = [&](auto next_c, bool relaxed, uint32_t next_part) {
        constexpr int next = decltype(next_c)::value;
        request_stage();
        read_w(1, fw1);
        read_t(1, ft1, 0u);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(fw0[ni], ft0[ti], acc[ni][ti]);
        stage_barrier(relaxed);
        next_slot();
        if constexpr (next == NEXT_REGULAR) read_w(0, fw0);
        read_t(0, ft0, next_part);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(fw1[ni], ft1[ti], acc[ni][ti]);
    };
    // Identity stage s (0 or 1) of a tile: the 32 window columns of the wave's s-th 32-column block,
    // read from the wave's piece of the slot (`part`: 0, or TOK_BYTES for waves whose 64 columns start
    // in the middle of a 128-wide head), times the identity fragment of each k-step.
    auto stage_identity = [&](auto s_c, uint32_t part) {
        constexpr int s = decltype(s_c)::value;
        u32x4 idf[2];
        make_idf(idf);
        request_stage();
        read_t(1, ft1, part);
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) acc[s][ti] = X::mfma(idf[0], ft0[ti], acc[s][ti]);
        stage_barrier(false);
        next_slot();
        if constexpr (s == 1) {                        // the next tile's first stage
            read_w(0, fw0);
            read_t(0, ft0, 0u);
        } else {
            read_t(0, ft0, part);
        }
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) acc[s][ti] = X::mfma(idf[1], ft1[ti], acc[s][ti]);
    };

    // ---- prologue: two stages requested, the first one landed and read ---------------------------------
    load_tile();
    request_stage();
    request_stage();
    clear_acc();
    wait_vmcnt<LOADS>();
    __syncthreads();
    read_w(0, fw0);
    read_t(0, ft0, 0u);

#pragma unroll 1
    for (int r = 0; r < rounds; ++r) {
        const Tile t = tile_of(r);
        // the wave's 64 columns start a head, or (128-wide heads, odd wave) lie in its second half
        const uint32_t id_part = (IDENT && q.d_h > 64 && (wave & 1)) ? (uint32_t)TOK_BYTES : 0u;
        stage_regular(std::integral_constant<int, NEXT_REGULAR>{}, r > 0, 0u);
#pragma unroll 1
        for (int k = 1; k + 1 < nk; ++k) stage_regular(std::integral_constant<int, NEXT_REGULAR>{}, false, 0u);
        if constexpr (IDENT) {
            stage_regular(std::integral_constant<int, NEXT_IDENTITY>{}, false, id_part);
            stage_identity(std::integral_constant<int, 0>{}, id_part);
            stage_identity(std::integral_constant<int, 1>{}, id_part);
        } else {
            stage_regular(std::integral_constant<int, NEXT_REGULAR>{}, false, 0u);
        }

        // ---- results: round, turn each 32 x 32 block round in the wave's staging tile, store -----------
        const int64_t t0 = (int64_t)t.mt * BT;
        const int64_t rows_left = t.valid ? q.M - t0 : 0;
        const __amdgpu_buffer_rsrc_t rD = make_rsrc((char*)q.D + (t.valid ? t0 * q.ldd + t.n0 : 0) * (int64_t)sizeof(OutT),
                                                    rows_left > 0 ? ((rows_left - 1) * q.ldd + BN) * (int64_t)sizeof(OutT) : 0);
        if constexpr (sizeof(OutT) == 4) {
            const int eln = duo_lane_id();
            uint32_t ep_row = (uint32_t)(eln & 31) * (uint32_t)(q.ldd * 4) + (uint32_t)(wave * (32 * TN) + (eln >> 5) * 4) * 4u;
            const uint32_t ep_row_step = 32u * (uint32_t)(q.ldd * 4);
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
                if (ti) ep_row += ep_row_step;
                asm volatile("" : "+v"(ep_row));
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const f32x4 vf = {acc[ni][ti][rg * 4 + 0], acc[ni][ti][rg * 4 + 1], acc[ni][ti][rg * 4 + 2], acc[ni][ti][rg * 4 + 3]};
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vf), rD, ep_row, (ni * 32 + rg * 8) * 4, kStreamStoreAux);
                    }
                }
            }
        } else {
            // lanes l and l + 32 hold columns 0..3 and 4..7 of the same 8-column group; after the swap
            // each lane owns 8 consecutive columns (16 bytes) of its token.  The block (32 tokens x 64
            // bytes) goes through the wave's staging tile and comes back with four lanes per token.
            unsigned char* stag = smem + kDuoStaging + wave * 2048;
            const int eln = duo_lane_id();
            const int e31 = eln & 31;
            const int st_wr = e31 * 64, st_sw = (e31 >> 2) & 3;
            const int rd_row = eln >> 2, rd_c = eln & 3;
            const int rd_off = rd_row * 64 + ((rd_c ^ ((rd_row >> 2) & 3)) << 4);   // rows rd_row and rd_row + 16 share the swizzle
            const uint32_t g_row = (uint32_t)rd_row * (uint32_t)(q.ldd * 2) + (uint32_t)(wave * (32 * TN) + rd_c * 8) * 2u;
            const uint32_t g_step16 = 16u * (uint32_t)(q.ldd * 2);
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr) {
                        uint32_t xv[2], yv[2];
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            xv[h] = X::pack2(acc[ni][ti][(2 * pr) * 4 + 2 * h], acc[ni][ti][(2 * pr) * 4 + 2 * h + 1]);
                            yv[h] = X::pack2(acc[ni][ti][(2 * pr + 1) * 4 + 2 * h], acc[ni][ti][(2 * pr + 1) * 4 + 2 * h + 1]);
                        }
                        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(xv[0], yv[0], false, false);
                        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(xv[1], yv[1], false, false);
                        const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
                        const int chunk = pr * 2 + (eln >> 5);
                        *(u32x4*)(stag + st_wr + ((chunk ^ st_sw) << 4)) = v;
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const u32x4 v = *(const u32x4*)(stag + rd_off + j * 1024);
                        uint32_t off = g_row + (uint32_t)(ti * 2 + j) * g_step16;
                        asm volatile("" : "+v"(off));
                        __builtin_amdgcn_raw_buffer_store_b128(v, rD, off, ni * 64, kStreamStoreAux);
                    }
                }
            }
        }
        clear_acc();
    }
    // nothing of this workgroup may still be on its way into LDS when the workgroup's LDS is handed on
    wait_vmcnt<0>();
}

}  // namespace bda
