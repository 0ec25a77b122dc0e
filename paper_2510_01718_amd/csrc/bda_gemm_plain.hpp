// Lean variant of the streaming MFMA GEMM (bda_gemm_stream.hpp) for launches in which every stage
// of every tile is "plain": K and the head width are multiples of the stage length 64, the basis
// windows start on multiples of 8 and every group's width is a multiple of the 256-column tile.
// Then no stage needs a per-lane decision (but for the one stage per tile that holds the start of a
// window off the 64 grid, which shifts some lanes' offsets by the window's width), and everything
// that changes from stage to stage is uniform:
//   * the vector offset of each of a wave's eight loads never changes; the stage's column / row
//     offset travels in the load's scalar offset;
//   * the LDS addresses of the fragment reads flip between the two stage slots with one addition each.
// Counters on the general kernel showed it to be bound by instruction issue (about 340 instructions
// per wave and stage for 32 MFMAs, a third of them scalar bookkeeping); this variant brings a stage
// down to the MFMAs, the 32 LDS reads, the 8 loads and a few dozen scalar operations.
// Same tile order, pipeline, swizzles and epilogue as the streaming kernel; SK = 64, two slots,
// eight waves (2 x 4).  Three tile heights share the code: 256 tokens (128 tokens x 64 columns per
// wave), 128 and 64 tokens (64 and 32 tokens per wave); the column width is 256 in all of them.
#pragma once
#include <type_traits>

#include "bda_gemm_stream.hpp"

namespace bda {

// one LDS DMA load: LDS address = lds_base + LDS_IMM (lane-linear), global address = descriptor +
// vector offset + scalar offset
template <int LDS_IMM>
__device__ __forceinline__ void lds_dma_imm(u32x4 rsrc, uint32_t lds_base, uint32_t voff, uint32_t soff)
{
    asm volatile(
        "s_add_u32 m0, %0, %4\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, %3 offen lds\n\t"
        :
        : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff), "n"(LDS_IMM)
        : "memory", "m0", "scc");
}

template <typename X, typename OutT, int TT_ = 4>
__global__ __launch_bounds__(512) void gemm_plain_kernel(const GemmArgs p)
{
    constexpr int SK = 64, WN = 4, NW = 8;
    constexpr int TT = TT_, TN = 2;           // TT = 4: 256-token tiles; TT = 2: 128-token tiles; TT = 1: 64-token tiles
    constexpr int BT = 64 * TT, BN = 256;
    constexpr int PR = SK / 8, RB = SK * 2, RPI = 64 / PR, KS = SK / 16;
    constexpr int PIT = BT / RPI / NW, PIW = SK / 2 / NW;
    constexpr int TOK_BYTES = BT * RB;
    constexpr int STAGE_BYTES = TOK_BYTES + SK * BN * 2;
    constexpr int STORES = TT * TN * (sizeof(OutT) == 4 ? 4 : 2);
    static_assert((TT == 4 || TT == 2 || TT == 1) && PIT == TT && PIW == 4 && STAGE_BYTES % 1024 == 0, "layout constants of this variant");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    struct {
        const void *A, *B; void* D;
        int64_t lda, ldb, ldd, M;
        int K, n_groups, d_h, a_skip, ident, m_tiles, n_tiles, sm, sn, n_stage_id, n_super_m, n_super_n, sn_shift;
        uint64_t dh_magic;
        int ts1, ts2, rounds, xq0, xr0, xcount, lin_slots;
    } q = {p.A, p.B, p.D, p.lda, p.ldb, p.ldd, p.M, p.K, p.n_groups, p.d_h, p.a_skip, p.ident, p.m_tiles, p.n_tiles,
           p.sm, p.sn, p.n_stage_id, p.n_super_m, p.n_super_n, p.sn_shift, p.dh_magic, p.tile_start[1], p.tile_start[2],
           p.rounds, p.xcd_q0[blockIdx.x % kNumXcd], p.xcd_r0[blockIdx.x % kNumXcd], p.xcd_count[blockIdx.x % kNumXcd], p.lin_slots};
    asm volatile("" : "+s"(q.A), "+s"(q.B), "+s"(q.D), "+s"(q.lda), "+s"(q.ldb), "+s"(q.ldd), "+s"(q.M), "+s"(q.dh_magic));
    asm volatile("" : "+s"(q.K), "+s"(q.n_groups), "+s"(q.d_h), "+s"(q.a_skip), "+s"(q.ident), "+s"(q.m_tiles), "+s"(q.n_tiles),
                 "+s"(q.sm), "+s"(q.sn), "+s"(q.n_stage_id), "+s"(q.n_super_m), "+s"(q.n_super_n), "+s"(q.sn_shift),
                 "+s"(q.ts1), "+s"(q.ts2), "+s"(q.rounds), "+s"(q.xq0), "+s"(q.xr0), "+s"(q.xcount), "+s"(q.lin_slots));

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave / WN, wn = wave % WN;
    const int l31 = lane & 31, lhi = lane >> 5;

    const int nk = q.K / SK;
    const int n_id = q.ident ? q.n_stage_id : 0;
    const int S = nk + n_id;
    const int xcd = blockIdx.x % kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    const bool linear = q.lin_slots > 0;      // tiles one by one in column-major order (sm = sn = 1 on the host side)
    const int slot_m = linear ? 0 : slot >> q.sn_shift, slot_n = linear ? 0 : slot & (q.sn - 1);
    auto mod_dh = [&](int x) { return x - (int)(((uint64_t)(uint32_t)x * q.dh_magic) >> 40) * q.d_h; };

    // ---- tile set-up (scalar) -----------------------------------------------------------------------
    // Super-tiles (sm x sn tiles) are numbered down the token dimension first; die x works through
    // the numbers [x R, (x + 1) R), R = rounds.  A workgroup keeps its slot inside the super-tile, so
    // from one round to the next it usually moves down by sm token tiles and keeps its columns: the
    // die's L2 keeps the sn weight tiles and only the token tiles stream, and the column half of the
    // set-up (group lookup, weight descriptor) is done only when the column changes.
    const int n_rounds = q.rounds;
    // Small tile grids, where whole super-tiles would leave dies or compute units without work, are
    // dealt out tile by tile instead: die x takes a contiguous run of the column-major tile order and
    // its workgroups walk the run with stride lin_slots (the same code with one-tile "super-tiles").
    const int su_step = linear ? q.lin_slots : 1;
    int su_q = q.xq0 + (linear ? slot : 0), su_r = q.xr0, su_left = q.xcount - (linear ? slot : 0);
    while (su_q >= q.n_super_m) { su_q -= q.n_super_m; ++su_r; }
    struct { u32x4 rB; int64_t n0; int cols_left, a_off, j_lo, rel_blk0; bool ok; } col;
    bool col_dirty = true;
    auto setup_cols = [&]() {
        const int nt = su_r * q.sn + slot_n;
        col.ok = nt < q.n_tiles;
        int g = 0;
        if (q.n_groups <= 2) g = (q.n_groups == 2 && nt >= q.ts1) ? 1 : 0;
        else if (nt >= q.ts1) { g = 1; while (g + 1 < q.n_groups && nt >= p.tile_start[g + 1]) ++g; }
        // (column starts fit 24 bits here; the three table reads go out together)
        const int g_tile0 = g == 0 ? 0 : g == 1 ? q.ts1 : p.tile_start[g];
        const int g_col0 = (int)p.col_start[g], g_col1 = (int)p.col_start[g + 1], g_off = p.a_off[g];
        const int rel0 = col.ok ? (nt - g_tile0) * BN : 0;
        col.n0 = col.ok ? g_col0 + rel0 : 0;
        const int left = g_col1 - (int)col.n0;
        col.cols_left = col.ok ? (left > BN ? BN : left) : 0;
        col.a_off = g_off;
        const int r0 = q.ident ? mod_dh(rel0) : 0;
        col.j_lo = (q.ident && (q.d_h & (BN - 1)) == 0) ? r0 : 0;
        col.rel_blk0 = q.ident ? mod_dh(r0 + wn * (32 * TN)) : 0;
        col.rB = make_rsrc_words((const char*)q.B + col.n0 * 2,
                                 col.ok ? ((int64_t)(q.K - 1) * q.ldb + col.cols_left) * 2 : 0);
    };
    auto setup = [&]() -> StreamTile {
        StreamTile t;
        if (su_left <= 0) {                   // past the die's last super-tile: a tile that fetches and stores nothing
            t.rA = make_rsrc_words(q.A, 0);
            t.rB = make_rsrc_words(q.B, 0);
            t.d_off = 0; t.rows_left = 0; t.cols_left = 0; t.a_off = 0; t.j_lo = 0; t.rel_blk0 = 0;
            return t;
        }
        if (col_dirty) setup_cols();
        const int mt = su_q * q.sm + slot_m;
        const bool valid = su_left > 0 && col.ok && mt < q.m_tiles;
        const int64_t t0 = valid ? (int64_t)mt * BT : 0;
        t.rows_left = valid ? q.M - t0 : 0;
        t.cols_left = valid ? col.cols_left : 0;
        t.a_off = col.a_off;
        t.j_lo = col.j_lo;
        t.rel_blk0 = col.rel_blk0;
        t.d_off = t0 * q.ldd + col.n0;
        t.rA = make_rsrc_words((const char*)q.A + t0 * q.lda * 2,
                               valid ? ((t.rows_left - 1) * q.lda + q.K + q.a_skip) * 2 : 0);
        t.rB = col.rB;
        if (!valid) t.rB[2] = 0;
        // next super-tile of this die
        su_left -= su_step;
        col_dirty = false;
        su_q += su_step;
        while (su_q >= q.n_super_m) { su_q -= q.n_super_m; ++su_r; col_dirty = true; }
        return t;
    };


    // identity fragments (row operand): lane (row i = l31, half lhi) holds k' = 16 v + 8 lhi + e.
    // Built where they are used, from a copy of the lane id the optimiser cannot see through, so that
    // they do not occupy registers during the regular stages.
    auto make_idf = [&](u32x4 (&idf)[2]) {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int r31 = ln & 31, rhi = ln >> 5;
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int k0 = 16 * v + 8 * rhi + 2 * w;
                idf[v][w] = (k0 == r31 ? IdentityFrag<X>::one : 0u) | (k0 + 1 == r31 ? IdentityFrag<X>::one << 16 : 0u);
            }
    };


    // ---- producer: per-lane offsets are constants of the launch ----------------------------------------
    const uint32_t tok_row_bytes = (uint32_t)(q.lda * 2);
    const uint32_t wgt_row_bytes = (uint32_t)(q.ldb * 2);
    uint32_t vo_tok[PIT], vo_wgt[2];
#pragma unroll
    for (int j = 0; j < PIT; ++j)
        vo_tok[j] = (uint32_t)(wave * (RPI * PIT) + lane / PR + RPI * j) * tok_row_bytes
                    + (uint32_t)(((lane % PR) ^ tok_swz<SK>((wave * (RPI * PIT) + lane / PR + RPI * j) & 15)) * 16);   // (the row's own low bits: a wave of the 64-token variant owns 8 rows)
#pragma unroll
    for (int j = 0; j < 2; ++j)
        vo_wgt[j] = (uint32_t)(wave * (2 * PIW) + (lane >> 5)) * wgt_row_bytes + (uint32_t)(((lane & 31) ^ wgt_swz(2 * j + (lane >> 5))) * 16);
    const uint32_t wave_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem
                              + (uint32_t)wave * 4096u;           // this wave's 4 KiB of each half slot (absolute LDS address)
    const uint32_t wgt_step = 2u * wgt_row_bytes;                  // rows between a wave's weight loads

    // Requests stage k of tile t into the slot at byte `slot_b`; loads j0 .. j0+3 (0: tokens, 4: weights).
    auto stage_soff_tok = [&](const StreamTile& t, int k) -> uint32_t {
        const int k0 = k * SK;
        return k < nk ? (uint32_t)(k0 + (k0 >= t.a_off ? q.a_skip : 0)) * 2u : (uint32_t)(t.a_off + t.j_lo + (k - nk) * (2 * SK)) * 2u;
    };
    // Identity stages are two stage lengths wide: window columns [j, j + 64) of the stage go to the
    // token half of the slot and [j + 64, j + 128) to its weight half (same layout; an identity stage
    // has no weights).  A wave's 64 output columns take their slice from one of the two: which one.
    auto id_half = [&](const StreamTile& t, int k) -> int {
        const int diff = t.rel_blk0 - (t.j_lo + (k - nk) * (2 * SK));
        return (k >= nk && diff >= SK && diff < 2 * SK) ? 1 : 0;
    };
    // (a wave's token rows take PIT KiB of a slot's token half, its weight rows 4 KiB of the weight
    // half; `lds_b` is the slot plus 4 KiB per wave, so the token side steps back for PIT < 4)
    const uint32_t tok_back = (uint32_t)wave * (uint32_t)(4096 - 1024 * PIT);
    // Per-lane token offsets of stage k of tile t: the launch constants, except in the one stage
    // that holds the start of a basis window that is not a multiple of the stage length: there the
    // 16-byte pieces at or past the window's start skip the window (uniform branch, once per tile).
    const uint32_t skip_bytes = (uint32_t)q.a_skip * 2u;
    auto tok_voffs = [&](const StreamTile& t, int k, uint32_t (&vt)[PIT]) {
#pragma unroll
        for (int j = 0; j < PIT; ++j) vt[j] = vo_tok[j];
        const int e = t.a_off & (SK - 1);
        if (e != 0 && k == t.a_off / SK && k < nk) {
            int ln = lane;
            asm volatile("" : "+v"(ln));
#pragma unroll
            for (int j = 0; j < PIT; ++j) {
                const int x = ((ln % PR) ^ tok_swz<SK>((wave * (RPI * PIT) + ln / PR + RPI * j) & 15)) * 8;   // first k of the lane's piece, within the stage
                if (x >= e) vt[j] += skip_bytes;
            }
        }
    };
    auto tok_load = [&](auto jc, const StreamTile& t, uint32_t lds_b, uint32_t soff, const uint32_t (&vt)[PIT]) {
        constexpr int j = decltype(jc)::value;
        if constexpr (j < PIT) lds_dma_imm<1024 * j>(t.rA, lds_b - tok_back, vt[j], soff);
    };
    // The four loads of a stage that go to the weight half of the slot: rows of the weight tile, or
    // (identity stage) the second 64 window columns of the token rows.  Uniform choice per stage.
    // (With 128-token tiles the second token set has two loads per wave, with 64-token tiles one; the others keep the
    // stage's load count and write zeros to the unused part of the weight half, 2 KiB per wave.)
    auto slot_of = [&](uint32_t lds_b) { return lds_b - (uint32_t)wave * 4096u; };   // slot start (absolute LDS address)
    struct Second { u32x4 r; uint32_t base, base_unused; uint32_t so, so_step; uint32_t v[4]; };
    auto second_set = [&](const StreamTile& t, int k, uint32_t lds_b, uint32_t ts, const uint32_t (&vt)[PIT]) -> Second {
        Second z;
        const bool id = k >= nk;
        z.r = id ? t.rA : t.rB;
        z.base = id ? lds_b - tok_back : lds_b;
        z.base_unused = id ? slot_of(lds_b) + (uint32_t)(7 * PIT * 1024) + (uint32_t)wave * (uint32_t)((4 - PIT) * 1024) : lds_b;
        z.so = id ? ts + (uint32_t)(2 * SK) : (uint32_t)(k * SK) * wgt_row_bytes;
        z.so_step = id ? 0u : wgt_step;
#pragma unroll
        for (int j = 0; j < 4; ++j) z.v[j] = id ? (j < PIT ? vt[j < PIT ? j : 0] : kBadOffset) : vo_wgt[j & 1];
        return z;
    };
    auto wgt_load = [&](auto jc, const Second& z) {
        constexpr int j = decltype(jc)::value;
        lds_dma_imm<TOK_BYTES + 1024 * j>(z.r, j < PIT ? z.base : z.base_unused, z.v[j], z.so + (uint32_t)j * z.so_step);
    };
    auto produce_all = [&](const StreamTile& t, int k, uint32_t slot_b) {
        const uint32_t lds_b = slot_b + wave_lds;
        const uint32_t ts = stage_soff_tok(t, k);
        uint32_t vt[PIT];
        tok_voffs(t, k, vt);
        tok_load(std::integral_constant<int, 0>{}, t, lds_b, ts, vt);      // (loads with j >= PIT are no-ops)
        tok_load(std::integral_constant<int, 1>{}, t, lds_b, ts, vt);
        tok_load(std::integral_constant<int, 2>{}, t, lds_b, ts, vt);
        tok_load(std::integral_constant<int, 3>{}, t, lds_b, ts, vt);
        const Second z = second_set(t, k, lds_b, ts, vt);
        wgt_load(std::integral_constant<int, 0>{}, z);
        wgt_load(std::integral_constant<int, 1>{}, z);
        wgt_load(std::integral_constant<int, 2>{}, z);
        wgt_load(std::integral_constant<int, 3>{}, z);
    };

    // ---- consumer ---------------------------------------------------------------------------------
    auto mm = [](u32x4 a, u32x4 b, f32x16 c) -> f32x16 { return X::mfma(a, b, c); };
    f32x16 acc[TN][TT];
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    u32x4 fw0[TN], ft0[TT], fw1[TN], ft1[TT];

    // LDS addresses of this lane's fragments in the slot being read; moved to the other slot (plus or
    // minus the slot size) after a stage's last read
    // (absolute LDS addresses: the start of the dynamic LDS block is folded in here once)
    typedef __attribute__((address_space(3))) unsigned char* lds_u8;
    typedef __attribute__((address_space(3))) const u32x4* lds_u32x4;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8)smem;
    uint32_t a_tok = lds0 + (uint32_t)((wt * (32 * TT) + l31) * RB + ((lhi ^ tok_swz<SK>(l31 & 15)) << 4));
    uint32_t a_wgt[TN];
    {
        const int c_s = lane & 15, c_gq = lane >> 4;
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const int col = wn * (32 * TN) + ni * 32 + 16 * (c_gq & 1) + 4 * (c_s & 3);
            const int piece = (col >> 3) ^ wgt_swz(c_s >> 2);
            a_wgt[ni] = lds0 + (uint32_t)(TOK_BYTES + (8 * lhi + (c_s >> 2)) * 512 + (piece << 4) + ((col & 4) << 1));
        }
    }
    uint32_t flip = (uint32_t)STAGE_BYTES;     // uniform: +slot size, then -slot size, ...
    auto flip_slot = [&]() {
        a_tok += flip;
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) a_wgt[ni] += flip;
        flip = 0u - flip;
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
    auto read_t = [&](int ks, u32x4 (&ft)[TT], uint32_t half_off = 0u) {   // half_off: TOK_BYTES for the weight half (identity stages)
        const uint32_t a = (a_tok ^ (uint32_t)(ks << 5)) + half_off;
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) ft[ti] = *(lds_u32x4)(uintptr_t)(a + ti * (32 * RB));
    };
    // k-step s (16 window columns from jc + 16 s) of an identity stage.  The stage's 64 window columns start
    // at a multiple of 64 (jc), and so do the wave's 64 output columns within their head (rel_blk0; the head
    // width is a multiple of 64).  So either the stage holds the wave's slice (`hit`: jc == rel_blk0), and then
    // k-steps 0, 1 meet the wave's first 32-column block and k-steps 2, 3 its second, with the lower or upper
    // 16 columns of the block in turn (which identity fragment) - or it holds none of it.
    static_assert(TN == 2, "identity k-steps are laid out for waves of two 32-column blocks");
    auto mma_identity = [&](auto sc, bool hit, const u32x4 (&idf)[2], const u32x4 (&ft)[TT]) {
        constexpr int s = decltype(sc)::value;
        if (hit) {
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[s >> 1][ti] = mm(idf[s & 1], ft[ti], acc[s >> 1][ti]);
        }
    };

    // One stage of tile `cur` out of the slot at `slot_b`, during which stage pk of tile pt is requested
    // into the same slot once every wave has read it.  In a regular stage the eight MFMAs of each of the
    // last two k-steps carry four loads between them.
    uint32_t slot_b = 0;
    u32x4 idf_keep[2];
    make_idf(idf_keep);
    auto stage = [&](auto regular, auto first_of_tile, const StreamTile& cur, int kc, const StreamTile& pt, int pk, bool relaxed) {
        constexpr bool REG = decltype(regular)::value;
        constexpr bool FIRST = decltype(first_of_tile)::value;   // only then may result stores be in flight
        const bool next_regular = kc + 1 < nk || kc + 1 == S;
        const int half_cur = REG ? 0 : id_half(cur, kc);
        const uint32_t off_cur = half_cur ? (uint32_t)TOK_BYTES : 0u;
        const uint32_t off_next = (!next_regular && id_half(cur, kc + 1)) ? (uint32_t)TOK_BYTES : 0u;
        const int jc = cur.j_lo + (kc - nk) * (2 * SK) + half_cur * SK;
        const bool id_hit = !REG && jc == cur.rel_blk0;
        const u32x4 (&idf)[2] = idf_keep;
        // The two waves of a SIMD run the same code and the older one wins every arbitration, so it
        // runs ahead to the barrier and leaves the other to work through the stage alone.  Alternating
        // the priority by half stages keeps them side by side (measured: 4-8 % faster).
        if (wt == 0) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
        if constexpr (!REG) {
            // An identity stage has half the MFMAs of a regular one and moves as many bytes, so it does
            // not split into halves: all its token fragments are asked for at once (this frees the slot),
            // the barrier follows, and the eight requests for the next tile go between all sixteen MFMAs.
            u32x4 ft2[TT], ft3[TT];
            read_t(1, ft1, off_cur); read_t(2, ft2, off_cur); read_t(3, ft3, off_cur);
            flip_slot();
            const uint32_t lds_b = slot_b + wave_lds;
            const uint32_t ts = stage_soff_tok(pt, pk);
            uint32_t vt[PIT];
            tok_voffs(pt, pk, vt);
            const Second z = second_set(pt, pk, lds_b, ts, vt);
            wait_vmcnt<0>();
            __syncthreads();
            if (wt == 0) __builtin_amdgcn_s_setprio(0); else __builtin_amdgcn_s_setprio(1);
            mma_identity(std::integral_constant<int, 0>{}, id_hit, idf, ft0);
            tok_load(std::integral_constant<int, 0>{}, pt, lds_b, ts, vt);
            tok_load(std::integral_constant<int, 1>{}, pt, lds_b, ts, vt);
            if (next_regular) read_w(0, fw0);
            read_t(0, ft0, off_next);
            mma_identity(std::integral_constant<int, 1>{}, id_hit, idf, ft1);
            tok_load(std::integral_constant<int, 2>{}, pt, lds_b, ts, vt);
            tok_load(std::integral_constant<int, 3>{}, pt, lds_b, ts, vt);
            mma_identity(std::integral_constant<int, 2>{}, id_hit, idf, ft2);
            wgt_load(std::integral_constant<int, 0>{}, z);
            wgt_load(std::integral_constant<int, 1>{}, z);
            mma_identity(std::integral_constant<int, 3>{}, id_hit, idf, ft3);
            wgt_load(std::integral_constant<int, 2>{}, z);
            wgt_load(std::integral_constant<int, 3>{}, z);
            slot_b = (uint32_t)STAGE_BYTES - slot_b;
            return;
        }
        // ---- a regular stage ----
        read_w(1, fw1); read_t(1, ft1);
        // the first k-step of a tile starts the sums: its MFMAs take zero as their addend, so the
        // accumulators are never cleared
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(fw0[ni], ft0[ti], FIRST ? zero16 : acc[ni][ti]);
        read_w(2, fw0); read_t(2, ft0);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(fw1[ni], ft1[ti], acc[ni][ti]);
        // last read of this slot
        read_w(3, fw1); read_t(3, ft1);
        flip_slot();
        // uniform part of the requests that follow the barrier
        const uint32_t lds_b = slot_b + wave_lds;
        const uint32_t ts = stage_soff_tok(pt, pk);
        uint32_t vt[PIT];
        tok_voffs(pt, pk, vt);
        const Second z = second_set(pt, pk, lds_b, ts, vt);
        if (FIRST && relaxed) wait_vmcnt<STORES>(); else wait_vmcnt<0>();
        __syncthreads();
        if (wt == 0) __builtin_amdgcn_s_setprio(0); else __builtin_amdgcn_s_setprio(1);
        if constexpr (TT == 4) {
            acc[0][0] = mm(fw0[0], ft0[0], acc[0][0]); acc[0][1] = mm(fw0[0], ft0[1], acc[0][1]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 0>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
            acc[0][2] = mm(fw0[0], ft0[2], acc[0][2]); acc[0][3] = mm(fw0[0], ft0[3], acc[0][3]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 1>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mm(fw0[1], ft0[0], acc[1][0]); acc[1][1] = mm(fw0[1], ft0[1], acc[1][1]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 2>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
            acc[1][2] = mm(fw0[1], ft0[2], acc[1][2]); acc[1][3] = mm(fw0[1], ft0[3], acc[1][3]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 3>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
        } else if constexpr (TT == 2) {
            acc[0][0] = mm(fw0[0], ft0[0], acc[0][0]); acc[0][1] = mm(fw0[0], ft0[1], acc[0][1]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 0>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mm(fw0[1], ft0[0], acc[1][0]); acc[1][1] = mm(fw0[1], ft0[1], acc[1][1]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 1>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
        } else {
            acc[0][0] = mm(fw0[0], ft0[0], acc[0][0]);
            __builtin_amdgcn_sched_barrier(0); tok_load(std::integral_constant<int, 0>{}, pt, lds_b, ts, vt); __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mm(fw0[1], ft0[0], acc[1][0]);
        }
        // first fragments of the next stage, out of the other slot
        if (next_regular) read_w(0, fw0);
        read_t(0, ft0, off_next);
        if constexpr (TT == 4) {
            acc[0][0] = mm(fw1[0], ft1[0], acc[0][0]); acc[0][1] = mm(fw1[0], ft1[1], acc[0][1]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 0>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[0][2] = mm(fw1[0], ft1[2], acc[0][2]); acc[0][3] = mm(fw1[0], ft1[3], acc[0][3]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 1>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mm(fw1[1], ft1[0], acc[1][0]); acc[1][1] = mm(fw1[1], ft1[1], acc[1][1]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 2>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[1][2] = mm(fw1[1], ft1[2], acc[1][2]); acc[1][3] = mm(fw1[1], ft1[3], acc[1][3]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 3>{}, z); __builtin_amdgcn_sched_barrier(0);
        } else if constexpr (TT == 2) {
            acc[0][0] = mm(fw1[0], ft1[0], acc[0][0]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 0>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[0][1] = mm(fw1[0], ft1[1], acc[0][1]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 1>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mm(fw1[1], ft1[0], acc[1][0]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 2>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[1][1] = mm(fw1[1], ft1[1], acc[1][1]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 3>{}, z); __builtin_amdgcn_sched_barrier(0);
        } else {
            acc[0][0] = mm(fw1[0], ft1[0], acc[0][0]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 0>{}, z); wgt_load(std::integral_constant<int, 1>{}, z); __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mm(fw1[1], ft1[0], acc[1][0]);
            __builtin_amdgcn_sched_barrier(0); wgt_load(std::integral_constant<int, 2>{}, z); wgt_load(std::integral_constant<int, 3>{}, z); __builtin_amdgcn_sched_barrier(0);
        }
        slot_b = (uint32_t)STAGE_BYTES - slot_b;
    };

    StreamTile cur = setup();
    // prologue: the first two stages of the first tile; every wave's first stage is queued before
    // anybody's second
    produce_all(cur, 0, 0u);
    __builtin_amdgcn_s_barrier();
    produce_all(cur, 1, (uint32_t)STAGE_BYTES);
    wait_vmcnt<PIT + PIW>();
    __syncthreads();
    read_w(0, fw0);
    read_t(0, ft0);

    const std::true_type REGULAR{};
    const std::false_type IDENTITY{};
    const int split = S - 2;                  // from this stage on, the next tile is being requested
    const int r_same = nk < split ? nk : split;
    const int i_same = split > nk ? split : nk;
#pragma unroll 1
    for (int round = 0; round < n_rounds; ++round) {
        const bool after_tile = round > 0;
        // stage 0 of the tile apart (host contract: S >= 3, so it requests stage 2 of the same tile)
        stage(REGULAR, std::true_type{}, cur, 0, cur, 2, after_tile);
        // (the next tile is not needed before stage S - 2; its scalar set-up sits here, where the MFMA
        // pipe has work queued, rather than at the top of the round, where it has none)
        const StreamTile nxt = setup();
        int kc = 1;
#pragma unroll 1
        for (; kc < r_same; ++kc) stage(REGULAR, std::false_type{}, cur, kc, cur, kc + 2, false);
#pragma unroll 1
        for (; kc < nk; ++kc) stage(REGULAR, std::false_type{}, cur, kc, nxt, kc - split, false);
#pragma unroll 1
        for (; kc < i_same; ++kc) stage(IDENTITY, std::false_type{}, cur, kc, cur, kc + 2, false);
#pragma unroll 1
        for (; kc < S; ++kc) stage(IDENTITY, std::false_type{}, cur, kc, nxt, kc - split, false);

        // ---- epilogue ---------------------------------------------------------------------------
        // rows past the end of the tensor and tiles outside the grid fall outside rD's range
        const __amdgpu_buffer_rsrc_t rD = make_rsrc(
            (char*)q.D + cur.d_off * (int64_t)sizeof(OutT),
            cur.cols_left > 0 ? ((cur.rows_left - 1) * q.ldd + cur.cols_left) * (int64_t)sizeof(OutT) : 0);
        if constexpr (sizeof(OutT) == 4) {
            // float32 results: a lane holds runs of 4 consecutive columns (16 bytes) of one row, lanes l and
            // l+32 adjacent runs.  Stored as they are, an instruction would write 32 bytes of each of 32
            // rows, which the memory pipeline takes at a third of its rate; so a 32-row x 32-column block
            // (4 KiB) is turned round in the wave's staging region, as below for the 16-bit types, and 8
            // consecutive lanes store one full 128-byte line of a row.
            unsigned char* stag = smem + 2 * STAGE_BYTES + wave * 4096;
            int eln = lane;
            asm volatile("" : "+v"(eln));
            const int e31 = eln & 31;
            const int st_wr = e31 * 128;
            const int st_sw = (e31 ^ (e31 >> 3)) & 7;
            const int rd_row = eln >> 3, rd_chunk = eln & 7;
            uint32_t g_row = (uint32_t)(wt * (32 * TT) + rd_row) * (uint32_t)(q.ldd * 4) + (uint32_t)(wn * (32 * TN) * 4 + rd_chunk * 16);
            const uint32_t g_step8 = 8u * (uint32_t)(q.ldd * 4);
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const f32x4 vf = {acc[ni][ti][rg * 4 + 0], acc[ni][ti][rg * 4 + 1], acc[ni][ti][rg * 4 + 2], acc[ni][ti][rg * 4 + 3]};
                        const int chunk = 2 * rg + (eln >> 5);           // 16-byte piece of the row's 128 bytes
                        *(u32x4*)(stag + st_wr + ((chunk ^ st_sw) << 4)) = __builtin_bit_cast(u32x4, vf);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int row = j * 8 + rd_row;
                        const u32x4 v = *(const u32x4*)(stag + row * 128 + ((rd_chunk ^ ((row ^ (row >> 3)) & 7)) << 4));
                        uint32_t off = g_row + (uint32_t)(ti * 4 + j) * g_step8;
                        asm volatile("" : "+v"(off));
                        __builtin_amdgcn_raw_buffer_store_b128(v, rD, off, ni * 128, kStreamStoreAux);
                    }
                }
            }
        } else {
            // lanes l and l+32 hold columns 0..3 and 4..7 of the same 8-column block; after the swap
            // the lower half-wave owns the even blocks and the upper half-wave the odd blocks, each
            // lane with 8 consecutive columns = 16 bytes.  A 32-row x 64-column piece is then turned
            // round in a 4 KiB LDS region private to the wave, so that 8 consecutive lanes store one
            // full 128-byte line of a row (the memory pipeline works on whole lines).
            unsigned char* stag = smem + 2 * STAGE_BYTES + wave * 4096;
            int eln = lane;                       // opaque copy: keeps these constants out of the k loops
            asm volatile("" : "+v"(eln));
            const int e31 = eln & 31;
            const int st_wr = e31 * 128;                                    // + ((chunk ^ sw) << 4)
            const int st_sw = (e31 ^ (e31 >> 3)) & 7;
            const int rd_row = eln >> 3, rd_chunk = eln & 7;
            uint32_t g_row = (uint32_t)(wt * (32 * TT) + rd_row) * (uint32_t)(q.ldd * 2) + (uint32_t)(wn * (32 * TN) + rd_chunk * 8) * 2u;
            const uint32_t g_step8 = 8u * (uint32_t)(q.ldd * 2);
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
#pragma unroll
                for (int h = 0; h < TN / 2; ++h) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int nn = 0; nn < 2; ++nn) {
                        const int ni = 2 * h + nn;
#pragma unroll
                        for (int pr = 0; pr < 2; ++pr) {
                            uint32_t xv[2], yv[2];
#pragma unroll
                            for (int q = 0; q < 2; ++q) {
                                xv[q] = X::pack2(acc[ni][ti][(2 * pr) * 4 + 2 * q], acc[ni][ti][(2 * pr) * 4 + 2 * q + 1]);
                                yv[q] = X::pack2(acc[ni][ti][(2 * pr + 1) * 4 + 2 * q], acc[ni][ti][(2 * pr + 1) * 4 + 2 * q + 1]);
                            }
                            const u32x2 s0 = __builtin_amdgcn_permlane32_swap(xv[0], yv[0], false, false);
                            const u32x2 s1 = __builtin_amdgcn_permlane32_swap(xv[1], yv[1], false, false);
                            const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
                            const int chunk = nn * 4 + pr * 2 + (eln >> 5);  // 16-byte piece of the 64 columns
                            *(u32x4*)(stag + st_wr + ((chunk ^ st_sw) << 4)) = v;
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int row = j * 8 + rd_row;
                        const u32x4 v = *(const u32x4*)(stag + row * 128 + ((rd_chunk ^ ((row ^ (row >> 3)) & 7)) << 4));
                        uint32_t off = g_row + (uint32_t)(ti * 4 + j) * g_step8;
                        asm volatile("" : "+v"(off));
                        __builtin_amdgcn_raw_buffer_store_b128(v, rD, off, h * 128, kStreamStoreAux);
                    }
                }
            }
        }
        cur = nxt;
    }
    wait_vmcnt<0>();
}

}  // namespace bda
