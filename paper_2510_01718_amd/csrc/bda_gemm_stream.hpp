// Streaming MFMA GEMM for gfx950: the large-T kernel of libbda.
//
//   D[t, n] = ident(t, n) + sum_{k < K} A[t, acol_g(k)] * B[k, n]        (see bda_gemm_kernels.hpp)
//
// What is different from the register-staged kernel in bda_gemm_kernels.hpp:
//   * Global -> LDS copies never touch registers: every 16-byte piece is moved by
//     buffer_load_dwordx4 ... lds (LDS DMA).  The token tile lands k-contiguous, the weight tile
//     n-contiguous exactly as it lies in memory; the weight fragments are then read with the
//     transposing LDS read ds_read_b64_tr_b16, so no shuffling instructions are spent on them.
//   * The contraction is cut into stages of SK (64 in the library) and the LDS holds NS (2) stages.
//     The stage sequence continues across output tiles: while the last stage of one tile is
//     multiplied and its results are stored, the first stages of the workgroup's next tile are
//     already in flight.  One barrier per stage, placed after the stage's last fragment read; the
//     loads that refill the freed slot are issued one by one between the MFMAs of the stage's last
//     two k-steps, so that no wave sits in the memory pipeline's queue with nothing else to issue.
//     Every workgroup runs the same number of tiles of the same number of stages (a tile position
//     that falls outside the grid becomes a tile whose loads fetch nothing and whose stores are
//     dropped), so the per-stage code has no tile bookkeeping in it.
//   * Bank conflicts are avoided by permuting which 16-byte piece each lane of a load fetches (the
//     LDS image of one load instruction is always lane-linear), so the tiles need no padding.
//   * 16-bit results are exchanged between the two half-waves (v_permlane32_swap) and turned round
//     in a small per-wave LDS region so that eight lanes store one full 128-byte line.
//   * Tile order: super-tiles of sm x sn tiles are numbered down the token dimension first and die x
//     takes a contiguous range of them, so a workgroup usually keeps its columns from one tile to
//     the next: the die's L2 keeps the weight tiles, and only the row half of the set-up is redone.
//
// The LDS DMA loads are issued from inline assembly: the compiler would otherwise wait for ALL
// outstanding loads before any LDS read, which would serialise the stages.  Their completion is
// tracked by hand with s_waitcnt vmcnt(n); every wave issues the same number of loads per stage
// (loads that have nothing to fetch use an out-of-range offset and return zeros).  For the same
// reason the kernel must not spill: a register reload is a memory load the compiler does know
// about, and it would wait for it - and with it for every DMA load - inside the k loop.  Values
// needed only in one phase (identity fragments, store addresses) are therefore rebuilt there from
// a copy of the lane id that the optimiser cannot see through.
#pragma once
#include <type_traits>

#include "bda_gemm_kernels.hpp"

namespace bda {


// Cache policy of the result stores: bit 1 = non-temporal.  The output is written once and not read
// again by this kernel; streaming it keeps the latent and weight tiles in the L2.
constexpr int kStreamStoreAux = 2;

// s_waitcnt vmcnt(n) with the other counters left alone.  Issued as volatile assembly with a memory
// clobber: the count includes loads the compiler issues for builtins (token fragments, identity
// values) next to the DMA requests written in assembly, so no memory access may be moved across the
// wait in either direction - it is the program order at this point that the count was made for.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is six bits");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// N (2 or 4) LDS DMA loads of 16 bytes per lane through one descriptor; the LDS image of load j
// starts at lds_base + 1024 j and is lane-linear (lane l -> bytes [16 l, 16 l + 16)).  The LDS address
// of such a load is M0 + instruction offset + 16 lane, and the instruction offset would also be added
// to the global address, so M0 is advanced instead.
__device__ __forceinline__ void lds_dma2(u32x4 rsrc, uint32_t lds_base, uint32_t v0, uint32_t v1)
{
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %3, 0 offen lds\n\t"
        "s_add_u32 m0, m0, 0x400\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %2, %3, 0 offen lds\n\t"
        :
        : "s"(lds_base), "v"(v0), "v"(v1), "s"(rsrc)
        : "memory", "m0", "scc");
}
__device__ __forceinline__ void lds_dma1(u32x4 rsrc, uint32_t lds_addr, uint32_t v0)
{
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, 0 offen lds\n\t"
        :
        : "s"(lds_addr), "v"(v0), "s"(rsrc)
        : "memory", "m0");
}
// the same with a scalar byte offset added to the address (the LDS side is unaffected)
__device__ __forceinline__ void lds_dma1s(u32x4 rsrc, uint32_t lds_addr, uint32_t v0, uint32_t soff)
{
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, %3 offen lds\n\t"
        :
        : "s"(lds_addr), "v"(v0), "s"(rsrc), "s"(soff)
        : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void lds_dma(u32x4 rsrc, uint32_t lds_base, const uint32_t (&v)[N])
{
    static_assert(N % 2 == 0, "an even number of loads per call");
#pragma unroll
    for (int j = 0; j < N; j += 2) lds_dma2(rsrc, lds_base + 1024u * j, v[j], v[j + 1]);
}

__device__ __forceinline__ u32x4 make_rsrc_words(const void* base, int64_t bytes)
{
    const uint64_t a = (uint64_t)base;
    const uint32_t range = (uint32_t)(bytes > kMaxRange ? kMaxRange : (bytes < 0 ? 0 : bytes));
    u32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    r[2] = __builtin_amdgcn_readfirstlane(range);
    r[3] = 0x00020000u;
    return r;
}

// Token tile in LDS: row = SK k = four (SK = 32) or eight (SK = 64) 16-byte pieces; piece q of row r
// sits at position q ^ tok_swz<SK>(r).  Chosen so that the 32 lanes of a fragment read (32
// consecutive rows, same q) are conflict-free whether the LDS serves 16 lanes x 16 bytes over 64
// banks or 8 lanes over 32 banks.
template <int SK>
__device__ __forceinline__ int tok_swz(int r)
{
    if constexpr (SK == 32)
        return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1);
    else
        return (r ^ (r >> 3)) & 7;
}
// Weight tile in LDS: row = one k = 256 columns = 512 bytes = thirty-two 16-byte pieces; piece c of
// row k sits at position c ^ wgt_swz(k): the four rows one transposing read touches spread over
// different banks.
__device__ __forceinline__ int wgt_swz(int k) { return (k & 3) * 5; }

struct StreamTile {
    u32x4 rA, rB;              // producer descriptors (range 0 for a tile outside the grid)
    int64_t d_off;             // element offset of the tile's first output
    int64_t rows_left;         // valid token rows from the tile's first row (<= 0: none)
    int cols_left;             // valid columns of the tile (a group may end inside it; 0: none)
    int a_off;                 // basis window start of the tile's group
    int j_lo;                  // first identity-slice column the tile needs
    int rel_blk0;              // slice column of the first 32-column block of the calling wave's part
};

// WT x WN waves share the 256 x 256 tile: 2 x 2 waves of 128 x 128 (one wave per SIMD) or 2 x 4 waves
// of 128 tokens x 64 columns (two waves per SIMD, so that one wave's LDS reads, barrier wait and
// address arithmetic overlap the other's MFMAs).
//
// SK = contraction length of one stage (32 or 64), NS = LDS stages (a power of two); loads run
// NS - 1 stages ahead of the MFMAs.
//
// Host contract: p.n_stage_id = identity stages per tile (the same for every tile of a launch),
// stages per tile S = ceil(K / SK) + n_stage_id >= NS; grid = 8 * sm * sn workgroups;
// dynamic LDS = NS * (256 * 2 SK + SK * 512) + 4096 * waves.
template <typename X, typename OutT, int WT, int WN, int SK, int NS>
__global__ __launch_bounds__(64 * WT * WN) void gemm_stream_kernel(const GemmArgs p)
{
    constexpr int kStageK = SK, kStages = NS, kAhead = NS - 1;
    constexpr int NW = WT * WN;
    constexpr int TT = 8 / WT, TN = 8 / WN;
    constexpr int BT = 256, BN = 256;
    constexpr int PR = SK / 8;                         // 16-byte pieces per token row
    constexpr int RB = SK * 2;                         // bytes per token row in LDS
    constexpr int RPI = 64 / PR;                       // token rows per load instruction
    constexpr int KS = SK / 16;                        // k-steps per stage
    constexpr int PIT = BT / RPI / NW;                 // token load instructions per wave per stage
    constexpr int PIW = SK / 2 / NW;                   // weight load instructions per wave per stage
    constexpr int TOK_BYTES = BT * RB;
    constexpr int STAGE_BYTES = TOK_BYTES + SK * BN * 2;
    constexpr int LOADS = PIT + PIW;                   // per thread per stage
    constexpr int STORES = TT * TN * (sizeof(OutT) == 4 ? 4 : 2);   // 16-byte stores per thread per tile
    constexpr int WAIT_STEADY = (NS - 2) * LOADS;      // the younger stages may stay in flight
    constexpr int WAIT_AFTER_STORES = WAIT_STEADY + STORES < 63 ? WAIT_STEADY + STORES : 63;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // The scalar kernel arguments are fetched here in one batch and made opaque, so that they live in
    // registers; otherwise each use re-fetches its argument from memory and the per-tile set-up
    // becomes a chain of dependent scalar loads.
    struct {
        const void *A, *B; void* D;
        int64_t lda, ldb, ldd, M;
        int K, n_groups, d_h, a_skip, ident, m_tiles, n_tiles, sm, sn, n_stage_id, n_super_m, n_super_n, sn_shift;
        uint64_t dh_magic;
        int ts1, ts2, rounds, xq0, xr0, xcount;
    } q = {p.A, p.B, p.D, p.lda, p.ldb, p.ldd, p.M, p.K, p.n_groups, p.d_h, p.a_skip, p.ident, p.m_tiles, p.n_tiles,
           p.sm, p.sn, p.n_stage_id, p.n_super_m, p.n_super_n, p.sn_shift, p.dh_magic, p.tile_start[1], p.tile_start[2],
           p.rounds, p.xcd_q0[blockIdx.x % kNumXcd], p.xcd_r0[blockIdx.x % kNumXcd], p.xcd_count[blockIdx.x % kNumXcd]};
    asm volatile("" : "+s"(q.A), "+s"(q.B), "+s"(q.D), "+s"(q.lda), "+s"(q.ldb), "+s"(q.ldd), "+s"(q.M), "+s"(q.dh_magic));
    asm volatile("" : "+s"(q.K), "+s"(q.n_groups), "+s"(q.d_h), "+s"(q.a_skip), "+s"(q.ident), "+s"(q.m_tiles), "+s"(q.n_tiles),
                 "+s"(q.sm), "+s"(q.sn), "+s"(q.n_stage_id), "+s"(q.n_super_m), "+s"(q.n_super_n), "+s"(q.sn_shift),
                 "+s"(q.ts1), "+s"(q.ts2), "+s"(q.rounds), "+s"(q.xq0), "+s"(q.xr0), "+s"(q.xcount));

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave / WN, wn = wave % WN;
    const int l31 = lane & 31, lhi = lane >> 5;

    const int nk = (q.K + kStageK - 1) / kStageK;
    const int n_id = q.ident ? q.n_stage_id : 0;
    const int S = nk + n_id;
    const int xcd = blockIdx.x % kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    const int slot_m = slot >> q.sn_shift, slot_n = slot & (q.sn - 1);
    // x % d_h for 0 <= x < 2^24, d_h < 2^16: floor(x M / 2^40) with M = ceil(2^40 / d_h) is exact
    auto mod_dh = [&](int x) { return x - (int)(((uint64_t)(uint32_t)x * q.dh_magic) >> 40) * q.d_h; };

    // ---- tile set-up (scalar) -----------------------------------------------------------------------
    // Super-tiles (sm x sn tiles) are numbered down the token dimension first; die x works through
    // the numbers [x R, (x + 1) R), R = rounds.  A workgroup keeps its slot inside the super-tile, so
    // from one round to the next it usually moves down by sm token tiles and keeps its columns: the
    // die's L2 keeps the sn weight tiles and only the token tiles stream, and the column half of the
    // set-up (group lookup, weight descriptor) is done only when the column changes.
    const int n_rounds = q.rounds;
    int su_q = q.xq0, su_r = q.xr0, su_left = q.xcount;
    struct { u32x4 rB; int64_t n0; int cols_left, a_off, j_lo, rel_blk0; bool ok; } col;
    bool col_dirty = true;
    auto setup_cols = [&]() {
        const int nt = su_r * q.sn + slot_n;
        col.ok = nt < q.n_tiles;
        int g = 0;
        if (q.n_groups <= 2) g = (q.n_groups == 2 && nt >= q.ts1) ? 1 : 0;
        else if (nt >= q.ts1) { g = 1; while (g + 1 < q.n_groups && nt >= p.tile_start[g + 1]) ++g; }
        const int rel0 = col.ok ? (nt - p.tile_start[g]) * BN : 0;
        col.n0 = col.ok ? p.col_start[g] + rel0 : 0;
        const int64_t left = p.col_start[g + 1] - col.n0;
        col.cols_left = col.ok ? (int)(left > BN ? BN : left) : 0;
        col.a_off = p.a_off[g];
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
        --su_left;
        col_dirty = false;
        if (++su_q == q.n_super_m) { su_q = 0; ++su_r; col_dirty = true; }
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

    // producer, token tile: load j of wave w fills LDS rows RPI (w PIT + j) + lane/PR, position lane%PR
    // with the piece (lane%PR) ^ swizzle(row) of that row; weight tile: load j of wave w fills k rows
    // 2 (w PIW + j) + lane/32, position lane%32 with piece (lane%32) ^ swizzle(k).
    // Plain vector offset = byte offset of this lane's piece for a stage that starts at column 0 /
    // row 0; the stage's own offset is uniform and travels in the load's scalar offset, so that a
    // stage costs no vector arithmetic.  (The range check sees the vector part, which holds the whole
    // row term: rows past the end of the tensor stay out of range.)
    const uint32_t tok_row_bytes = (uint32_t)(q.lda * 2);
    const uint32_t wgt_row_bytes = (uint32_t)(q.ldb * 2);
    auto tok_k8 = [&](int ln, int j) { return ((ln % PR) ^ tok_swz<SK>((ln / PR + RPI * j) & 15)) * 8; };
    auto wgt_c = [&](int ln, int j) { return (ln & 31) ^ wgt_swz(2 * j + (ln >> 5)); };
    // vo_tok[j], vo_wgt[j]: vector offsets of the next stage to request.  Between plain stages they
    // do not change; a stage that needs per-lane decisions overwrites them and the next plain stage
    // restores them (vo_is_plain tells which).
    uint32_t vo_tok[PIT], vo_wgt[PIW];
    bool vo_is_plain = true;
    auto plain_offsets = [&](int ln) {
#pragma unroll
        for (int j = 0; j < PIT; ++j)
            vo_tok[j] = (uint32_t)(wave * (RPI * PIT) + ln / PR + RPI * j) * tok_row_bytes + (uint32_t)tok_k8(ln, j & 1) * 2u;
#pragma unroll
        for (int j = 0; j < PIW; ++j)
            vo_wgt[j] = (uint32_t)(wave * (2 * PIW) + (ln >> 5)) * wgt_row_bytes + (uint32_t)wgt_c(ln, j & 1) * 16u;
    };
    plain_offsets(lane);
    static_assert((RPI * PIT) % 16 == 0 && (2 * PIW) % 4 == 0, "per-wave row blocks must keep the swizzle phase");

    // consumer, token fragments: row = wt*32*TT + ti*32 + l31, piece q = 2 ks + lhi
    // piece (2 ks + lhi) ^ swz = ((lhi ^ swz) ^ (ks << 1)): k-step ks is the k-step 0 address with bit 5 + ... flipped
    const uint32_t c_tok0 = (uint32_t)((wt * (32 * TT) + l31) * RB + ((lhi ^ tok_swz<SK>(l31 & 15)) << 4));
    // consumer, weight fragments (transposing read): 16-lane group gq = lane/16, s = lane%16:
    // k = 16 ks + 8 lhi + 4 rd + s/4, columns wn*32*TN + ni*32 + 16 (gq&1) + 4 (s&3) .. +3
    const int c_s = lane & 15, c_gq = lane >> 4;
    uint32_t c_wgt[TN];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
        const int col = wn * (32 * TN) + ni * 32 + 16 * (c_gq & 1) + 4 * (c_s & 3);
        const int piece = (col >> 3) ^ wgt_swz(c_s >> 2);
        c_wgt[ni] = (uint32_t)(TOK_BYTES + (8 * lhi + (c_s >> 2)) * 512 + (piece << 4) + ((col & 4) << 1));
    }

    // ---- producer: stage `k` of tile `t` into LDS slot `g & 3` -------------------------------------
    // Always issues LOADS loads per thread; whatever has nothing to fetch (weights of an identity
    // stage, columns past the group's end, a tile outside the grid) uses an out-of-range offset.
    auto general_offsets = [&](const StreamTile& t, int k) {
        int ln = lane;                        // per-lane terms rebuilt here: this path is rare
        asm volatile("" : "+v"(ln));
        plain_offsets(ln);
#pragma unroll
        for (int j = 0; j < PIT; ++j) {
            const int k8 = tok_k8(ln, j & 1);
            int col, lim_ok;
            if (k < nk) {
                const int kk = k * SK + k8;
                col = kk < t.a_off ? kk : kk + q.a_skip;
                lim_ok = kk < q.K;
            } else {
                const int jc = t.j_lo + (k - nk) * SK + k8;
                col = t.a_off + jc;
                lim_ok = jc < q.d_h;
            }
            vo_tok[j] = lim_ok ? vo_tok[j] + (uint32_t)(col - k8) * 2u : kBadOffset;
        }
#pragma unroll
        for (int j = 0; j < PIW; ++j)
            vo_wgt[j] = (k < nk && wgt_c(ln, j & 1) * 8 < t.cols_left)
                            ? vo_wgt[j] + (uint32_t)(k * SK + 2 * j) * wgt_row_bytes : kBadOffset;
    };
    // vector offsets for stage k of tile t (uniform branches only)
    auto prepare_offsets = [&](bool plain, const StreamTile& t, int k) {
        if (!plain) {
            general_offsets(t, k);
            vo_is_plain = false;
        } else if (!vo_is_plain) {
            int ln = lane;
            asm volatile("" : "+v"(ln));
            plain_offsets(ln);
            vo_is_plain = true;
        }
    };
    // A stage whose pieces all exist (full 256 columns, no window edge and no end of K or of the
    // identity slice inside it) needs no per-lane decisions: uniform offsets only.
    auto stage_is_plain = [&](const StreamTile& t, int k) -> bool {
        if (t.cols_left != BN) return false;
        if (k < nk) {
            const int k0 = k * SK;
            return k0 + SK <= q.K && (k0 + SK <= t.a_off || k0 >= t.a_off);
        }
        return t.j_lo + (k - nk + 1) * SK <= q.d_h;
    };
    // Uniform part of the addresses of stage k of tile t, and which form applies.
    struct StageOff { bool plain; uint32_t tok_soff, wgt_soff; u32x4 rB; };
    auto stage_offsets = [&](const StreamTile& t, int k) -> StageOff {
        StageOff o;
        o.plain = stage_is_plain(t, k);
        const int k0 = k * SK;
        const uint32_t colb = k < nk ? (uint32_t)(k0 < t.a_off ? k0 : k0 + q.a_skip) : (uint32_t)(t.a_off + t.j_lo + (k - nk) * SK);
        o.tok_soff = o.plain ? colb * 2u : 0u;
        o.wgt_soff = (o.plain && k < nk) ? (uint32_t)k0 * wgt_row_bytes : 0u;
        o.rB = t.rB;
        if (o.plain && k >= nk) o.rB[2] = 0;  // identity stage: the weight slot is filled with zeros
        return o;
    };
    // load j (0 .. LOADS-1) of the stage whose vector offsets prepare_offsets has set
    auto issue_load = [&](const StreamTile& t, const StageOff& o, int g, int j) {
        const uint32_t lds_slot = (uint32_t)((g & (kStages - 1)) * STAGE_BYTES);
        if (j < PIT) {
            lds_dma1s(t.rA, lds_slot + (uint32_t)wave * (1024u * PIT) + 1024u * j, vo_tok[j < PIT ? j : 0], o.tok_soff);
        } else {
            const int jj = j >= PIT ? j - PIT : 0;
            lds_dma1s(o.rB, lds_slot + (uint32_t)TOK_BYTES + (uint32_t)wave * (1024u * PIW) + 1024u * jj, vo_wgt[jj],
                      o.plain ? o.wgt_soff + (uint32_t)(2 * jj) * wgt_row_bytes : 0u);
        }
    };
    auto produce = [&](const StreamTile& t, int k, int g) {
        const StageOff o = stage_offsets(t, k);
        prepare_offsets(o.plain, t, k);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) issue_load(t, o, g, j);
    };

    // ---- consumer ---------------------------------------------------------------------------------
    // Each stage is two k-steps of 16.  The fragments of a k-step are read from LDS one k-step
    // before its MFMAs are issued (two register sets), so within a wave the LDS latency, the
    // barrier, the producer's address arithmetic and the DMA issue sit behind queued MFMAs:
    //     read(stage i, k-step 1) | MFMA(stage i, k-step 0) | wait + barrier + produce(stage i + 4)
    //     | read(stage i + 1, k-step 0) | MFMA(stage i, k-step 1) | ...
    auto mm = [](u32x4 a, u32x4 b, f32x16 c) -> f32x16 { return X::mfma(a, b, c); };
    f32x16 acc[TN][TT];
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    u32x4 fw0[TN], ft0[TT], fw1[TN], ft1[TT];

    auto read_w = [&](uint32_t sbase, int ks, u32x4 (&fw)[TN]) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + sbase + c_wgt[ni] + (16 * ks) * 512));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + sbase + c_wgt[ni] + (16 * ks + 4) * 512));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            fw[ni] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
        }
    };
    auto read_t = [&](uint32_t sbase, int ks, u32x4 (&ft)[TT]) {
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) ft[ti] = *(const u32x4*)(smem + ((sbase + c_tok0) ^ (uint32_t)(ks << 5)) + ti * (32 * RB));
    };
    auto mma_regular = [&](const u32x4 (&fw)[TN], const u32x4 (&ft)[TT]) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(fw[ni], ft[ti], acc[ni][ti]);
    };
    int rel_blk[TN] = {};                     // slice column of each 32-column block of this wave's tile part
    auto mma_identity = [&](const u32x4 (&idf)[2], int col0, const u32x4 (&ft)[TT]) {
        // col0: first of the 16 slice columns this k-step holds
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const int d = col0 - rel_blk[ni];
            if (d == 0 || d == 16) {
                const u32x4 f = d == 0 ? idf[0] : idf[1];
#pragma unroll
                for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(f, ft[ti], acc[ni][ti]);
            }
        }
    };
    // the same products with this stage's loads j0 .. j0 + n - 1 issued between them, so that the
    // address unit sees a steady trickle instead of every wave's loads at once
    auto mma_regular_loads = [&](const u32x4 (&fw)[TN], const u32x4 (&ft)[TT], const StreamTile& pt, const StageOff& so, int g, int j0) {
        constexpr int NL = LOADS / 2, EVERY = (TN * TT) / NL > 0 ? (TN * TT) / NL : 1;
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
                acc[ni][ti] = mm(fw[ni], ft[ti], acc[ni][ti]);
                const int m = ni * TT + ti;
                if (m % EVERY == EVERY - 1 && m / EVERY < NL) {
                    __builtin_amdgcn_sched_barrier(0);
                    issue_load(pt, so, g, j0 + m / EVERY);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        static_assert(NL <= TN * TT, "more loads than products in a k-step");
    };
    auto slot_base = [&](int g) { return (uint32_t)((g & (kStages - 1)) * STAGE_BYTES); };
    auto clear_acc = [&]() {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = zero16;
    };

    // One stage of the consumer's tile `cur` (stage kc, global stage counter g), during which stage
    // `pk` of tile `pt` is loaded.  `regular`: compile-time kind of the stage (rows of B, or a piece
    // of the identity slice).  `relaxed`: an epilogue's stores may still be in flight.
    auto stage = [&](auto regular, const StreamTile& cur, int kc, int g, const StreamTile& pt, int pk, bool relaxed) {
        constexpr bool REG = decltype(regular)::value;
        const uint32_t sb = slot_base(g), nb = slot_base(g + 1);
        const bool next_regular = kc + 1 < nk || kc + 1 == S;
        const int jc = cur.j_lo + (kc - nk) * SK;
        u32x4 idf[2];
        if constexpr (!REG) make_idf(idf);
        static_assert(KS % 2 == 0, "fragment sets alternate");
        // addresses of the stage requested after this stage's barrier: worked out here, behind the
        // MFMAs of the first k-steps, so that nothing but the loads themselves follows the barrier
        const StageOff so = stage_offsets(pt, pk);
        prepare_offsets(so.plain, pt, pk);
#pragma unroll
        for (int ks = 0; ks + 2 < KS; ++ks) {
            if (ks % 2 == 0) {
                if constexpr (REG) { read_w(sb, ks + 1, fw1); read_t(sb, ks + 1, ft1); mma_regular(fw0, ft0); }
                else { read_t(sb, ks + 1, ft1); mma_identity(idf, jc + 16 * ks, ft0); }
            } else {
                if constexpr (REG) { read_w(sb, ks + 1, fw0); read_t(sb, ks + 1, ft0); mma_regular(fw1, ft1); }
                else { read_t(sb, ks + 1, ft0); mma_identity(idf, jc + 16 * ks, ft1); }
            }
        }
        // last read of this stage's slot, then the slot is free once every wave is here
        if constexpr (REG) read_w(sb, KS - 1, fw1);
        read_t(sb, KS - 1, ft1);
        if (relaxed) wait_vmcnt<WAIT_AFTER_STORES>(); else wait_vmcnt<WAIT_STEADY>();
        __syncthreads();
        if constexpr (REG) mma_regular_loads(fw0, ft0, pt, so, g, 0);
        else {
            mma_identity(idf, jc + 16 * (KS - 2), ft0);
#pragma unroll
            for (int j = 0; j < LOADS / 2; ++j) issue_load(pt, so, g, j);
        }
        if (next_regular) read_w(nb, 0, fw0);
        read_t(nb, 0, ft0);
        if constexpr (REG) mma_regular_loads(fw1, ft1, pt, so, g, LOADS / 2);
        else {
            mma_identity(idf, jc + 16 * (KS - 1), ft1);
#pragma unroll
            for (int j = LOADS / 2; j < LOADS; ++j) issue_load(pt, so, g, j);
        }
    };

    StreamTile cur = setup();
    bool prev_full = true;                    // did the previous tile issue all its result stores?
    int g = 0;
    // prologue: the first kStages stages of the first tile
#pragma unroll 1
    for (int k = 0; k < kStages; ++k) {
        produce(cur, k, k);
        if (k == 0) __builtin_amdgcn_s_barrier();   // the first stage of all waves goes ahead of everything else
    }
    clear_acc();
    wait_vmcnt<(kStages - 1) * LOADS>();
    __syncthreads();
    read_w(slot_base(0), 0, fw0);
    read_t(slot_base(0), 0, ft0);

    const std::true_type REGULAR{};
    const std::false_type IDENTITY{};
    const int split = S - kStages;            // from this stage on, the next tile is being loaded
    const int r_same = nk < split ? nk : split;
    const int i_same = split > nk ? split : nk;
#pragma unroll 1
    for (int round = 0; round < n_rounds; ++round) {
        const StreamTile nxt = setup();
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {      // d_h >= 32 is a multiple of 32 and rel_blk0 < d_h
            rel_blk[ni] = cur.rel_blk0 + 32 * ni;
            if (rel_blk[ni] >= q.d_h) rel_blk[ni] -= q.d_h;
            if (rel_blk[ni] >= q.d_h) rel_blk[ni] -= q.d_h;
        }
        // The relaxed wait counts on all STORES result stores of the previous tile being in flight
        // behind the loads it waits for; a tile that a group's end cut short skipped some, so after
        // such a tile (and after a tile outside the grid, which stores nothing) the wait is the full one.
        const bool after_tile = round > 0 && prev_full;
        int kc = 0;
#pragma unroll 1
        for (; kc < r_same; ++kc, ++g) stage(REGULAR, cur, kc, g, cur, kc + kStages, after_tile && kc < (kAhead > 1 ? kAhead : 1));
#pragma unroll 1
        for (; kc < nk; ++kc, ++g) stage(REGULAR, cur, kc, g, nxt, kc - split, after_tile && kc < (kAhead > 1 ? kAhead : 1));
#pragma unroll 1
        for (; kc < i_same; ++kc, ++g) stage(IDENTITY, cur, kc, g, cur, kc + kStages, after_tile && kc < (kAhead > 1 ? kAhead : 1));
#pragma unroll 1
        for (; kc < S; ++kc, ++g) stage(IDENTITY, cur, kc, g, nxt, kc - split, after_tile && kc < (kAhead > 1 ? kAhead : 1));

        // ---- epilogue ---------------------------------------------------------------------------
        // rows past the end of the tensor and tiles outside the grid fall outside rD's range
        const __amdgpu_buffer_rsrc_t rD = make_rsrc(
            (char*)q.D + cur.d_off * (int64_t)sizeof(OutT),
            cur.cols_left > 0 ? ((cur.rows_left - 1) * q.ldd + cur.cols_left) * (int64_t)sizeof(OutT) : 0);
        const bool full = cur.cols_left == BN;      // uniform; a group may end inside its last tile
        prev_full = full;
        if constexpr (sizeof(OutT) == 4) {
            // float32 results: a lane holds runs of 4 consecutive columns (16 bytes) of one row, lanes l and
            // l+32 adjacent runs.  Stored as they are, an instruction would write 32 bytes of each of 32
            // rows, which the memory pipeline takes at a third of its rate; so a 32-row x 32-column block
            // (4 KiB) is turned round in the wave's staging region, as below for the 16-bit types, and 8
            // consecutive lanes store one full 128-byte line of a row.
            unsigned char* stag = smem + kStages * STAGE_BYTES + wave * 4096;
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
                        const bool ok = full || wn * (32 * TN) + ni * 32 + rd_chunk * 4 < cur.cols_left;
                        if (ok) __builtin_amdgcn_raw_buffer_store_b128(v, rD, off, ni * 128, kStreamStoreAux);
                    }
                }
            }
        } else {
            // lanes l and l+32 hold columns 0..3 and 4..7 of the same 8-column block; after the swap
            // the lower half-wave owns the even blocks and the upper half-wave the odd blocks, each
            // lane with 8 consecutive columns = 16 bytes.  A 32-row x 64-column piece is then turned
            // round in a 4 KiB LDS region private to the wave, so that 8 consecutive lanes store one
            // full 128-byte line of a row (the memory pipeline works on whole lines).
            unsigned char* stag = smem + kStages * STAGE_BYTES + wave * 4096;
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
                        const bool ok = full || wn * (32 * TN) + h * 64 + rd_chunk * 8 < cur.cols_left;
                        if (ok) __builtin_amdgcn_raw_buffer_store_b128(v, rD, off, h * 128, kStreamStoreAux);
                    }
                }
            }
        }
        clear_acc();
        cur = nxt;
    }
    wait_vmcnt<0>();
}

}  // namespace bda
