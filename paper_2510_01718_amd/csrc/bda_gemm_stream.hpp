// Streaming MFMA GEMM for gfx950: the large-T kernel of libbda.
//
//   D[t, n] = ident(t, n) + sum_{k < K} A[t, acol_g(k)] * B[k, n]        (see bda_gemm_kernels.hpp)
//
// What is different from the register-staged kernel in bda_gemm_kernels.hpp:
//   * Global -> LDS copies never touch registers: every 16-byte piece is moved by
//     buffer_load_dwordx4 ... lds (LDS DMA).  The token tile lands k-contiguous, the weight tile
//     n-contiguous exactly as it lies in memory; the weight fragments are then read with the
//     transposing LDS read ds_read_b64_tr_b16, so no shuffling instructions are spent on them.
//   * The contraction is cut into stages of 32 and the LDS holds four stages.  Loads run three
//     stages ahead of the MFMAs, and the stage sequence continues across output tiles: while the
//     last stages of one tile are multiplied and its results are stored, the first stages of the
//     workgroup's next tile are already in flight.  One barrier per stage.
//   * Bank conflicts are avoided by permuting which 16-byte piece each lane of a load fetches (the
//     LDS image of one load instruction is always lane-linear), so the tiles need no padding.
//   * 16-bit results are exchanged between the two half-waves (v_permlane32_swap) so that every
//     lane stores 16 contiguous bytes.
//
// The LDS DMA loads are issued from inline assembly: the compiler would otherwise wait for ALL
// outstanding loads before any LDS read, which would serialise the stages.  Their completion is
// tracked by hand with s_waitcnt vmcnt(n); every wave issues the same number of loads per stage
// (loads that have nothing to fetch use an out-of-range offset and return zeros).
#pragma once
#include "bda_gemm_kernels.hpp"

namespace bda {

constexpr int kStageK = 32;          // contraction length of one stage
constexpr int kStages = 4;           // LDS stages
constexpr int kAhead = kStages - 1;  // stages in flight ahead of the MFMAs

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt = [15:14|3:0]).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Four LDS DMA loads of 16 bytes per lane through one descriptor; the LDS image of load j starts at
// lds_base + 1024 j and is lane-linear (lane l -> bytes [16 l, 16 l + 16)).  The LDS address of such a
// load is M0 + instruction offset + 16 lane, and the instruction offset would also be added to the
// global address, so M0 is advanced instead.
__device__ __forceinline__ void lds_dma4(u32x4 rsrc, uint32_t lds_base, uint32_t v0, uint32_t v1,
                                         uint32_t v2, uint32_t v3)
{
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %5, 0 offen lds\n\t"
        "s_add_u32 m0, m0, 0x400\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %2, %5, 0 offen lds\n\t"
        "s_add_u32 m0, m0, 0x400\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %3, %5, 0 offen lds\n\t"
        "s_add_u32 m0, m0, 0x400\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %4, %5, 0 offen lds\n\t"
        :
        : "s"(lds_base), "v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(rsrc)
        : "memory", "m0", "scc");
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

// Token tile in LDS: row = 32 k = 64 bytes = four 16-byte pieces; piece q of row r sits at position
// q ^ tok_swz(r).  Chosen so that the 32 lanes of a fragment read (32 consecutive rows, same q) are
// conflict-free whether the LDS serves 16 lanes x 16 bytes over 64 banks or 8 lanes over 32 banks.
__device__ __forceinline__ int tok_swz(int r) { return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1); }
// Weight tile in LDS: row = one k = 256 columns = 512 bytes = thirty-two 16-byte pieces; piece c of
// row k sits at position c ^ wgt_swz(k): the four rows one transposing read touches spread over
// different banks.
__device__ __forceinline__ int wgt_swz(int k) { return (k & 3) * 5; }

struct TileInfo {
    int valid;
    int super;                 // super-tile index this tile came from (the iterator's position)
    int mt;                    // token tile
    int rel0;                  // first column of the tile inside its group
    int64_t n0;                // first output column of the tile
    int cols_left;             // valid columns of the tile (a group may end inside it)
    int a_off;                 // basis window start of the tile's group
    int j_lo, n_id, n_stage;   // identity slice start, identity stages, total stages
};

// DBG is for timing experiments only (0 in the library): bit 0 drops the result stores, bit 1 the
// MFMAs, bit 2 the global loads.
template <typename X, typename OutT, int DBG = 0>
__global__ __launch_bounds__(256) void gemm_stream_kernel(const GemmArgs p)
{
    constexpr int TT = 4, TN = 4;
    constexpr int BT = 256, BN = 256;
    constexpr int TOK_BYTES = BT * 64;                 // 16 KiB
    constexpr int STAGE_BYTES = TOK_BYTES + kStageK * BN * 2;   // 32 KiB
    constexpr int LOADS = 8;                           // per thread per stage: 4 token + 4 weight
    constexpr int STORES = sizeof(OutT) == 4 ? 64 : 32;   // 16-byte stores per thread per tile
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lhi = lane >> 5;

    const int nk = (p.K + kStageK - 1) / kStageK;
    const int n_super_n = (p.n_tiles + p.sn - 1) / p.sn;
    const int n_super_m = (p.m_tiles + p.sm - 1) / p.sm;
    const int total_super = n_super_m * n_super_n;
    const int slots = p.sm * p.sn;
    const int xcd = blockIdx.x % kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    if (slot >= slots) return;

    // ---- tile iterator ---------------------------------------------------------------------
    auto tile_at = [&](int s) -> TileInfo {
        TileInfo ti{};
        for (; s < total_super; s += kNumXcd) {
            const int mt = (s / n_super_n) * p.sm + slot / p.sn;
            const int nt = (s % n_super_n) * p.sn + slot % p.sn;
            if (mt < p.m_tiles && nt < p.n_tiles) {
                int g = 0;
                while (g + 1 < p.n_groups && nt >= p.tile_start[g + 1]) ++g;
                ti.valid = 1;
                ti.super = s;
                ti.mt = mt;
                ti.rel0 = (nt - p.tile_start[g]) * BN;
                ti.n0 = p.col_start[g] + ti.rel0;
                const int64_t left = p.col_start[g + 1] - ti.n0;
                ti.cols_left = (int)(left > BN ? BN : left);
                ti.a_off = p.a_off[g];
                if (p.ident) {
                    const bool nested = (p.d_h % BN) == 0;
                    ti.j_lo = nested ? ti.rel0 % p.d_h : 0;
                    ti.n_id = ((nested ? BN : p.d_h) + kStageK - 1) / kStageK;
                }
                ti.n_stage = nk + ti.n_id;
                return ti;
            }
        }
        return ti;
    };

    // ---- per-lane constants ------------------------------------------------------------------
    // identity fragments (row operand): lane (row i = l31, half lhi) holds k' = 16 v + 8 lhi + e
    u32x4 idf[2];
#pragma unroll
    for (int v = 0; v < 2; ++v)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int k0 = 16 * v + 8 * lhi + 2 * w;
            idf[v][w] = (k0 == l31 ? IdentityFrag<X>::one : 0u) | (k0 + 1 == l31 ? IdentityFrag<X>::one << 16 : 0u);
        }

    // producer, token tile: load j of wave w fills LDS rows w*64 + 16 j + lane/4, position lane%4
    const int p_tok_row = wave * 64 + (lane >> 2);
    const int p_tok_q = (lane & 3) ^ tok_swz(lane >> 2);          // rows differ by multiples of 16
    const uint32_t tok_row_bytes = (uint32_t)(p.lda * 2);
    // producer, weight tile: load j of wave w fills k rows w*8 + 2 j + lane/32, position lane%32
    const int p_wgt_k = wave * 8 + (lane >> 5);
    const uint32_t wgt_row_bytes = (uint32_t)(p.ldb * 2);
    int p_wgt_c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) p_wgt_c[j] = (lane & 31) ^ wgt_swz(2 * j + (lane >> 5));

    // consumer, token fragments: row = wt*128 + ti*32 + l31, piece q = 2 ks + lhi
    uint32_t c_tok[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
        c_tok[ks] = (uint32_t)((wt * 128 + l31) * 64 + (((2 * ks + lhi) ^ tok_swz(l31)) << 4));
    // consumer, weight fragments (transposing read): 16-lane group gq = lane/16, s = lane%16:
    // k = 16 ks + 8 lhi + 4 rd + s/4, columns wn*128 + ni*32 + 16 (gq&1) + 4 (s&3) .. +3
    const int c_s = lane & 15, c_gq = lane >> 4;
    uint32_t c_wgt[TN];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
        const int col = wn * 128 + ni * 32 + 16 * (c_gq & 1) + 4 * (c_s & 3);
        const int piece = (col >> 3) ^ wgt_swz(c_s >> 2);
        c_wgt[ni] = (uint32_t)(TOK_BYTES + (8 * lhi + (c_s >> 2)) * 512 + (piece << 4) + ((col & 4) << 1));
    }

    // ---- producer -------------------------------------------------------------------------------
    TileInfo pt = tile_at(xcd);
    int pk = 0;            // next stage of pt to load
    int pcount = 0;        // stages issued so far (LDS slot = pcount % kStages)
    u32x4 rA = {0, 0, 0, 0}, rB = {0, 0, 0, 0};
    auto producer_enter_tile = [&]() {
        if (pt.valid) {
            const int64_t t0 = (int64_t)pt.mt * BT;
            const int64_t rows_left = p.M - t0;
            rA = make_rsrc_words((const char*)p.A + t0 * p.lda * 2, ((rows_left - 1) * p.lda + p.K + p.a_skip) * 2);
            rB = make_rsrc_words((const char*)p.B + pt.n0 * 2, ((int64_t)(p.K - 1) * p.ldb + pt.cols_left) * 2);
        }
    };
    producer_enter_tile();
    auto produce = [&]() {
        // always issues LOADS loads per thread (out-of-range ones return zeros) while a tile is left
        const uint32_t lds_slot = (uint32_t)((pcount % kStages) * STAGE_BYTES);
        uint32_t tv[4], wv[4];
        if (pk < nk) {
            const int k = pk * kStageK + p_tok_q * 8;
            const int col = k < pt.a_off ? k : k + p.a_skip;
            const uint32_t base = k < p.K ? (uint32_t)p_tok_row * tok_row_bytes + (uint32_t)col * 2u : kBadOffset;
#pragma unroll
            for (int j = 0; j < 4; ++j) tv[j] = base + (uint32_t)(16 * j) * tok_row_bytes;
            const uint32_t kbase = (uint32_t)(pk * kStageK + p_wgt_k) * wgt_row_bytes;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                wv[j] = p_wgt_c[j] * 8 < pt.cols_left ? kbase + (uint32_t)(2 * j) * wgt_row_bytes + (uint32_t)p_wgt_c[j] * 16u
                                                       : kBadOffset;
        } else {
            const int jcol = pt.j_lo + (pk - nk) * kStageK + p_tok_q * 8;
            const uint32_t base = jcol < p.d_h ? (uint32_t)p_tok_row * tok_row_bytes + (uint32_t)(pt.a_off + jcol) * 2u : kBadOffset;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                tv[j] = base + (uint32_t)(16 * j) * tok_row_bytes;
                wv[j] = kBadOffset;
            }
        }
        if constexpr (!(DBG & 4)) {
            lds_dma4(rA, lds_slot + (uint32_t)wave * 4096u, tv[0], tv[1], tv[2], tv[3]);
            lds_dma4(rB, lds_slot + (uint32_t)TOK_BYTES + (uint32_t)wave * 4096u, wv[0], wv[1], wv[2], wv[3]);
        }
        ++pcount;
        if (++pk == pt.n_stage) {
            pt = tile_at(pt.super + kNumXcd);
            pk = 0;
            producer_enter_tile();
        }
    };

    // prologue: kAhead stages in flight
    int issued_real = 0;
#pragma unroll 1
    for (int i = 0; i < kAhead; ++i) {
        if (pt.valid) {
            produce();
            ++issued_real;
        }
    }

    // ---- consumer -------------------------------------------------------------------------------
    TileInfo ct = tile_at(xcd);
    int ccount = 0;
    int since_store = 100;     // stages consumed since the last epilogue (its stores sit in vmcnt too)
    auto mm = [](u32x4 a, u32x4 b, f32x16 c) -> f32x16 {
        if constexpr (DBG & 2) {
            c[0] += __builtin_bit_cast(float, a[0] ^ b[0]);     // keeps the operands alive
            return c;
        } else {
            return X::mfma(a, b, c);
        }
    };
    f32x16 acc[TN][TT];
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;

    // waits until stage `ccount` has landed in LDS for every wave, then refills the slot that has
    // just been read.  Younger operations may stay in flight: the loads of the stages behind it
    // and, shortly after an epilogue, that epilogue's stores (they count in vmcnt as well).
    auto stage_begin = [&]() {
        if (!pt.valid) {
            wait_vmcnt<0>();
        } else if (since_store < kAhead) {
            wait_vmcnt<(kAhead - 1) * LOADS + STORES < 63 ? (kAhead - 1) * LOADS + STORES : 63>();
        } else {
            wait_vmcnt<(kAhead - 1) * LOADS>();
        }
        __syncthreads();
        if (pt.valid) produce();
        ++since_store;
    };
    auto load_frags = [&](uint32_t sbase, int ks, u32x4 (&fw)[TN], u32x4 (&ft)[TT]) {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + sbase + c_wgt[ni] + (16 * ks) * 512));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + sbase + c_wgt[ni] + (16 * ks + 4) * 512));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            fw[ni] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
        }
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) ft[ti] = *(const u32x4*)(smem + sbase + c_tok[ks] + ti * 2048);
    };

    while (ct.valid) {
        const int rel_wave = (ct.rel0 + wn * (32 * TN)) % (p.d_h > 0 ? p.d_h : 1);

        // first stage of the tile: its first k-step starts the accumulators from zero (the zero is
        // an operand of the MFMA, no register is cleared)
        {
            stage_begin();
            const uint32_t sbase = (uint32_t)((ccount % kStages) * STAGE_BYTES);
            u32x4 fw[TN], ft[TT];
            load_frags(sbase, 0, fw, ft);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(fw[ni], ft[ti], zero16);
            load_frags(sbase, 1, fw, ft);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(fw[ni], ft[ti], acc[ni][ti]);
            ++ccount;
        }
#pragma unroll 1
        for (int kc = 1; kc < nk; ++kc) {
            stage_begin();
            const uint32_t sbase = (uint32_t)((ccount % kStages) * STAGE_BYTES);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u32x4 fw[TN], ft[TT];
                load_frags(sbase, ks, fw, ft);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                    for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(fw[ni], ft[ti], acc[ni][ti]);
            }
            ++ccount;
        }
#pragma unroll 1
        for (int kc = nk; kc < ct.n_stage; ++kc) {
            stage_begin();
            const uint32_t sbase = (uint32_t)((ccount % kStages) * STAGE_BYTES);
            const int jc = ct.j_lo + (kc - nk) * kStageK;     // first slice column of this stage
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u32x4 ft[TT];
#pragma unroll
                for (int ti = 0; ti < TT; ++ti) ft[ti] = *(const u32x4*)(smem + sbase + c_tok[ks] + ti * 2048);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    const int d = jc + 16 * ks - (rel_wave + 32 * ni) % p.d_h;
                    if (d == 0 || d == 16) {
                        const u32x4 f = d == 0 ? idf[0] : idf[1];
#pragma unroll
                        for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = mm(f, ft[ti], acc[ni][ti]);
                    }
                }
            }
            ++ccount;
        }

        // ---- epilogue ---------------------------------------------------------------------------
        const int64_t ct0 = (int64_t)ct.mt * BT;
        const int64_t rows_left = p.M - ct0;
        const __amdgpu_buffer_rsrc_t rD = make_rsrc(
            (char*)p.D + (ct0 * p.ldd + ct.n0) * (int64_t)sizeof(OutT),
            ((rows_left - 1) * p.ldd + ct.cols_left) * (int64_t)sizeof(OutT));
        const uint32_t ep_row_step = 32u * (uint32_t)(p.ldd * sizeof(OutT));
        const bool full = ct.cols_left == BN;      // uniform; a group may end inside its last tile
        if constexpr (DBG & 1) {
            float sum = 0.f;
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int ti = 0; ti < TT; ++ti)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum += acc[ni][ti][r];
            if (sum == 12345.678f) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, sum), rD, 0, 0, 0);
        } else if constexpr (sizeof(OutT) == 4) {
            uint32_t ep_row = (uint32_t)(wt * (32 * TT) + l31) * (uint32_t)(p.ldd * 4) + (uint32_t)(wn * (32 * TN) + lhi * 4) * 4u;
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
                if (ti) ep_row += ep_row_step;
                asm volatile("" : "+v"(ep_row));
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int c0 = ni * 32 + rg * 8;
                        if (!full && wn * (32 * TN) + c0 >= ct.cols_left) continue;
                        const float e0 = acc[ni][ti][rg * 4 + 0], e1 = acc[ni][ti][rg * 4 + 1];
                        const float e2 = acc[ni][ti][rg * 4 + 2], e3 = acc[ni][ti][rg * 4 + 3];
                        const f32x4 vf = {e0, e1, e2, e3};
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vf), rD, ep_row, c0 * 4, 0);
                    }
                }
            }
        } else {
            // lanes l and l+32 hold columns 0..3 and 4..7 of the same 8-column block; after the swap
            // the lower half-wave owns the even blocks and the upper half-wave the odd blocks, each
            // lane with 8 consecutive columns = 16 bytes
            uint32_t ep_row = (uint32_t)(wt * (32 * TT) + l31) * (uint32_t)(p.ldd * 2) + (uint32_t)(wn * (32 * TN) + lhi * 8) * 2u;
#pragma unroll
            for (int ti = 0; ti < TT; ++ti) {
                if (ti) ep_row += ep_row_step;
                asm volatile("" : "+v"(ep_row));    // keeps the offset a per-tile value (one register)
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr) {
                        uint32_t xv[2], yv[2];
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            xv[h] = (uint32_t)X::from_f32(acc[ni][ti][(2 * pr) * 4 + 2 * h]) |
                                    ((uint32_t)X::from_f32(acc[ni][ti][(2 * pr) * 4 + 2 * h + 1]) << 16);
                            yv[h] = (uint32_t)X::from_f32(acc[ni][ti][(2 * pr + 1) * 4 + 2 * h]) |
                                    ((uint32_t)X::from_f32(acc[ni][ti][(2 * pr + 1) * 4 + 2 * h + 1]) << 16);
                        }
                        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(xv[0], yv[0], false, false);
                        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(xv[1], yv[1], false, false);
                        const int c0 = ni * 32 + pr * 16;           // this pair's two 8-column blocks
                        const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
                        // the column offset is a compile-time constant: it travels in the
                        // instruction's scalar-offset operand, not in a register per store
                        if (full) {
                            __builtin_amdgcn_raw_buffer_store_b128(v, rD, ep_row, c0 * 2, 0);
                        } else if (wn * (32 * TN) + c0 + lhi * 8 < ct.cols_left) {
                            __builtin_amdgcn_raw_buffer_store_b128(v, rD, ep_row, c0 * 2, 0);
                        }
                    }
                }
            }
        }
        since_store = 0;
        ct = tile_at(ct.super + kNumXcd);
    }
    wait_vmcnt<0>();
}

}  // namespace bda
