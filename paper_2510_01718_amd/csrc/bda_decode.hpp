// Small-T ("decode") kernel of libbda for gfx950: T <= 128 tokens (NTB blocks of 32 token rows per
// workgroup: 1 for T <= 32, 2 for T <= 64, 4 above).
//
// With a handful of tokens the projection is a stream over the weights: every element of C is read
// exactly once and used for at most 128 multiply-adds, so the kernel is organised around that read
// (bandwidth / latency bound), not around MFMA occupancy:
//   * one workgroup per 32-column slice of the output, all K rows of it: its part of C
//     (K x 64 bytes) goes global -> LDS in one burst of LDS DMA loads, which are the first thing the
//     kernel issues (all arguments and group tables come in one batch of scalar loads; token
//     fragments and identity values are requested while C is on its way);
//   * slices are handed out so that neighbouring slices (which share 128-byte lines of C) run on
//     the same die and meet in its L2;
//   * the four waves split the k-steps; their partial sums are added in a fixed order through LDS,
//     so the result does not depend on scheduling;
//   * the token fragments come straight from global memory in MFMA operand layout (a row of the
//     latent is k-contiguous) or, for 33 .. 64 tokens, through LDS; the identity slice is added in
//     float32 after the reduction.
// A second kernel at the end of this file gives a workgroup 128 columns, for wide outputs.
// Both also read C in the packed layout of bda_pack_weights (GemmArgs.ldb == 0): 32-column slices
// stored one after the other, each as K rows of 64 bytes, so that a workgroup's slice is one
// contiguous block instead of a 64-byte piece out of every row of C.
#pragma once
#include <type_traits>

#include "bda_gemm_stream.hpp"

namespace bda {

constexpr int kDecodeMaxT = 128;

// s_waitcnt vmcnt(n) for a run-time n (even, <= 26): the largest immediate that is not above n.
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    if (n >= 26) wait_vmcnt<26>();
    else if (n >= 24) wait_vmcnt<24>();
    else if (n >= 22) wait_vmcnt<22>();
    else if (n >= 20) wait_vmcnt<20>();
    else if (n >= 18) wait_vmcnt<18>();
    else if (n >= 16) wait_vmcnt<16>();
    else if (n >= 14) wait_vmcnt<14>();
    else if (n >= 12) wait_vmcnt<12>();
    else if (n >= 10) wait_vmcnt<10>();
    else if (n >= 8) wait_vmcnt<8>();
    else if (n >= 6) wait_vmcnt<6>();
    else if (n >= 4) wait_vmcnt<4>();
    else if (n >= 2) wait_vmcnt<2>();
    else wait_vmcnt<0>();
}

// Group of a column slice and that group's table entries.  Every table entry is read whatever the
// slice (one batch of scalar loads from the kernel arguments, no load depends on another) and the
// entries wanted are picked by comparison: the chain from kernel start to the first request for C
// is what a launch with a few tokens waits for.
struct SliceGroup { int tile0; int64_t col0, col1; int a_off; };
__device__ __forceinline__ SliceGroup slice_group(const GemmArgs& p, int slice)
{
    int g = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroups; ++i) g += (i < p.n_groups && slice >= p.tile_start[i]) ? 1 : 0;
    SliceGroup r = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < kMaxGroups; ++i) {
        const bool hit = g == i;
        r.tile0 = hit ? p.tile_start[i] : r.tile0;
        r.col0 = hit ? p.col_start[i] : r.col0;
        r.col1 = hit ? p.col_start[i + 1] : r.col1;
        r.a_off = hit ? p.a_off[i] : r.a_off;
    }
    return r;
}
constexpr int kDecodeMaxK = 1536;       // K x 64 bytes of LDS for the slice of C
constexpr int kDecodeTokLdsMaxK = 512;  // up to here (and 64 tokens) the token rows go through LDS as well

// Every kernel argument a small-T kernel uses, the slice of this workgroup and its group's table
// entries, read in one batch of scalar loads at kernel start and pinned to registers there: three
// dependent trips to the argument block (tile count, tables, pitches) were about a tenth of such a
// launch.
struct DecodeArgs {
    const void *A, *B; void* D;
    int64_t lda, ldb, ldd, M;
    int K, d_h, a_skip, ident, n_tiles, slice;
    SliceGroup sg;
};
// More tokens than a workgroup takes (ROWS) are cut into token tiles: the grid is m_tiles copies of
// the slice grid, and a workgroup sees its tile as a problem of its own (A, D and M are those of
// the tile), so the kernels below never know.
template <int ROWS>
__device__ __forceinline__ DecodeArgs decode_args(const GemmArgs& p, int out_elem_bytes)
{
    DecodeArgs q = {p.A, p.B, p.D, p.lda, p.ldb, p.ldd, p.M, p.K, p.d_h, p.a_skip, p.ident, p.n_tiles, 0, {0, 0, 0, 0}};
    // dies take contiguous runs of slices
    const int per_xcd = (q.n_tiles + kNumXcd - 1) / kNumXcd;
    const int idx = (int)(blockIdx.x / kNumXcd);
    const int ttile = p.m_tiles > 1 ? idx / per_xcd : 0;
    q.slice = (int)(blockIdx.x % kNumXcd) * per_xcd + idx - ttile * per_xcd;
    const int64_t t0 = (int64_t)ttile * ROWS;
    q.A = (const char*)q.A + t0 * q.lda * 2;
    q.D = (char*)q.D + t0 * q.ldd * out_elem_bytes;
    q.M = q.M - t0 < ROWS ? q.M - t0 : ROWS;
    q.sg = slice_group(p, q.slice);
    asm volatile("" : "+s"(q.A), "+s"(q.B), "+s"(q.D), "+s"(q.lda), "+s"(q.ldb), "+s"(q.ldd), "+s"(q.M),
                 "+s"(q.sg.col0), "+s"(q.sg.col1));
    asm volatile("" : "+s"(q.K), "+s"(q.d_h), "+s"(q.a_skip), "+s"(q.ident), "+s"(q.n_tiles), "+s"(q.slice),
                 "+s"(q.sg.tile0), "+s"(q.sg.a_off));
    return q;
}

// TOK_LDS (used for 33 .. 64 tokens with K <= 512): the token rows go through LDS like the slice of C,
// requested as full 128-byte pieces (8 rows per instruction) instead of as MFMA fragments straight
// from global memory (32 rows x 32 bytes per instruction, which costs four times the address work:
// with 64 tokens those loads were what a launch waited for).  LDS then holds [slice of C][token rows:
// 64-k stage, token, 128 bytes, swizzled like the streaming kernel's token stages][partial sums];
// with two token blocks the partial sums reuse the token rows' space (one more barrier).
template <typename X, typename OutT, int NTB, bool TOK_LDS>
__global__ __launch_bounds__(256) void kv_decode_kernel(const GemmArgs p_in)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, lhi = lane >> 5;

    // slice owned by this workgroup
    const DecodeArgs p = decode_args<32 * NTB>(p_in, (int)sizeof(OutT));
    const int slice = p.slice;
    if (slice >= p.n_tiles) return;
    const SliceGroup sg = p.sg;
    const int rel0 = (slice - sg.tile0) * 32;
    const int64_t n0 = sg.col0 + rel0;
    const int64_t left = sg.col1 - n0;
    const int cols_left = (int)(left > 32 ? 32 : left);
    const int a_off = sg.a_off;
    const int T = (int)p.M;
    const int nks = (p.K + 15) >> 4;                     // k-steps of 16
    const int wgt_bytes = nks * 16 * 64;                 // LDS: [k][32 columns] 16-bit

    // ---- the slice of C: K rows x 64 bytes, 16 rows per DMA instruction (first of all: everything
    // else the kernel does before its MFMAs hides behind this request) --------------------------------
    const bool packed = p.ldb == 0;                      // (slices of a packed C are whole: widths are multiples of 32)
    const u32x4 rB = packed ? make_rsrc_words((const char*)p.B + n0 * p.K * 2, (int64_t)p.K * 64)
                            : make_rsrc_words((const char*)p.B + n0 * 2, ((int64_t)(p.K - 1) * p.ldb + cols_left) * 2);
    {
        const uint32_t row_bytes = packed ? 64u : (uint32_t)(p.ldb * 2);
        const int piece = lane & 3;
        const uint32_t lane_off = piece * 8 < cols_left ? (uint32_t)(lane >> 2) * row_bytes + (uint32_t)piece * 16u : kBadOffset;
        const int n_instr = nks;                          // 16 rows each
        for (int i = wave * 2; i < n_instr; i += 8) {     // two instructions per wave per round
            const uint32_t v0 = lane_off + (uint32_t)(i * 16) * row_bytes;
            const uint32_t v1 = i + 1 < n_instr ? lane_off + (uint32_t)((i + 1) * 16) * row_bytes : kBadOffset;
            lds_dma2(rB, (uint32_t)(i * 1024), v0, v1);   // rows past K fall outside rB's range -> zeros
        }
    }

    // ---- token fragments for this wave's k-steps (ks = wave, wave + 4, ...) --------------------------
    const int n_tb = (T + 31) >> 5;                      // <= NTB (host contract)
    const __amdgpu_buffer_rsrc_t rA = make_rsrc(p.A, ((int64_t)(T - 1) * p.lda + p.K + p.a_skip) * 2);
    const int ep_col = 8 * wave + 4 * lhi;               // this wave finishes columns 8 wave + 4 lhi + 0..3
    u32x2 idv[NTB];
    f32x16 acc[NTB];
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tb][r] = 0.0f;

    // transposing-read addresses: 16-lane group gq, s = lane % 16: row 8 lhi + 4 rd + s/4,
    // columns 16 (gq & 1) + 4 (s & 3) .. + 3
    const int c_s = lane & 15, c_gq = lane >> 4;
    const uint32_t w_rd = (uint32_t)((8 * lhi + (c_s >> 2)) * 64 + (16 * (c_gq & 1) + 4 * (c_s & 3)) * 2);
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;

    // identity values of the columns this wave finishes, wanted only in the epilogue: requested
    // behind the first token fragments; returns whether there were requests
    auto load_identity = [&]() -> bool {
        if (p.ident) {
            const int j = (rel0 + ep_col) % p.d_h;
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
                idv[tb] = __builtin_amdgcn_raw_buffer_load_b64(
                    rA, ep_col < cols_left ? (uint32_t)(tb * 32 + l31) * (uint32_t)(p.lda * 2) + (uint32_t)(a_off + j) * 2u : kBadOffset, 0, 0);
        } else {
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) idv[tb] = (u32x2){0u, 0u};
        }
        return p.ident != 0;
    };
    constexpr bool PART_ALIAS = TOK_LDS && NTB == 2;
    const int n_st = (p.K + 63) >> 6;
    const int tok_bytes = TOK_LDS ? n_st * NTB * 4096 : 0;
    if constexpr (TOK_LDS) {
        // token rows: one request = 8 rows x 128 bytes, the waves take turns; then the identity values;
        // all of it and the slice of C must have landed before anybody multiplies
        const u32x4 rAw = make_rsrc_words(p.A, ((int64_t)(T - 1) * p.lda + p.K + p.a_skip) * 2);
        const int row8 = lane >> 3;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + (uint32_t)wgt_bytes;
        const int n_req = n_st * NTB * 4;
        for (int i = wave; i < n_req; i += 4) {           // request i: stage i / (4 NTB), rows 8 (i % (4 NTB)) .. + 7
            const int st = i / (4 * NTB), row = 8 * (i % (4 * NTB)) + row8;
            const int k = 64 * st + 8 * ((lane & 7) ^ tok_swz<64>(row & 15));
            const int col = k < a_off ? k : k + p.a_skip;
            lds_dma1(rAw, lds0 + (uint32_t)i * 1024u,
                     row < T && k < p.K ? (uint32_t)row * (uint32_t)(p.lda * 2) + (uint32_t)col * 2u : kBadOffset);
        }
        if (load_identity()) wait_vmcnt<NTB>(); else wait_vmcnt<0>();
        __syncthreads();
        typedef __attribute__((address_space(3))) const u32x4* lds_u32x4;
        const uint32_t t_rd = lds0 + (uint32_t)(l31 * 128 + ((lhi ^ tok_swz<64>(l31 & 15)) << 4));
        for (int ks0 = wave; ks0 < nks; ks0 += 4 * 6) {   // chunks of six of this wave's k-steps: fragments first, then MFMAs
            u32x4 fw[6], ft[6][NTB];
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const bool ok = ks0 + 4 * i < nks;
                const int ks = ok ? ks0 + 4 * i : nks - 1;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + w_rd + ks * 1024));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + w_rd + ks * 1024 + 256));
                const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
                fw[i] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
                const uint32_t ta = (t_rd + (uint32_t)((ks >> 2) * (NTB * 4096))) ^ (uint32_t)((ks & 3) << 5);
#pragma unroll
                for (int tb = 0; tb < NTB; ++tb) {
                    const u32x4 t = *(lds_u32x4)(uintptr_t)(ta + tb * 4096);
                    ft[i][tb] = ok ? t : (u32x4){0u, 0u, 0u, 0u};          // a k-step past K adds nothing
                }
            }
#pragma unroll
            for (int i = 0; i < 6; ++i)
#pragma unroll
                for (int tb = 0; tb < NTB; ++tb) acc[tb] = X::mfma(fw[i], ft[i][tb], acc[tb]);
        }
        if constexpr (PART_ALIAS) __syncthreads();        // the partial sums overwrite the token rows
    } else {
    // first the token loads of all this wave's k-steps (they overlap the DMA), in chunks of 6 k-steps
    for (int ks0 = wave; ks0 < nks; ks0 += 4 * 6) {
        u32x4 ft[6][NTB];
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const int ks = ks0 + 4 * i;
            const int k = ks * 16 + 8 * lhi;
            const int col = k < a_off ? k : k + p.a_skip;
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) {
                const bool ok = ks < nks && k < p.K && tb < n_tb;
                ft[i][tb] = __builtin_amdgcn_raw_buffer_load_b128(
                    rA, ok ? (uint32_t)(tb * 32 + l31) * (uint32_t)(p.lda * 2) + (uint32_t)col * 2u : kBadOffset, 0, 0);
            }
        }
        if (ks0 == wave) {
            // the slice of C must have landed (all waves); the loads issued after it may still fly
            if (load_identity()) wait_vmcnt<7 * NTB>(); else wait_vmcnt<6 * NTB>();
            __syncthreads();
        }
        // the chunk's fragments of C first, then its MFMAs (k-steps past K read rows of zeros)
        u32x4 fw[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const int ks = ks0 + 4 * i < nks ? ks0 + 4 * i : nks - 1;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + w_rd + ks * 1024));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + w_rd + ks * 1024 + 256));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            fw[i] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
        }
#pragma unroll
        for (int i = 0; i < 6; ++i)                        // (token fragments past K or T hold zeros)
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) acc[tb] = X::mfma(fw[i], ft[i][tb], acc[tb]);
    }
    if (wave >= nks) {                                    // a wave without k-steps still joins the barrier
        load_identity();
        wait_vmcnt<0>();
        __syncthreads();
    }
    }

    // ---- fixed-order reduction over the four waves ------------------------------------------------
    // partial sums in LDS: [wave][tb][lane][4 groups of 4 accumulator rows], group q of lane l at
    // position q ^ (l / 4 % 4) (16-byte accesses of neighbouring lanes then fall into different banks)
    f32x4* part = (f32x4*)(smem + wgt_bytes + (PART_ALIAS ? 0 : tok_bytes));
    const int part_swz = (lane >> 2) & 3;
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
        if (tb < n_tb)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                part[((wave * NTB + tb) * 64 + lane) * 4 + (q ^ part_swz)] =
                    (f32x4){acc[tb][4 * q], acc[tb][4 * q + 1], acc[tb][4 * q + 2], acc[tb][4 * q + 3]};
    __syncthreads();
    // wave w finishes accumulator rows 4 w .. 4 w + 3 = output columns 8 w + 4 lhi + 0..3
    const int col = ep_col;
    const __amdgpu_buffer_rsrc_t rD = make_rsrc((char*)p.D + n0 * (int64_t)sizeof(OutT),
                                                ((int64_t)(T - 1) * p.ldd + cols_left) * (int64_t)sizeof(OutT));
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
        if (tb >= n_tb) break;
        f32x4 pw[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) pw[w] = part[((w * NTB + tb) * 64 + lane) * 4 + (wave ^ part_swz)];
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = ((pw[0][e] + pw[1][e]) + pw[2][e]) + pw[3][e];   // fixed order
        const int t = tb * 32 + l31;
        if (p.ident) {
            v[0] += X::to_f32((uint16_t)(idv[tb][0] & 0xffffu));
            v[1] += X::to_f32((uint16_t)(idv[tb][0] >> 16));
            v[2] += X::to_f32((uint16_t)(idv[tb][1] & 0xffffu));
            v[3] += X::to_f32((uint16_t)(idv[tb][1] >> 16));
        }
        const uint32_t off = col < cols_left ? (uint32_t)t * (uint32_t)(p.ldd * sizeof(OutT)) + (uint32_t)col * (uint32_t)sizeof(OutT) : kBadOffset;
        if constexpr (sizeof(OutT) == 4) {
            const f32x4 vf = {v[0], v[1], v[2], v[3]};
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vf), rD, off, 0, 0);
        } else {
            u32x2 o;
            o[0] = X::pack2(v[0], v[1]);
            o[1] = X::pack2(v[2], v[3]);
            __builtin_amdgcn_raw_buffer_store_b64(o, rD, off, 0, 0);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Wide-slice variant for K <= 384: one workgroup per 128-column slice of the output (up to 64 tokens)
// or per 64-column slice (up to 128 tokens).
//
// The 32-column kernel above needs N / 32 workgroups, which for a wide projection is several per
// compute unit one after the other, each with its own burst, reduction and tail.  Here a workgroup
// takes CW columns (K x 2 CW bytes of C, up to 96 KiB in flight per compute unit from the first
// instruction on); its four waves are WC = CW / 32 along the columns times WT = 4 / WC along the
// token blocks, each wave owns 32 columns and NTB / WT token blocks for the whole of K, so there
// is no reduction between waves, and the MFMAs of a quarter of the k-steps start as soon as that
// quarter of the slice has landed.
//   * C slice in LDS: [k][2 CW bytes]; the 16-byte pieces of a row are XOR-swizzled by the row number
//     so that the transposing reads of a wave (rows k .. k + 3, its own 64 bytes) hit 16 different
//     pieces per 32 lanes (CW = 128: piece ^ 4 (k & 3); CW = 64: piece ^ 4 (k / 2 & 1));
//   * the token rows go through LDS too (full 128-byte pieces per row and request, issued behind the
//     first quarter's requests for C: they hit L2, and the in-order counter then covers them with it);
//   * the identity slice is added in float32 from the latent, requested last, used in the epilogue.
constexpr int kDecodeWideMaxKS = 24;    // k-steps of 16: K <= 384

template <typename X, typename OutT, int NTB, int CW>
__global__ __launch_bounds__(256) void kv_decode_wide_kernel(const GemmArgs p_in)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    static_assert(CW == 128 || CW == 64, "slice width");
    constexpr int CH = 6;                                 // k-steps per chunk (four chunks)
    constexpr int WC = CW / 32, WT = 4 / WC, TPW = NTB / WT;
    static_assert(NTB % WT == 0, "token blocks per wave");
    constexpr int ROW_B = 2 * CW;                         // bytes of a row of the slice
    constexpr int RPI = 1024 / ROW_B;                     // rows per request: 4 or 8
    constexpr int KSPR = 4 * RPI / 16;                    // k-steps per round of four requests (one per wave): 1 or 2
    constexpr int RPC = CH / KSPR;                        // requests per wave and chunk: 6 or 3
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = wave % WC, wt = wave / WC;
    const int l31 = lane & 31, lhi = lane >> 5;

    const DecodeArgs p = decode_args<32 * NTB>(p_in, (int)sizeof(OutT));
    const int slice = p.slice;
    if (slice >= p.n_tiles) return;
    const SliceGroup sg = p.sg;
    const int rel0 = (slice - sg.tile0) * CW;
    const int64_t n0 = sg.col0 + rel0;
    const int64_t left = sg.col1 - n0;
    const int cols_left = (int)(left > CW ? CW : left);
    const int a_off = sg.a_off;
    const int T = (int)p.M;
    const int nks = (p.K + 15) >> 4;                     // <= kDecodeWideMaxKS (host contract)
    const int n_tb = (T + 31) >> 5;                      // <= NTB (host contract)
    const int issued = (nks + KSPR - 1) / KSPR;          // requests per wave for C

    // ---- the slice of C: request j of wave w brings rows 4 RPI j + RPI w .. + RPI - 1 to LDS offset
    // 4096 j + 1024 w; the first chunk's requests go out before anything else, the rest behind the
    // token rows ---------------------------------------------------------------------------------------
    // (packed C: the slice is CW / 32 sub-slices of K rows x 64 bytes one after the other; piece q of row k
    // lies in sub-slice q / 4 at byte 64 k + 16 (q % 4))
    const bool packed = p.ldb == 0;
    const u32x4 rB = packed ? make_rsrc_words((const char*)p.B + n0 * p.K * 2, (int64_t)(CW / 32) * p.K * 64)
                            : make_rsrc_words((const char*)p.B + n0 * 2, ((int64_t)(p.K - 1) * p.ldb + cols_left) * 2);
    const uint32_t row_bytes = packed ? 64u : (uint32_t)(p.ldb * 2);
    uint32_t c_lane_off;
    {
        constexpr int PPR = ROW_B / 16;                               // pieces per row: 16 or 8
        const int r = lane / PPR;                                     // row within the request
        const int swz = CW == 128 ? 4 * (r & 3) : 4 * ((r >> 1) & 1);
        const int piece = (lane % PPR) ^ swz;                         // global piece held at LDS position lane % PPR
        const uint32_t in_row = packed ? (uint32_t)(piece >> 2) * (uint32_t)p.K * 64u + (uint32_t)(piece & 3) * 16u : (uint32_t)piece * 16u;
        c_lane_off = piece * 8 < cols_left ? (uint32_t)(RPI * wave + r) * row_bytes + in_row : kBadOffset;
    }
    const int c_row0 = RPI * wave + lane / (ROW_B / 16);              // this lane's row in request 0
    const uint32_t c_lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + (uint32_t)wave * 1024u;
    auto request_c = [&](auto first, auto last) {                     // requests [first, last) of this wave
#pragma unroll
        for (int j = decltype(first)::value; j < decltype(last)::value; ++j)   // rows past K fall outside rB's range -> zeros
            if (j < issued)                                           // (packed: a row past K would be the next sub-slice's)
                lds_dma1(rB, c_lds0 + (uint32_t)j * 4096u,
                         (!packed || c_row0 + j * 4 * RPI < p.K) ? c_lane_off + (uint32_t)(j * 4 * RPI) * row_bytes : kBadOffset);
    };
    request_c(std::integral_constant<int, 0>{}, std::integral_constant<int, RPC>{});

    // ---- the token rows: [64-k stage][token][128 bytes] behind the slice of C, piece q of a row at
    // position q ^ tok_swz<64>(row); one request = 8 rows x 128 bytes, the waves take turns -----------
    const int n_st = (p.K + 63) >> 6;
    const uint32_t tok_lds = (uint32_t)issued * 4096u;
    const u32x4 rA = make_rsrc_words(p.A, ((int64_t)(T - 1) * p.lda + p.K + p.a_skip) * 2);
    {
        const int row8 = lane >> 3;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + tok_lds;
        const int n_req = n_st * NTB * 4;
        for (int i = wave; i < n_req; i += 4) {           // request i: stage i / (4 NTB), rows 8 (i % (4 NTB)) .. + 7
            const int st = i / (4 * NTB), row = 8 * (i % (4 * NTB)) + row8;
            const int k = 64 * st + 8 * ((lane & 7) ^ tok_swz<64>(row & 15));
            const int col = k < a_off ? k : k + p.a_skip;
            lds_dma1(rA, lds0 + (uint32_t)i * 1024u,
                     row < T && k < p.K ? (uint32_t)row * (uint32_t)(p.lda * 2) + (uint32_t)col * 2u : kBadOffset);
        }
    }
    request_c(std::integral_constant<int, RPC>{}, std::integral_constant<int, kDecodeWideMaxKS / KSPR>{});

    // ---- identity values of this lane's results (token l31 of the wave's block tbl, columns
    // 32 wc + 8 q + 4 lhi + 0..3), wanted only in the epilogue: requested last ------------------------
    const __amdgpu_buffer_rsrc_t rI = make_rsrc(p.A, ((int64_t)(T - 1) * p.lda + p.K + p.a_skip) * 2);
    u32x2 idv[TPW][4];
#pragma unroll
    for (int tbl = 0; tbl < TPW; ++tbl)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = 32 * wc + 8 * q + 4 * lhi;
            if (p.ident) {
                const int j = (rel0 + col) % p.d_h;
                idv[tbl][q] = __builtin_amdgcn_raw_buffer_load_b64(
                    rI, col < cols_left ? (uint32_t)((wt * TPW + tbl) * 32 + l31) * (uint32_t)(p.lda * 2) + (uint32_t)(a_off + j) * 2u : kBadOffset, 0, 0);
            } else idv[tbl][q] = (u32x2){0u, 0u};
        }
    const int n_idv = p.ident ? 4 * TPW : 0;

    f32x16 acc[TPW], acc2[TPW];                           // even and odd k-steps
#pragma unroll
    for (int tbl = 0; tbl < TPW; ++tbl)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tbl][r] = acc2[tbl][r] = 0.0f;

    // transposing-read address: 16-lane group gq, s = lane % 16: row 8 lhi + s / 4 (+ 4 for the second
    // read), columns 32 wc + 16 (gq & 1) + 4 (s & 3) .. + 3
    const int c_s = lane & 15, c_gq = lane >> 4;
    const int w_col = 32 * wc + 16 * (c_gq & 1) + 4 * (c_s & 3);
    const int w_swz = CW == 128 ? 4 * (c_s >> 2) : 4 * ((c_s >> 3) & 1);
    const uint32_t w_rd = (uint32_t)((8 * lhi + (c_s >> 2)) * ROW_B + (((w_col >> 3) ^ w_swz) << 4) + ((w_col & 4) << 1));
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;

    // fragment read of token block tb, k-step ks: row 32 tb + l31, pieces 2 (ks & 3) + lhi of stage ks / 4
    typedef __attribute__((address_space(3))) const u32x4* lds_u32x4;
    const uint32_t t_rd = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + tok_lds
                          + (uint32_t)(wt * TPW * 4096 + l31 * 128 + ((lhi ^ tok_swz<64>(l31 & 15)) << 4));

    // ---- four chunks of six k-steps: wait for this wave's requests of the chunk, meet the others ---
    // (the counter is in order: the token requests follow the first chunk's, so whatever may still
    // fly at chunk c are the requests for C of later chunks and the identity values)
#pragma unroll
    for (int c = 0; c < kDecodeWideMaxKS / CH; ++c) {
        const int later = issued - RPC * (c + 1);
        wait_vmcnt_at_most((later > 0 ? later : 0) + n_idv);
        __syncthreads();
        // the chunk's fragments first (eighteen reads in flight together), then its MFMAs; a k-step past K
        // multiplies zeros; the k-steps alternate between two accumulators per token block, which halves
        // the chain of dependent MFMAs
        u32x4 fw[CH], ft[CH][TPW];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool ok = CH * c + i < nks;
            const int ks = ok ? CH * c + i : nks - 1;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + w_rd + ks * (16 * ROW_B)));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(smem + w_rd + ks * (16 * ROW_B) + 4 * ROW_B));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            fw[i] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
            const uint32_t ta = (t_rd + (uint32_t)((ks >> 2) * (NTB * 4096))) ^ (uint32_t)((ks & 3) << 5);
#pragma unroll
            for (int tbl = 0; tbl < TPW; ++tbl) {          // (blocks past T hold zeros)
                const u32x4 t = *(lds_u32x4)(uintptr_t)(ta + tbl * 4096);
                ft[i][tbl] = ok ? t : (u32x4){0u, 0u, 0u, 0u};
            }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int tbl = 0; tbl < TPW; ++tbl) {
                if (i & 1) acc2[tbl] = X::mfma(fw[i], ft[i][tbl], acc2[tbl]);
                else acc[tbl] = X::mfma(fw[i], ft[i][tbl], acc[tbl]);
            }
    }
#pragma unroll
    for (int tbl = 0; tbl < TPW; ++tbl)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tbl][r] += acc2[tbl][r];

    // ---- epilogue: lane (token l31, half lhi) holds columns 32 wc + 8 q + 4 lhi + 0..3, q = 0..3 -----
    const __amdgpu_buffer_rsrc_t rD = make_rsrc((char*)p.D + n0 * (int64_t)sizeof(OutT),
                                                ((int64_t)(T - 1) * p.ldd + cols_left) * (int64_t)sizeof(OutT));
#pragma unroll
    for (int tbl = 0; tbl < TPW; ++tbl) {
        const int tb = wt * TPW + tbl;
        if (tb >= n_tb) break;
        const int t = tb * 32 + l31;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = 32 * wc + 8 * q + 4 * lhi;
            float v[4] = {acc[tbl][4 * q], acc[tbl][4 * q + 1], acc[tbl][4 * q + 2], acc[tbl][4 * q + 3]};
            if (p.ident) {
                v[0] += X::to_f32((uint16_t)(idv[tbl][q][0] & 0xffffu));
                v[1] += X::to_f32((uint16_t)(idv[tbl][q][0] >> 16));
                v[2] += X::to_f32((uint16_t)(idv[tbl][q][1] & 0xffffu));
                v[3] += X::to_f32((uint16_t)(idv[tbl][q][1] >> 16));
            }
            const uint32_t off = col < cols_left ? (uint32_t)t * (uint32_t)(p.ldd * sizeof(OutT)) + (uint32_t)col * (uint32_t)sizeof(OutT) : kBadOffset;
            if constexpr (sizeof(OutT) == 4) {
                const f32x4 vf = {v[0], v[1], v[2], v[3]};
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vf), rD, off, 0, 0);
            } else {
                u32x2 o;
                o[0] = X::pack2(v[0], v[1]);
                o[1] = X::pack2(v[2], v[3]);
                __builtin_amdgcn_raw_buffer_store_b64(o, rD, off, 0, 0);
            }
        }
    }
}

}  // namespace bda
