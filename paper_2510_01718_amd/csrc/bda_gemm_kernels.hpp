// Device kernels of libbda for gfx950 (CDNA4, wave64).
//
// One kernel family serves every run-time operator of the BD path:
//
//   D[t, n] = ident(t, n) + sum_{k < K} A[t, acol_g(k)] * B[k, n]
//
//   * BD K/V projection (steps 2-3 of Algorithm "BD Attention Inference"): A = latent c, B = C,
//     acol_g(k) skips the basis window of the group that owns column n, ident = c[t, off_g + j];
//   * dense projection (Algorithm "MHA Inference", steps 2-3): acol(k) = k, ident = 0;
//   * the two products of the BD linear layer (Section "BD for Linear Layer").
//
// The activations (A) are k-contiguous in memory, the weights (B) are n-contiguous.  MFMA wants
// both operands k-contiguous per lane, so the weight tile is transposed in registers (8x8 blocks of
// 16-bit values) on its way from global memory to LDS.  The weight tile is fed as the MFMA's row
// operand and the token tile as its column operand: the accumulator layout then gives each lane
// four consecutive output columns of one token, which are stored as one 8- or 16-byte write.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bda {

constexpr int kMaxGroups = 8;
constexpr int kNumXcd = 8;           // MI355X: 8 accelerator dies, each with its own L2
constexpr int kSlotsPerXcd = 32;     // 32 compute units per die -> 256 persistent workgroups

struct GemmArgs {
    const void* A;
    const void* B;
    void* D;
    int64_t lda, ldb, ldd;           // in elements
    int64_t M;                       // tokens
    int K;                           // contraction length (rows of B)
    int n_groups;
    int d_h;                         // period of the identity slice (ident != 0)
    int a_skip;                      // width of the basis window skipped in A's columns (0: none)
    int ident;                       // 1: D starts from A[t, a_off_g + (n - col_start_g) % d_h]
    int m_tiles, n_tiles;            // tile grid (n_tiles counts the tiles of all groups)
    int sm, sn;                      // super-tile shape handed to one die at a time (sm*sn = 32)
    int n_stage_id;                  // streaming kernel: identity stages per tile (0 if ident == 0)
    int n_super_m, n_super_n;        // streaming kernel: super-tile grid, ceil(m_tiles / sm) x ceil(n_tiles / sn)
    int sn_shift;                    // streaming kernel: log2(sn)
    uint64_t dh_magic;               // streaming kernel: ceil(2^40 / d_h), for x % d_h with x < 2^24
    int rounds;                      // streaming kernel: super-tiles per die, ceil(n_super_m n_super_n / 8)
    int xcd_q0[8], xcd_r0[8];        // streaming kernel: first super-tile of die x (token, column index)
    int xcd_count[8];                // streaming kernel: super-tiles of die x (<= rounds)
    int lin_slots;                   // lean streaming kernel: > 0 = tile-by-tile order, workgroups per die
    int tile_start[kMaxGroups + 1];  // first column tile of each group
    int64_t col_start[kMaxGroups + 1];  // first output column of each group
    int a_off[kMaxGroups];           // basis window start of each group (k >= a_off -> k + a_skip)
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct F16 {
    typedef _Float16 elem;
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
    static __device__ __forceinline__ uint16_t from_f32(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }
    // two values rounded (nearest even) and packed, lo in bits 0..15: one v_cvt_pk_f16_f32
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        const f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
};

struct BF16 {
    typedef __bf16 elem;
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_f32(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
    static __device__ __forceinline__ uint16_t from_f32(float v)
    {
        // round to nearest even; NaN stays NaN (quiet)
        uint32_t u = __builtin_bit_cast(uint32_t, v);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
        u += 0x7fffu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    // two values rounded (nearest even) and packed, lo in bits 0..15: one v_cvt_pk_bf16_f32
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        const f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
};

// LDS tile layout: row r holds BK = 64 16-bit values (128 bytes) as eight 16-byte chunks, rows are
// 144 bytes apart.  The 16-byte pad makes the lanes of one ds_read_b128 / ds_write_b128 (consecutive
// rows, same chunk) fall on different banks, and keeps every address of the form
// "per-lane base + compile-time constant", so the reads use immediate offsets.
constexpr int kRowBytes = 144;
__device__ __forceinline__ int lds_off(int r, int q) { return r * kRowBytes + (q << 4); }

// 8x8 transpose of 16-bit values held as eight 16-byte rows: in[i] = row k_i with columns n0..n7;
// out[j] = column n_j with rows k0..k7.
__device__ __forceinline__ void transpose8x8_b16(const u32x4 (&in)[8], u32x4 (&out)[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t x = in[2 * p][j >> 1];       // row 2p   : columns (j&~1, j|1)
            const uint32_t y = in[2 * p + 1][j >> 1];   // row 2p+1
            out[j][p] = (j & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
        }
    }
}

// Buffer resources: every global access of the MFMA kernel goes through a raw buffer descriptor
// whose range ends with the last valid byte of the tile's rows, so rows past the end of the tensor
// read as zero and are never written, without per-lane branches.  Offsets that must not be
// accessed for other reasons (columns past a group's end) are replaced by kBadOffset, which lies
// beyond any range this kernel builds (ranges are capped at 2 GiB).
constexpr uint32_t kBadOffset = 0x80000000u;
constexpr int64_t kMaxRange = 0x80000000ll;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes)
{
    const int range = (int)(bytes > kMaxRange ? kMaxRange : (bytes < 0 ? 0 : bytes));
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, range, 0x00020000);
}

template <typename X>
struct IdentityFrag;   // 32 x 32 identity as an MFMA row operand, for k-steps 0 and 1
template <>
struct IdentityFrag<F16> { static constexpr uint32_t one = 0x3C00u; };
template <>
struct IdentityFrag<BF16> { static constexpr uint32_t one = 0x3F80u; };

// Persistent MFMA GEMM.  256 threads = 4 waves in a 2 (tokens) x 2 (columns) arrangement; each wave
// owns TT x TN MFMA tiles of 32 x 32, so the workgroup tile is (64 TT) tokens x (64 TN) columns.
//
// The contraction runs over chunks of 64: first the K rows of B, then -- for the BD projection --
// the identity slice as extra chunks whose weight tile is the identity matrix and is therefore
// never loaded: token columns [off + j, ...) are staged like any other chunk and each 32-column
// MFMA tile multiplies the one 32-wide piece that belongs to it by a constant identity fragment.
// The slice is thus added in float32 inside the accumulator (x * 1 + acc is exact up to the
// accumulator's own rounding), with no extra pass, no extra registers and no epilogue arithmetic.
template <typename X, typename OutT, int TT, int TN>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const GemmArgs p)
{
    constexpr int BT = 64 * TT;            // tokens per workgroup tile
    constexpr int BN = 64 * TN;            // output columns per workgroup tile
    constexpr int TOK_STAGE = BT * kRowBytes;  // bytes of one token-tile stage (BK = 64)
    constexpr int WGT_STAGE = BN * kRowBytes;  // bytes of one weight-tile stage
    constexpr int WGT_BASE = 2 * TOK_STAGE;    // LDS: [tok 0][tok 1][wgt 0][wgt 1]
    constexpr int TOK_LOADS = BT / 32;     // 16-byte chunks of the token tile per thread
    constexpr int WGT_BLOCKS = (BN + 255) / 256;  // 8x8 weight blocks per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lives in an SGPR
    const int wt = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lhi = lane >> 5;

    const int nk = (p.K + 63) >> 6;
    const int n_super_n = (p.n_tiles + p.sn - 1) / p.sn;
    const int n_super_m = (p.m_tiles + p.sm - 1) / p.sm;
    const int total_super = n_super_m * n_super_n;
    const int slots = p.sm * p.sn;
    const int xcd = blockIdx.x % kNumXcd;
    const int slot = blockIdx.x / kNumXcd;
    if (slot >= slots) return;

    // identity fragments (row operand): lane (row i = l31, half lhi) holds k' = 16 v + 8 lhi + e
    u32x4 idf[2];
#pragma unroll
    for (int v = 0; v < 2; ++v)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int k0 = 16 * v + 8 * lhi + 2 * w;
            idf[v][w] = (k0 == l31 ? IdentityFrag<X>::one : 0u) | (k0 + 1 == l31 ? IdentityFrag<X>::one << 16 : 0u);
        }

    // per-thread tile-independent offsets
    const int tq = tid & 7;                          // token tile: chunk within the row
    const uint32_t tok_row_bytes = (uint32_t)(p.lda * 2);
    const uint32_t tok_voff0 = (uint32_t)(tid >> 3) * tok_row_bytes;
    const int wq = tid & 7;                          // weight tile: 8-row block within the chunk
    const uint32_t wgt_row_bytes = (uint32_t)(p.ldb * 2);

    for (int s = xcd; s < total_super; s += kNumXcd) {
        const int mt = (s / n_super_n) * p.sm + slot / p.sn;
        const int nt = (s % n_super_n) * p.sn + slot % p.sn;
        if (mt >= p.m_tiles || nt >= p.n_tiles) continue;   // uniform over the workgroup
        int g = 0;
        while (g + 1 < p.n_groups && nt >= p.tile_start[g + 1]) ++g;
        const int64_t rel0 = (int64_t)(nt - p.tile_start[g]) * BN;   // column inside the group
        const int64_t n0 = p.col_start[g] + rel0;
        const int cols_left = (int)((p.col_start[g + 1] - n0) > BN ? BN : (p.col_start[g + 1] - n0));
        const int64_t t0 = (int64_t)mt * BT;
        const int64_t rows_left = p.M - t0;
        const int a_off = p.a_off[g];

        const __amdgpu_buffer_rsrc_t rA = make_rsrc(
            (const char*)p.A + t0 * p.lda * 2, ((rows_left - 1) * p.lda + p.K + p.a_skip) * 2);
        const __amdgpu_buffer_rsrc_t rB = make_rsrc(
            (const char*)p.B + n0 * 2, ((int64_t)(p.K - 1) * p.ldb + cols_left) * 2);
        const __amdgpu_buffer_rsrc_t rD = make_rsrc(
            (char*)p.D + (t0 * p.ldd + n0) * (int64_t)sizeof(OutT),
            ((rows_left - 1) * p.ldd + cols_left) * (int64_t)sizeof(OutT));

        // identity slice: columns [j_lo, j_lo + W) of the window, in chunks of 64
        int j_lo = 0, n_id = 0;
        if (p.ident) {
            const bool nested = (p.d_h % BN) == 0;
            j_lo = nested ? (int)(rel0 % p.d_h) : 0;
            n_id = ((nested ? BN : p.d_h) + 63) >> 6;
        }
        const int nk_total = nk + n_id;
        const int rel_wave = (int)((rel0 + wn * (32 * TN)) % (p.d_h > 0 ? p.d_h : 1));

        u32x4 tok_reg[TOK_LOADS];
        u32x4 wgt_reg[WGT_BLOCKS][8];

        // weight tile: columns past the group's end are never read (offset beyond any range); rows
        // past K fall outside rB's range by construction
        uint32_t wgt_voff[WGT_BLOCKS];
#pragma unroll
        for (int b = 0; b < WGT_BLOCKS; ++b) {
            const int nb = (tid >> 3) + 32 * b;
            wgt_voff[b] = nb * 8 < cols_left ? (uint32_t)(wq * 8) * wgt_row_bytes + (uint32_t)nb * 16u : kBadOffset;
        }
        auto load_chunk = [&](int kc) {
            uint32_t voff;
            if (kc < nk) {
                const int k = kc * 64 + tq * 8;
                const int col = k < a_off ? k : k + p.a_skip;
                voff = k < p.K ? tok_voff0 + (uint32_t)col * 2u : kBadOffset;
            } else {
                const int j = j_lo + (kc - nk) * 64 + tq * 8;
                voff = j < p.d_h ? tok_voff0 + (uint32_t)(a_off + j) * 2u : kBadOffset;
            }
#pragma unroll
            for (int i = 0; i < TOK_LOADS; ++i)
                tok_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(rA, voff + (uint32_t)(32 * i) * tok_row_bytes, 0, 0);
            if (kc < nk) {
#pragma unroll
                for (int b = 0; b < WGT_BLOCKS; ++b) {
                    const uint32_t base = wgt_voff[b] + (uint32_t)(kc * 64) * wgt_row_bytes;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        wgt_reg[b][i] = __builtin_amdgcn_raw_buffer_load_b128(rB, base + (uint32_t)i * wgt_row_bytes, 0, 0);
                }
            }
        };
        auto store_chunk = [&](int kc) {
            unsigned char* tok_s = smem + (kc & 1) * TOK_STAGE;
            unsigned char* wgt_s = smem + WGT_BASE + (kc & 1) * WGT_STAGE;
#pragma unroll
            for (int i = 0; i < TOK_LOADS; ++i)
                *(u32x4*)(tok_s + lds_off((tid >> 3) + 32 * i, tq)) = tok_reg[i];
            if (kc < nk) {
#pragma unroll
                for (int b = 0; b < WGT_BLOCKS; ++b) {
                    const int nb = (tid >> 3) + 32 * b;
                    if (nb * 8 < BN) {
                        u32x4 tr[8];
                        transpose8x8_b16(wgt_reg[b], tr);
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            *(u32x4*)(wgt_s + lds_off(nb * 8 + j, wq)) = tr[j];
                    }
                }
            }
        };

        // accumulators: acc[ni][ti], rows = output columns, columns = tokens
        f32x16 acc[TN][TT];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int ti = 0; ti < TT; ++ti)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ni][ti][r] = 0.0f;

        // main loop: double-buffered LDS, next chunk's global loads in flight during the MFMAs
        const int tok_rd = (wt * (32 * TT) + l31) * kRowBytes + lhi * 16;
        const int wgt_rd = WGT_BASE + (wn * (32 * TN) + l31) * kRowBytes + lhi * 16;
        load_chunk(0);
        store_chunk(0);
        __syncthreads();
        for (int kc = 0; kc < nk; ++kc) {
            const bool more = kc + 1 < nk_total;
            if (more) load_chunk(kc + 1);
            const unsigned char* tok_s = smem + tok_rd + (kc & 1) * TOK_STAGE;
            const unsigned char* wgt_s = smem + wgt_rd + (kc & 1) * WGT_STAGE;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4 fw[TN], ft[TT];
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
                    fw[ni] = *(const u32x4*)(wgt_s + ni * 32 * kRowBytes + ks * 32);
#pragma unroll
                for (int ti = 0; ti < TT; ++ti)
                    ft[ti] = *(const u32x4*)(tok_s + ti * 32 * kRowBytes + ks * 32);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                    for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(fw[ni], ft[ti], acc[ni][ti]);
            }
            if (more) store_chunk(kc + 1);
            __syncthreads();
        }
        // identity chunks: the staged token columns are slice columns jc .. jc + 63
        for (int kc = nk; kc < nk_total; ++kc) {
            const bool more = kc + 1 < nk_total;
            if (more) load_chunk(kc + 1);
            const unsigned char* tok_s = smem + tok_rd + (kc & 1) * TOK_STAGE;
            const int jc = j_lo + (kc - nk) * 64;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4 ft[TT];
#pragma unroll
                for (int ti = 0; ti < TT; ++ti)
                    ft[ti] = *(const u32x4*)(tok_s + ti * 32 * kRowBytes + ks * 32);
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) {
                    // position of this k-step's 16 slice columns inside the MFMA tile's 32 columns
                    const int d = jc + 16 * ks - (rel_wave + 32 * ni) % p.d_h;
                    if (d == 0 || d == 16) {
                        const u32x4 f = d == 0 ? idf[0] : idf[1];
#pragma unroll
                        for (int ti = 0; ti < TT; ++ti) acc[ni][ti] = X::mfma(f, ft[ti], acc[ni][ti]);
                    }
                }
            }
            if (more) store_chunk(kc + 1);
            __syncthreads();
        }

        // epilogue: one rounding, four consecutive columns per lane; rows past M fall outside rD's
        // range, column blocks past the group's end are skipped (uniform per wave: groups end on
        // multiples of 8 columns)
        const uint32_t ep_lane = (uint32_t)(wt * (32 * TT) + l31) * (uint32_t)(p.ldd * sizeof(OutT)) +
                                 (uint32_t)(wn * (32 * TN) + lhi * 4) * (uint32_t)sizeof(OutT);
        const uint32_t ep_row_step = 32u * (uint32_t)(p.ldd * sizeof(OutT));
#pragma unroll
        for (int ti = 0; ti < TT; ++ti) {
            const uint32_t row_off = ep_lane + (uint32_t)ti * ep_row_step;
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
                __builtin_amdgcn_sched_barrier(0);   // keep one MFMA tile's conversions live at a time
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int c0 = ni * 32 + rg * 8;
                    if (wn * (32 * TN) + c0 >= cols_left) continue;
                    const uint32_t off = row_off + (uint32_t)c0 * (uint32_t)sizeof(OutT);
                    if constexpr (sizeof(OutT) == 4) {
                        // (the elements are copied to named floats first: bit-casting a vector
                        // element expression directly reads element 0 with this compiler)
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
}

// General kernel: any element type, any shape or alignment.  64 x 64 output tile per workgroup of
// 256 threads (4 x 4 outputs each), BK = 16, scalar guarded loads, float32 FMA accumulation.
template <typename InT>
__device__ __forceinline__ float load_as_f32(const InT* p);
template <>
__device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
struct RawF16 { uint16_t b; };
struct RawBF16 { uint16_t b; };
template <>
__device__ __forceinline__ float load_as_f32<RawF16>(const RawF16* p) { return F16::to_f32(p->b); }
template <>
__device__ __forceinline__ float load_as_f32<RawBF16>(const RawBF16* p) { return BF16::to_f32(p->b); }

template <typename OutT>
__device__ __forceinline__ void store_from_f32(OutT* p, float v);
template <>
__device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_from_f32<RawF16>(RawF16* p, float v) { p->b = F16::from_f32(v); }
template <>
__device__ __forceinline__ void store_from_f32<RawBF16>(RawBF16* p, float v) { p->b = BF16::from_f32(v); }

template <typename InT, typename OutT>
__global__ __launch_bounds__(256) void gemm_general_kernel(const GemmArgs p, int64_t N_total)
{
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const InT* __restrict__ Ag = (const InT*)p.A;
    const InT* __restrict__ Bg = (const InT*)p.B;
    OutT* __restrict__ Dg = (OutT*)p.D;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    // column tiles are laid out per group so that a tile never straddles two basis windows
    const int nt = blockIdx.x;
    int g = 0;
    while (g + 1 < p.n_groups && nt >= p.tile_start[g + 1]) ++g;
    const int64_t n0 = p.col_start[g] + (int64_t)(nt - p.tile_start[g]) * 64;
    const int64_t n_end = p.col_start[g + 1];
    const int64_t t0 = (int64_t)blockIdx.y * 64;
    const int a_off = p.a_off[g];
    (void)N_total;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t t = t0 + ty * 4 + i, n = n0 + tx * 4 + j;
            float v = 0.0f;
            if (p.ident && t < p.M && n < n_end)
                v = load_as_f32(Ag + t * p.lda + a_off + (int)((n - p.col_start[g]) % p.d_h));
            acc[i][j] = v;
        }
    for (int k0 = 0; k0 < p.K; k0 += 16) {
        // 64 x 16 slice of A and 16 x 64 slice of B, four elements per thread each
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            {
                const int kk = idx & 15, r = idx >> 4;
                const int k = k0 + kk;
                const int64_t t = t0 + r;
                float v = 0.0f;
                if (k < p.K && t < p.M) v = load_as_f32(Ag + t * p.lda + (k < a_off ? k : k + p.a_skip));
                As[kk][r] = v;
            }
            {
                const int c = idx & 63, kk = idx >> 6;
                const int k = k0 + kk;
                const int64_t n = n0 + c;
                float v = 0.0f;
                if (k < p.K && n < n_end) v = load_as_f32(Bg + (int64_t)k * p.ldb + n);
                Bs[kk][c] = v;
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
            const int64_t t = t0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (t < p.M && n < n_end) store_from_f32(Dg + t * p.ldd + n, acc[i][j]);
        }
}

}  // namespace bda
