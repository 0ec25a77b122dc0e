// GPU preparation of one projection (Algorithm "BD Attention Preparation (QK)", Appendix "BD for VO in
// MHA", Algorithm "BD Decomposition (Row)" for the window choice, Appendix "Residual-Min with Offset
// Search" for the candidate windows).  Float64 throughout, four kernels:
//   prepare_kernel   C_h = W_h[Bbar,:] W_h[B,:]^{-1}, one workgroup per head (several when there are few heads:
//                    each inverts for itself and takes a share of the rows): the d_h x d_h basis block
//                    is inverted in place by Gauss-Jordan elimination with partial (row) pivoting (in
//                    LDS up to d_h = 128, in the caller's workspace up to 256; the row interchanges are
//                    undone as column interchanges at the end), then the d_c - d_h rows outside the
//                    window are multiplied by the inverse, 16 rows at a time staged through LDS, and
//                    stored rounded to the requested type;
//   side_kernel      the companion block: W_q^h W_h[B,:]^T or W_h[B,:] W_o^h, rounded the same way;
//   residual_kernel  the Frobenius reconstruction error of the stored form of one head - what was just
//                    written to C and to the companion output, read back - as partial sums of squares
//                    (a fixed number of parts per head, each summed in a fixed order);
//   select_kernel    per candidate window the mean over heads of the residuals, the smallest mean
//                    (earlier candidate on ties, NaN as +inf), the chosen window start.
// A search runs prepare / side / residual once per candidate window into the caller's outputs, selects,
// and runs prepare / side once more for the chosen window, whose start it reads from device memory:
// nothing comes back to the host in between.
// The host routine bda_prepare solves with an orthogonal factorisation instead of forming the inverse;
// the two agree to a small multiple of cond(W_h[B,:]) * 2^-53.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "bda_internal.h"

// Scratch memory of bda_prepare_device_static, the entry point for callers that cannot allocate: part of
// the code object, so every GPU the library runs on holds its own copy from the moment the code is loaded
// there until the process ends.  Host code never uses this name as an address: it asks the runtime for
// the array's address on the current device (static_scratch below) and passes that to the kernels.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace bda {
namespace {

template <typename T> __device__ __forceinline__ double load_as_double(const void* p, int64_t i);
template <> __device__ __forceinline__ double load_as_double<double>(const void* p, int64_t i) { return ((const double*)p)[i]; }
template <> __device__ __forceinline__ double load_as_double<float>(const void* p, int64_t i) { return (double)((const float*)p)[i]; }
template <> __device__ __forceinline__ double load_as_double<_Float16>(const void* p, int64_t i) { return (double)((const _Float16*)p)[i]; }
template <> __device__ __forceinline__ double load_as_double<__bf16>(const void* p, int64_t i)
{
    const uint32_t b = (uint32_t)((const uint16_t*)p)[i] << 16;
    return (double)__builtin_bit_cast(float, b);
}

// One rounding, to nearest even, from double to the stored type.
template <typename T> __device__ __forceinline__ void store_rounded(void* p, int64_t i, double v);
template <> __device__ __forceinline__ void store_rounded<double>(void* p, int64_t i, double v) { ((double*)p)[i] = v; }
template <> __device__ __forceinline__ void store_rounded<float>(void* p, int64_t i, double v) { ((float*)p)[i] = (float)v; }
template <> __device__ __forceinline__ void store_rounded<_Float16>(void* p, int64_t i, double v)
{
    ((_Float16*)p)[i] = (_Float16)v;          // the compiler converts f64 -> f16 with one rounding
}
template <> __device__ __forceinline__ void store_rounded<__bf16>(void* p, int64_t i, double v)
{
    // bf16 = the upper half of a float: round the double to 8 significant bits directly.  Going through
    // float first would round twice; instead the float is formed by truncation toward zero plus a
    // sticky bit, and the final rounding looks at that.
    float f = (float)v;
    if ((double)f != v) {                     // inexact: make sure the discarded part is seen below
        uint32_t b = __builtin_bit_cast(uint32_t, f);
        const bool too_big = (v >= 0) ? ((double)f > v) : ((double)f < v);
        if (too_big) b -= 1;                  // f is now v truncated toward zero ...
        b |= 1u;                              // ... with a sticky bit (never lands on a bf16 tie)
        f = __builtin_bit_cast(float, b);
    }
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    if ((b & 0x7f800000u) != 0x7f800000u) b += 0x7fffu + ((b >> 16) & 1u);
    ((uint16_t*)p)[i] = (uint16_t)(b >> 16);
}

constexpr int kPrepThreads = 256;
constexpr int kPrepLdsDh = 128;               // largest head width whose basis block is inverted in LDS
constexpr int kPrepMaxDh = 256;               // largest head width at all (block in the workspace)
constexpr int kPrepRows = 16;                 // rows of W_h[Bbar,:] staged per pass
constexpr int kMaxCandidates = 256;
constexpr int kMaxParts = 64;                 // workgroups per head of the residual kernel, at most (heads x parts <= 1024: about four
                                              // workgroups per compute unit, which cover one another's exposed load latency)

struct PrepArgs {
    const void* W;
    const void* side;            // companion weight (type of W) or NULL
    void* C;
    void* side_out;              // companion output (type of C) or NULL
    int* status;                 // singular_head of the public calls, or NULL
    const int* off_ptr;          // device: window start chosen by select_kernel (NULL: `off`)
    int* cand_singular;          // workspace: one flag per candidate window, or NULL
    double* partials;            // workspace: [candidate][head][part] sums of squares, or NULL
    double* mat;                 // workspace: one d_h x d_h block per workgroup of a batch (d_h > 128), or NULL
    int64_t ldw, ld_side, ldC, ld_side_out;
    int d_c, H, d_h, off, d_side, side_kind;
    int h0;                      // first head of this launch (batches when the block lives in the workspace)
    int cand, n_parts;
};

__device__ __forceinline__ int window_start(const PrepArgs& a) { return a.off_ptr ? *a.off_ptr : a.off; }

// BIG: the basis block lives in global memory (a.mat, one block per workgroup) instead of LDS.
template <typename WT, typename CT, bool BIG>
__global__ __launch_bounds__(kPrepThreads) void prepare_kernel(const PrepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int n = a.d_h;
    const int ld = BIG ? n : n + 1;            // LDS: odd stride in doubles, a column walk touches all banks
    double* R;                                 // kPrepRows x n staging, also scratch for the reductions
    double* A;                                 // n x ld: the basis block, then its inverse
    if constexpr (BIG) {
        R = (double*)smem_raw;
        A = a.mat + (size_t)blockIdx.x * n * n;
    } else {
        A = (double*)smem_raw;
        R = A + (size_t)n * ld;
    }
    __shared__ int piv[kPrepMaxDh];
    __shared__ int s_pivot_row;
    __shared__ double s_pivot_val;
    __shared__ int s_singular;

    const int t = threadIdx.x;
    const int h = a.h0 + blockIdx.x;
    const int off = window_start(a);
    if (off < 0) return;                       // no usable window was found: nothing to prepare
    const int64_t col0 = (int64_t)h * n;

    // ---- basis block and its scale --------------------------------------------------------------
    double part = 0.0;
    for (int e = t; e < n * n; e += kPrepThreads) {
        const int i = e / n, j = e % n;
        const double v = load_as_double<WT>(a.W, (int64_t)(off + i) * a.ldw + col0 + j);
        A[i * ld + j] = v;
        part += v * v;
    }
    R[t] = part;
    if (t == 0) s_singular = 0;
    __syncthreads();
    if (t == 0) {
        double s = 0.0;
        for (int i = 0; i < kPrepThreads; ++i) s += R[i];
        s_pivot_val = s;
    }
    __syncthreads();
    const double tiny = sqrt(s_pivot_val) * n * 2.220446049250313e-16;
    __syncthreads();

    // ---- Gauss-Jordan inversion in place, partial pivoting ----------------------------------------
    // thread -> (row, segment of the columns): two threads per row up to 128 rows, one per row beyond
    const int rows_per_pass = n <= 128 ? 128 : 256;
    const int row = t % rows_per_pass, seg = t / rows_per_pass, n_seg = kPrepThreads / rows_per_pass;
    const int jn = (n + n_seg - 1) / n_seg;
    const int j_lo = seg * jn, j_hi = (j_lo + jn < n) ? j_lo + jn : n;
    for (int k = 0; k < n; ++k) {
        // pivot: the largest |A[i][k]|, i >= k (first such row on ties)
        if (t < 64) {
            double best = -1.0;
            int bi = k;
            for (int i = k + t; i < n; i += 64) {
                const double v = fabs(A[i * ld + k]);
                if (v > best) { best = v; bi = i; }
            }
            for (int s = 32; s >= 1; s >>= 1) {
                const double ov = __shfl_xor(best, s, 64);
                const int oi = __shfl_xor(bi, s, 64);
                if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
            }
            if (t == 0) {
                s_pivot_row = bi;
                piv[k] = bi;
                if (!(best > tiny)) s_singular = 1;
            }
        }
        __syncthreads();
        if (s_singular) break;
        const int p = s_pivot_row;
        if (p != k) {
            for (int j = t; j < n; j += kPrepThreads) {
                const double x = A[k * ld + j];
                A[k * ld + j] = A[p * ld + j];
                A[p * ld + j] = x;
            }
        }
        __syncthreads();
        const double pv = A[k * ld + k];
        const double f = (row < n) ? A[row * ld + k] : 0.0;      // multiplier of this thread's row
        __syncthreads();
        // row k becomes (row k with 1 in place of the pivot) / pivot
        const double inv = 1.0 / pv;
        for (int j = t; j < n; j += kPrepThreads) A[k * ld + j] = (j == k ? 1.0 : A[k * ld + j]) * inv;
        __syncthreads();
        if (row < n && row != k) {
#pragma unroll 8
            for (int j = j_lo; j < j_hi; ++j) {
                const double cur = (j == k) ? 0.0 : A[row * ld + j];
                A[row * ld + j] = cur - f * A[k * ld + j];
            }
        }
        __syncthreads();
    }
    if (s_singular) {
        if (t == 0) {
            if (a.status) atomicMax(a.status, h + 1);
            if (a.cand_singular) a.cand_singular[a.cand] = 1;    // (every writer stores the same value)
        }
        return;
    }
    // the elimination inverted P A; A^{-1} = (P A)^{-1} P: undo the interchanges on the columns, last first
    for (int k = n - 1; k >= 0; --k) {
        const int p = piv[k];
        if (p != k) {
            for (int i = t; i < n; i += kPrepThreads) {
                const double x = A[i * ld + k];
                A[i * ld + k] = A[i * ld + p];
                A[i * ld + p] = x;
            }
            __syncthreads();
        }
    }
    __syncthreads();

    // ---- C_h = W_h[Bbar,:] A^{-1} ------------------------------------------------------------------
    // With few heads a launch leaves most compute units idle, and the inversion above is one workgroup's
    // latency whatever else runs: gridDim.y workgroups per head each invert the block for themselves (the
    // same operations in the same order, so the same inverse bit for bit) and share out the row blocks of
    // the product, which is a third of the kernel's time when one workgroup does all of them.
    const int K = a.d_c - n;
    for (int r0 = (int)blockIdx.y * kPrepRows; r0 < K; r0 += (int)gridDim.y * kPrepRows) {
        for (int e = t; e < kPrepRows * n; e += kPrepThreads) {
            const int i = e / n, c = e % n;
            const int r = r0 + i;
            const int src = r < off ? r : r + n;                   // rows outside the window, ascending
            R[i * n + c] = r < K ? load_as_double<WT>(a.W, (int64_t)src * a.ldw + col0 + c) : 0.0;
        }
        __syncthreads();
        // thread -> (output column, subset of the staged rows): rows rg, rg + n_rg, ...
        const int cols_per_pass = n <= 128 ? 128 : 256;
        const int j = t % cols_per_pass, rg = t / cols_per_pass, n_rg = kPrepThreads / cols_per_pass;
        if (j < n) {
            double acc[kPrepRows];
#pragma unroll
            for (int m = 0; m < kPrepRows; ++m) acc[m] = 0.0;
            if (n_rg == 2) {
#pragma unroll 4
                for (int k = 0; k < n; ++k) {
                    const double b = A[k * ld + j];
#pragma unroll
                    for (int m = 0; m < kPrepRows / 2; ++m) acc[m] = fma(R[(2 * m + rg) * n + k], b, acc[m]);
                }
#pragma unroll
                for (int m = 0; m < kPrepRows / 2; ++m) {
                    const int r = r0 + 2 * m + rg;
                    if (r < K) store_rounded<CT>(a.C, (int64_t)r * a.ldC + col0 + j, acc[m]);
                }
            } else {
#pragma unroll 4
                for (int k = 0; k < n; ++k) {
                    const double b = A[k * ld + j];
#pragma unroll
                    for (int m = 0; m < kPrepRows; ++m) acc[m] = fma(R[m * n + k], b, acc[m]);
                }
#pragma unroll
                for (int m = 0; m < kPrepRows; ++m) {
                    const int r = r0 + m;
                    if (r < K) store_rounded<CT>(a.C, (int64_t)r * a.ldC + col0 + j, acc[m]);
                }
            }
        }
        __syncthreads();
    }
}

// Companion block of head blockIdx.x, rows (Q: rows of W_q; O: window rows) blockIdx.y, + gridDim.y, ...
//   Q:  side_out[s][h n + i] = sum_j W_q[s][h n + j] W[off + i][h n + j]        (B_qk^h = W_q^h W_h[B,:]^T)
//   O:  side_out[h n + i][m] = sum_j W[off + i][h n + j] W_o[h n + j][m]        (B_vo^h = W_h[B,:] W_o^h)
template <typename WT, typename CT>
__global__ __launch_bounds__(kPrepThreads) void side_kernel(const PrepArgs a)
{
    // Q: out[s, i] = sum_j W_q[s, col0 + j] W[off + i, col0 + j]      (d_side x d_h per head)
    // O: out[i, m] = sum_j W[off + i, col0 + j] W_o[col0 + j, m]      (d_h x d_side per head)
    // 64 x 64 output tiles, the contraction staged through LDS 16 at a time, 4 x 4 outputs per thread
    // (rows ty + 16 u, columns tx + 16 v); workgroup (head, part) takes tiles part, part + gridDim.y, ...
    // Each output is one sum in ascending j, whatever the grid.
    constexpr int TS = 64, KC = 16;
    __shared__ double As[TS][KC + 1];
    __shared__ double Bs[KC][TS + 1];
    const int n = a.d_h, h = blockIdx.x, t = threadIdx.x;
    const int off = window_start(a);
    if (off < 0) return;
    const int64_t col0 = (int64_t)h * n;
    const bool q = a.side_kind == BDA_SIDE_Q;
    const int R = q ? a.d_side : n, Cn = q ? n : a.d_side;
    auto w = [&](int i, int j) { return load_as_double<WT>(a.W, (int64_t)(off + i) * a.ldw + col0 + j); };
    const int tx = t % 16, ty = t / 16;
    const int tiles_c = (Cn + TS - 1) / TS, n_tiles = ((R + TS - 1) / TS) * tiles_c;
    for (int tile = blockIdx.y; tile < n_tiles; tile += gridDim.y) {
        const int r0 = (tile / tiles_c) * TS, c0 = (tile % tiles_c) * TS;
        double acc[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
        for (int j0 = 0; j0 < n; j0 += KC) {
            for (int e = t; e < TS * KC; e += kPrepThreads) {
                // both operands of Q and the first of O are contiguous along j; W_o is contiguous along m
                const int rr = e / KC, jj = e % KC;
                const bool okj = j0 + jj < n;
                As[rr][jj] = (okj && r0 + rr < R) ? (q ? load_as_double<WT>(a.side, (int64_t)(r0 + rr) * a.ld_side + col0 + j0 + jj)
                                                      : w(r0 + rr, j0 + jj)) : 0.0;
                if (q) Bs[jj][rr] = (okj && c0 + rr < Cn) ? w(c0 + rr, j0 + jj) : 0.0;
            }
            if (!q)
                for (int e = t; e < TS * KC; e += kPrepThreads) {
                    const int jj = e / TS, cc = e % TS;
                    Bs[jj][cc] = (j0 + jj < n && c0 + cc < Cn) ? load_as_double<WT>(a.side, (col0 + j0 + jj) * a.ld_side + c0 + cc) : 0.0;
                }
            __syncthreads();
#pragma unroll
            for (int jj = 0; jj < KC; ++jj) {
                double av[4], bv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) av[u] = As[ty + 16 * u][jj];
#pragma unroll
                for (int v = 0; v < 4; ++v) bv[v] = Bs[jj][tx + 16 * v];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[u][v] = fma(av[u], bv[v], acc[u][v]);
            }
            __syncthreads();
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = r0 + ty + 16 * u, c = c0 + tx + 16 * v;
                if (r < R && c < Cn) {
                    if (q) store_rounded<CT>(a.side_out, (int64_t)r * a.ld_side_out + col0 + c, acc[u][v]);
                    else store_rounded<CT>(a.side_out, (col0 + r) * a.ld_side_out + c, acc[u][v]);
                }
            }
    }
}

// Sum of squared reconstruction errors of the stored form of head blockIdx.x (Chat = C as stored, Bhat =
// the companion output as stored, kk = index of row / column k among those outside the window):
//   no companion   W_h[Bbar,:] - Chat A                                       (d_c - d_h) x d_h
//   Q              W_q^h W_h^T - [Bhat at the window columns, Bhat Chat^T]    d_side x d_c
//   O              W_h W_o^h - [Bhat at the window rows; Chat Bhat]           d_c x d_side
// In every case an element is  P1(r, c) - P2(r, c) - S(r, c)  with two products over the head width, of
// which one or the other (or S) is absent for some rows or columns.  The matrix is cut into 64 x 64
// tiles; workgroup (head, part) takes tiles part, part + gridDim.y, ...; the operands of a tile are
// staged through LDS 16 columns of the contraction at a time and every thread owns a 4 x 4 sub-grid
// of the tile (rows ty + 16 u, columns tx + 16 v).  Each thread adds its squares in a fixed order, the
// workgroup adds the 256 sums in thread order: the result does not depend on scheduling.
template <typename WT, typename CT>
__global__ __launch_bounds__(kPrepThreads) void residual_kernel(const PrepArgs a)
{
    constexpr int TS = 64, KC = 16;
    __shared__ double As[TS][KC + 1];
    __shared__ double Bs[KC][TS + 1];
    __shared__ double red[kPrepThreads];
    const int n = a.d_h, h = blockIdx.x, t = threadIdx.x, d_c = a.d_c, K = d_c - n;
    const int off = window_start(a);
    const int64_t col0 = (int64_t)h * n;
    const int kind = a.side_kind;
    const int R = kind == BDA_SIDE_Q ? a.d_side : kind == BDA_SIDE_O ? d_c : K;
    const int Cn = kind == BDA_SIDE_Q ? d_c : kind == BDA_SIDE_O ? a.d_side : n;
    auto w = [&](int k, int j) { return load_as_double<WT>(a.W, (int64_t)k * a.ldw + col0 + j); };
    auto chat = [&](int kk, int i) { return load_as_double<CT>(a.C, (int64_t)kk * a.ldC + col0 + i); };
    auto in_window = [&](int k) { return k >= off && k < off + n; };
    auto outside_index = [&](int k) { return k < off ? k : k - n; };
    // first product: P1(r, c) = sum_j a1(r, j) b1(j, c)
    auto a1 = [&](int r, int j) -> double {
        if (r >= R) return 0.0;
        if (kind == BDA_SIDE_Q) return load_as_double<WT>(a.side, (int64_t)r * a.ld_side + col0 + j);
        if (kind == BDA_SIDE_O) return w(r, j);
        return 0.0;
    };
    auto b1 = [&](int j, int c) -> double {
        if (c >= Cn) return 0.0;
        if (kind == BDA_SIDE_Q) return w(c, j);
        if (kind == BDA_SIDE_O) return load_as_double<WT>(a.side, (col0 + j) * a.ld_side + c);
        return 0.0;
    };
    // second product: P2(r, c) = sum_i a2(r, i) b2(i, c), absent at the window's columns (Q) / rows (O)
    auto a2 = [&](int r, int i) -> double {
        if (r >= R) return 0.0;
        if (kind == BDA_SIDE_Q) return load_as_double<CT>(a.side_out, (int64_t)r * a.ld_side_out + col0 + i);
        if (kind == BDA_SIDE_O) return in_window(r) ? 0.0 : chat(outside_index(r), i);
        return chat(r, i);
    };
    auto b2 = [&](int i, int c) -> double {
        if (c >= Cn) return 0.0;
        if (kind == BDA_SIDE_Q) return in_window(c) ? 0.0 : chat(outside_index(c), i);
        if (kind == BDA_SIDE_O) return load_as_double<CT>(a.side_out, (col0 + i) * a.ld_side_out + c);
        return w(off + i, c);
    };
    // what stands alone: minus Bhat at the window (Q, O); plus the row of W_h itself (no companion)
    auto lone = [&](int r, int c) -> double {
        if (r >= R || c >= Cn) return 0.0;
        if (kind == BDA_SIDE_Q) return in_window(c) ? -load_as_double<CT>(a.side_out, (int64_t)r * a.ld_side_out + col0 + (c - off)) : 0.0;
        if (kind == BDA_SIDE_O) return in_window(r) ? -load_as_double<CT>(a.side_out, (col0 + (r - off)) * a.ld_side_out + c) : 0.0;
        return w(r < off ? r : r + n, c);
    };
    const int tx = t % 16, ty = t / 16;
    const int tiles_c = (Cn + TS - 1) / TS, n_tiles = ((R + TS - 1) / TS) * tiles_c;
    double r2 = 0.0;
    if (off >= 0) {
        for (int tile = blockIdx.y; tile < n_tiles; tile += gridDim.y) {
            const int r0 = (tile / tiles_c) * TS, c0 = (tile % tiles_c) * TS;
            double acc[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
            for (int pass = (kind == BDA_SIDE_NONE ? 1 : 0); pass < 2; ++pass) {
                for (int j0 = 0; j0 < n; j0 += KC) {
                    for (int e = t; e < TS * KC; e += kPrepThreads) {
                        const int rr = e / KC, jj = e % KC;
                        const bool ok = j0 + jj < n;
                        As[rr][jj] = !ok ? 0.0 : pass == 0 ? a1(r0 + rr, j0 + jj) : -a2(r0 + rr, j0 + jj);
                        Bs[jj][rr] = !ok ? 0.0 : pass == 0 ? b1(j0 + jj, c0 + rr) : b2(j0 + jj, c0 + rr);
                    }
                    __syncthreads();
#pragma unroll
                    for (int jj = 0; jj < KC; ++jj) {
                        double av[4], bv[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) av[u] = As[ty + 16 * u][jj];
#pragma unroll
                        for (int v = 0; v < 4; ++v) bv[v] = Bs[jj][tx + 16 * v];
#pragma unroll
                        for (int u = 0; u < 4; ++u)
#pragma unroll
                            for (int v = 0; v < 4; ++v) acc[u][v] = fma(av[u], bv[v], acc[u][v]);
                    }
                    __syncthreads();
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const double d = acc[u][v] + lone(r0 + ty + 16 * u, c0 + tx + 16 * v);
                    r2 += d * d;
                }
        }
    }
    red[t] = r2;
    __syncthreads();
    if (t == 0) {
        double sum = 0.0;
        for (int i = 0; i < kPrepThreads; ++i) sum += red[i];
        a.partials[((size_t)a.cand * a.H + h) * a.n_parts + blockIdx.y] = sum;
    }
}

struct SelectArgs {
    double* partials;           // (a head's first part is overwritten with the root of its sum)
    const int* cand_singular;
    int* basis_offset_out;
    double* resid_out;           // NULL or 3 doubles: first window, last window, chosen window
    int n_cand, H, n_parts, d_c, d_h;
    int offs[kMaxCandidates];
};

// One workgroup.  Every sum is taken by one thread in a fixed order - a head's parts in order, a candidate's
// heads in order, the candidates in order - so the result does not depend on how the work is spread: first
// a thread per (candidate, head) adds that head's parts and leaves the root in the first part's place (the
// partial sums are the call's own workspace), then a thread per candidate takes the mean over the heads,
// then one thread compares the candidates.
constexpr int kSelectThreads = 256;
__global__ __launch_bounds__(kSelectThreads) void select_kernel(const SelectArgs a)
{
    __shared__ double s_mean[kMaxCandidates];
    const int t = threadIdx.x;
    if (a.partials) {
        for (int e = t; e < a.n_cand * a.H; e += kSelectThreads) {
            double* part = a.partials + (size_t)e * a.n_parts;
            double s = 0.0;
            for (int p = 0; p < a.n_parts; ++p) s += part[p];
            part[0] = sqrt(s);
        }
    }
    __syncthreads();
    for (int ci = t; ci < a.n_cand; ci += kSelectThreads) {
        double mean = 0.0;
        if (a.partials) {
            for (int h = 0; h < a.H; ++h) mean += a.partials[((size_t)ci * a.H + h) * a.n_parts];
            mean /= a.H;
        }
        s_mean[ci] = mean;
    }
    __syncthreads();
    if (t != 0) return;
    const double inf = __builtin_huge_val(), nan = __builtin_nan("");
    double best = inf, r_first = nan, r_last = nan;
    int best_off = -1;
    for (int ci = 0; ci < a.n_cand; ++ci) {
        const bool singular = a.cand_singular[ci] != 0;
        double mean = s_mean[ci];
        if (singular || mean != mean) mean = inf;
        if (a.offs[ci] == 0) r_first = mean;
        if (a.offs[ci] == a.d_c - a.d_h) r_last = mean;
        const bool take = best_off < 0 ? !singular : mean < best;
        if (take) { best = mean; best_off = a.offs[ci]; }
    }
    *a.basis_offset_out = best_off;
    if (a.resid_out) { a.resid_out[0] = r_first; a.resid_out[1] = r_last; a.resid_out[2] = best; }
}

__global__ void fill_int_kernel(int* p, int n, int v)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

int check_launch(const char* what)
{
    const hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "bda_prepare_device: %s: %s", what, hipGetErrorString(err));
}

template <typename WT, typename CT>
int launch_prepare(PrepArgs a, int batch, hipStream_t st)
{
    const int n = a.d_h;
    const bool big = n > kPrepLdsDh;
    const size_t stage = (size_t)(kPrepRows * n > kPrepThreads ? kPrepRows * n : kPrepThreads);
    const size_t lds = ((big ? 0 : (size_t)n * (n + 1)) + stage) * sizeof(double);
    const void* kern = big ? (const void*)prepare_kernel<WT, CT, true> : (const void*)prepare_kernel<WT, CT, false>;
    hipError_t err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return fail(BDA_EHIP, "bda_prepare_device: LDS size %zu: %s", lds, hipGetErrorString(err));
    const int per_launch = big ? batch : a.H;
    // workgroups per head (the block in LDS only: a block in the workspace belongs to one workgroup): up to
    // 64 per launch, at most one per row block.  More shorten a lone call a little further (16 heads x 16:
    // 52.6 ms for a layer's offset searches against 54.8) but fill every compute unit with redundant
    // inversions, and then calls on other streams no longer run beside this one (measured).
    const int row_blocks = (a.d_c - n + kPrepRows - 1) / kPrepRows;
    int per_head = big ? 1 : 64 / a.H;
    per_head = per_head < 1 ? 1 : per_head > row_blocks ? (row_blocks < 1 ? 1 : row_blocks) : per_head;
    for (int h0 = 0; h0 < a.H; h0 += per_launch) {
        a.h0 = h0;
        const int heads = a.H - h0 < per_launch ? a.H - h0 : per_launch;
        if (big) hipLaunchKernelGGL((prepare_kernel<WT, CT, true>), dim3(heads), dim3(kPrepThreads), lds, st, a);
        else hipLaunchKernelGGL((prepare_kernel<WT, CT, false>), dim3(heads, per_head), dim3(kPrepThreads), lds, st, a);
        if (int rc = check_launch("prepare kernel")) return rc;
    }
    return BDA_OK;
}

// What a call needs beyond its inputs and outputs, and where it lies in the workspace.
struct Plan {
    int n_cand, n_parts, batch;
    bool want_resid, big;
    size_t flags_bytes, partial_bytes, mat_bytes_per_head;
    int offs[kMaxCandidates];
};

int make_plan(const char* fn, int d_c, int H, int d_h, int mode, int explicit_offset, bool resid_wanted, Plan& p)
{
    const int last = d_c - d_h;
    p.n_cand = 0;
    switch (mode) {
    case BDA_BASIS_FIRST: p.offs[p.n_cand++] = 0; break;
    case BDA_BASIS_LAST: p.offs[p.n_cand++] = last; break;
    case BDA_BASIS_RESIDUAL_MIN: p.offs[p.n_cand++] = 0; p.offs[p.n_cand++] = last; break;
    case BDA_BASIS_OFFSET_SEARCH:
        if (last / 16 + 2 > kMaxCandidates) return fail(BDA_EINVAL, "%s: more than %d candidate windows", fn, kMaxCandidates);
        for (int o = 0; o <= last; o += 16) p.offs[p.n_cand++] = o;
        if (last % 16) p.offs[p.n_cand++] = last;
        break;
    case BDA_BASIS_EXPLICIT:
        if (explicit_offset < 0 || explicit_offset > last) return fail(BDA_EINVAL, "%s: basis_offset %d outside [0, %d]", fn, explicit_offset, last);
        p.offs[p.n_cand++] = explicit_offset;
        break;
    default: return fail(BDA_EINVAL, "%s: bad basis mode %d", fn, mode);
    }
    p.want_resid = p.n_cand > 1 || resid_wanted;
    p.big = d_h > kPrepLdsDh;
    int parts = 1024 / H;
    p.n_parts = parts < 1 ? 1 : parts > kMaxParts ? kMaxParts : parts;
    p.flags_bytes = kMaxCandidates * sizeof(int);
    p.partial_bytes = p.want_resid ? (((size_t)p.n_cand * H * p.n_parts * sizeof(double) + 255) & ~(size_t)255) : 0;
    p.mat_bytes_per_head = p.big ? (size_t)d_h * d_h * sizeof(double) : 0;
    p.batch = 0;
    return BDA_OK;
}

struct PrepCall {
    const void* W; int64_t ldw; int w_dtype; int d_c, H, d_h;
    const void* side; int64_t ld_side; int d_side; int side_kind;
    int mode, explicit_offset;
    void* C; int64_t ldC; void* side_out; int64_t ld_side_out; int c_dtype;
    int* basis_offset_out; double* resid_out; int* singular_head;
};

template <typename WT, typename CT>
int run_prepare(const PrepCall& c, const Plan& p, unsigned char* ws, hipStream_t st)
{
    int* flags = (int*)ws;
    double* partials = p.want_resid ? (double*)(ws + p.flags_bytes) : nullptr;
    double* mat = p.big ? (double*)(ws + p.flags_bytes + p.partial_bytes) : nullptr;
    PrepArgs a{};
    a.W = c.W; a.side = c.side; a.C = c.C; a.side_out = c.side_out;
    a.status = c.singular_head;
    a.cand_singular = ws ? flags : nullptr;
    a.partials = partials; a.mat = mat;
    a.ldw = c.ldw; a.ld_side = c.ld_side; a.ldC = c.ldC; a.ld_side_out = c.ld_side_out;
    a.d_c = c.d_c; a.H = c.H; a.d_h = c.d_h; a.d_side = c.d_side; a.side_kind = c.side_kind;
    a.n_parts = p.n_parts;
    const bool multi = p.n_cand > 1;
    int side_parts = 1;                      // workgroups per head of the companion kernel: its 64 x 64 tiles, at most 64
    if (c.side_kind != BDA_SIDE_NONE) {
        const int64_t tiles = (int64_t)((c.d_side + 63) / 64) * ((c.d_h + 63) / 64);
        side_parts = (int)(tiles < 64 ? tiles : 64);
    }
    if (ws) {
        hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(kMaxCandidates), 0, st, flags, kMaxCandidates, 0);
        if (int rc = check_launch("fill kernel")) return rc;
    }
    for (int ci = 0; ci < p.n_cand; ++ci) {
        a.off = p.offs[ci];
        a.off_ptr = nullptr;
        a.cand = ci;
        a.status = multi ? nullptr : c.singular_head;      // during a search a singular window is just a bad candidate
        if (int rc = launch_prepare<WT, CT>(a, p.batch, st)) return rc;
        if (c.side_kind != BDA_SIDE_NONE) {
            hipLaunchKernelGGL((side_kernel<WT, CT>), dim3(c.H, side_parts), dim3(kPrepThreads), 0, st, a);
            if (int rc = check_launch("companion kernel")) return rc;
        }
        if (p.want_resid) {
            hipLaunchKernelGGL((residual_kernel<WT, CT>), dim3(c.H, p.n_parts), dim3(kPrepThreads), 0, st, a);
            if (int rc = check_launch("residual kernel")) return rc;
        }
    }
    if (p.want_resid) {
        SelectArgs s{};
        s.partials = partials; s.cand_singular = flags; s.basis_offset_out = c.basis_offset_out; s.resid_out = c.resid_out;
        s.n_cand = p.n_cand; s.H = c.H; s.n_parts = p.n_parts; s.d_c = c.d_c; s.d_h = c.d_h;
        for (int i = 0; i < p.n_cand; ++i) s.offs[i] = p.offs[i];
        hipLaunchKernelGGL(select_kernel, dim3(1), dim3(kSelectThreads), 0, st, s);
        if (int rc = check_launch("select kernel")) return rc;
    } else if (c.basis_offset_out) {
        hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(64), 0, st, c.basis_offset_out, 1, p.offs[0]);
        if (int rc = check_launch("fill kernel")) return rc;
    }
    if (multi) {
        // the chosen window once more, into the outputs for good (its start is read on the device)
        a.off = -1;
        a.off_ptr = c.basis_offset_out;
        a.cand = 0;
        a.cand_singular = nullptr;
        a.status = c.singular_head;
        if (int rc = launch_prepare<WT, CT>(a, p.batch, st)) return rc;
        if (c.side_kind != BDA_SIDE_NONE) {
            hipLaunchKernelGGL((side_kernel<WT, CT>), dim3(c.H, side_parts), dim3(kPrepThreads), 0, st, a);
            if (int rc = check_launch("companion kernel")) return rc;
        }
    }
    return BDA_OK;
}

template <typename WT>
int dispatch_c(const PrepCall& c, const Plan& p, unsigned char* ws, hipStream_t st)
{
    switch (c.c_dtype) {
    case BDA_F64: return run_prepare<WT, double>(c, p, ws, st);
    case BDA_F32: return run_prepare<WT, float>(c, p, ws, st);
    case BDA_F16: return run_prepare<WT, _Float16>(c, p, ws, st);
    case BDA_BF16: return run_prepare<WT, __bf16>(c, p, ws, st);
    default: return fail(BDA_EDTYPE, "bda_prepare_device: bad c_dtype %d", c.c_dtype);
    }
}

int dispatch_w(const PrepCall& c, const Plan& p, unsigned char* ws, hipStream_t st)
{
    switch (c.w_dtype) {
    case BDA_F64: return dispatch_c<double>(c, p, ws, st);
    case BDA_F32: return dispatch_c<float>(c, p, ws, st);
    case BDA_F16: return dispatch_c<_Float16>(c, p, ws, st);
    case BDA_BF16: return dispatch_c<__bf16>(c, p, ws, st);
    default: return fail(BDA_EDTYPE, "bda_prepare_device: bad w_dtype %d", c.w_dtype);
    }
}

// Argument checks shared by the entry points; fills the plan (without the batch size).
int check_call(const char* fn, const PrepCall& c, Plan& p)
{
    if (!c.W || !c.C) return fail(BDA_EINVAL, "%s: NULL W or C", fn);
    if (c.d_h <= 0 || c.d_c <= c.d_h || c.H <= 0) return fail(BDA_EINVAL, "%s: need 0 < d_h < d_c and H > 0", fn);
    if (c.d_h > kPrepMaxDh) return fail(BDA_EINVAL, "%s: d_h = %d exceeds %d (use bda_prepare)", fn, c.d_h, kPrepMaxDh);
    const int64_t N = (int64_t)c.H * c.d_h;
    if (c.ldw < N || c.ldC < N) return fail(BDA_EINVAL, "%s: leading dimension smaller than H d_h = %lld", fn, (long long)N);
    if (c.side_kind != BDA_SIDE_NONE) {
        if (c.side_kind != BDA_SIDE_Q && c.side_kind != BDA_SIDE_O) return fail(BDA_EINVAL, "%s: bad side_kind %d", fn, c.side_kind);
        if (!c.side || !c.side_out || c.d_side <= 0) return fail(BDA_EINVAL, "%s: companion asked for but side or side_out NULL or d_side <= 0", fn);
        const int64_t need = c.side_kind == BDA_SIDE_Q ? N : c.d_side;
        if (c.ld_side < need || c.ld_side_out < need) return fail(BDA_EINVAL, "%s: companion leading dimension too small (need %lld)", fn, (long long)need);
    }
    if (int rc = make_plan(fn, c.d_c, c.H, c.d_h, c.mode, c.explicit_offset, c.resid_out != nullptr, p)) return rc;
    if ((p.n_cand > 1 || c.resid_out) && !c.basis_offset_out) return fail(BDA_EINVAL, "%s: basis_offset_out is NULL", fn);
    return BDA_OK;
}

// Workspace bytes of a call: the flags, the residual partial sums, and (d_h > 128) `batch` basis blocks.
size_t workspace_need(const Plan& p, int batch) { return p.flags_bytes + p.partial_bytes + p.mat_bytes_per_head * (size_t)batch; }

int run_with_workspace(const char* fn, const PrepCall& c, Plan& p, void* workspace, size_t workspace_bytes, hipStream_t st)
{
    const bool needs = p.want_resid || p.big;
    if (!needs) return dispatch_w(c, p, nullptr, st);
    const size_t least = workspace_need(p, p.big ? 1 : 0);
    if (!workspace || workspace_bytes < least)
        return fail(BDA_EINVAL, "%s: workspace of %zu bytes, this call needs at least %zu", fn, workspace ? workspace_bytes : (size_t)0, least);
    if ((uintptr_t)workspace % 16) return fail(BDA_EINVAL, "%s: workspace not 16-byte aligned", fn);
    if (p.big) {
        const size_t heads = (workspace_bytes - p.flags_bytes - p.partial_bytes) / p.mat_bytes_per_head;
        p.batch = (int)(heads < (size_t)c.H ? heads : (size_t)c.H);
    }
    return dispatch_w(c, p, (unsigned char*)workspace, st);
}

// Address of the static scratch array on the current device; looked up once per device.
int static_scratch(const char* fn, unsigned char** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return fail(BDA_EHIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(err));
    if (dev < 0 || dev >= kMaxDevices) return fail(BDA_EINVAL, "%s: device index %d beyond %d", fn, dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !p) return fail(BDA_EHIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(err));
        ptrs[dev] = p;
    }
    *out = (unsigned char*)ptrs[dev];
    return BDA_OK;
}

}  // namespace
}  // namespace bda

using namespace bda;

extern "C" size_t bda_prepare_device_workspace_bytes(int d_c, int H, int d_h, bda_basis_mode mode, int want_residuals)
{
    clear_error();
    if (d_h <= 0 || d_c <= d_h || H <= 0 || d_h > kPrepMaxDh) return 0;
    Plan p;
    if (make_plan("bda_prepare_device_workspace_bytes", d_c, H, d_h, (int)mode, 0, want_residuals != 0, p)) return 0;
    if (!p.want_resid && !p.big) return 0;
    return workspace_need(p, p.big ? (H < 32 ? H : 32) : 0);
}

extern "C" int bda_prepare_device_ex(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                                     const void* side, int64_t ld_side, int d_side, bda_side side_kind,
                                     bda_basis_mode mode, int explicit_offset,
                                     void* C, int64_t ldC, void* side_out, int64_t ld_side_out, bda_dtype c_dtype,
                                     int* basis_offset_out, double* resid_out, int* singular_head,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    const PrepCall c{W, ldw, (int)w_dtype, d_c, H, d_h, side, ld_side, d_side, side ? (int)side_kind : (int)BDA_SIDE_NONE,
                     (int)mode, explicit_offset, C, ldC, side_out, ld_side_out, (int)c_dtype,
                     basis_offset_out, resid_out, singular_head};
    Plan p;
    if (int rc = check_call("bda_prepare_device_ex", c, p)) return rc;
    return run_with_workspace("bda_prepare_device_ex", c, p, workspace, workspace_bytes, (hipStream_t)stream);
}

extern "C" int bda_prepare_device(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                                  int basis_offset, void* C, int64_t ldC, bda_dtype c_dtype,
                                  int* singular_head, void* stream)
{
    clear_error();
    if (d_h > kPrepLdsDh) return fail(BDA_EINVAL, "bda_prepare_device: d_h = %d exceeds %d (bda_prepare_device_ex takes a workspace for up to %d)", d_h, kPrepLdsDh, kPrepMaxDh);
    const PrepCall c{W, ldw, (int)w_dtype, d_c, H, d_h, nullptr, 0, 0, (int)BDA_SIDE_NONE, (int)BDA_BASIS_EXPLICIT, basis_offset,
                     C, ldC, nullptr, 0, (int)c_dtype, nullptr, nullptr, singular_head};
    Plan p;
    if (int rc = check_call("bda_prepare_device", c, p)) return rc;
    return dispatch_w(c, p, nullptr, (hipStream_t)stream);
}

extern "C" int bda_prepare_device_static(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                                         const void* side, int64_t ld_side, int d_side, bda_side side_kind,
                                         bda_basis_mode mode, int explicit_offset,
                                         void* C, int64_t ldC, void* side_out, int64_t ld_side_out, bda_dtype c_dtype,
                                         int* basis_offset_out, double* resid_out, int* singular_head, void* stream)
{
    clear_error();
    const char* fn = "bda_prepare_device_static";
    const PrepCall c{W, ldw, (int)w_dtype, d_c, H, d_h, side, ld_side, d_side, side ? (int)side_kind : (int)BDA_SIDE_NONE,
                     (int)mode, explicit_offset, C, ldC, side_out, ld_side_out, (int)c_dtype,
                     basis_offset_out, resid_out, singular_head};
    Plan p;
    if (int rc = check_call(fn, c, p)) return rc;
    if (!p.want_resid && !p.big) return dispatch_w(c, p, nullptr, (hipStream_t)stream);
    const size_t least = workspace_need(p, p.big ? 1 : 0);
    if (least > kStaticScratchBytes)
        return fail(BDA_EINVAL, "%s: this call needs %zu bytes of scratch, the built-in scratch holds %zu: use bda_prepare_device_ex with a workspace",
                    fn, least, kStaticScratchBytes);
    unsigned char* ws = nullptr;
    if (int rc = static_scratch(fn, &ws)) return rc;
    return run_with_workspace(fn, c, p, ws, kStaticScratchBytes, (hipStream_t)stream);
}
