// GPU preparation of the BD projection weights:  C_h = W_h[Bbar,:] W_h[B,:]^{-1}  for an explicit basis
// window (Algorithm "BD Attention Preparation (QK)" / Appendix "BD for VO in MHA", the part that does
// not depend on the companion weight).  One workgroup per head, float64 throughout:
//   1. the d_h x d_h basis block is copied into LDS and inverted in place by Gauss-Jordan elimination
//      with partial (row) pivoting; the row interchanges are undone as column interchanges at the end;
//   2. the (d_c - d_h) rows outside the window are multiplied by the inverse, 16 rows at a time staged
//      through LDS, and stored rounded to the requested type.
// The host routine bda_prepare solves with an orthogonal factorisation instead of forming the inverse;
// the two agree to a small multiple of cond(W_h[B,:]) * 2^-53.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bda_internal.h"

namespace bda {
namespace {

struct PrepArgs {
    const void* W;
    void* C;
    int* status;
    int64_t ldw, ldC;
    int d_c, H, d_h, off;
};

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
constexpr int kPrepMaxDh = 128;
constexpr int kPrepRows = 16;                 // rows of W_h[Bbar,:] staged per pass

template <typename WT, typename CT>
__global__ __launch_bounds__(kPrepThreads) void prepare_kernel(const PrepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int n = a.d_h;
    const int ld = n + 1;                      // odd stride in doubles: a column walk touches all banks
    double* A = (double*)smem_raw;             // n x ld: the basis block, then its inverse
    double* R = A + (size_t)n * ld;            // kPrepRows x n staging, also scratch for the pivot search
    __shared__ int piv[kPrepMaxDh];
    __shared__ int s_pivot_row;
    __shared__ double s_pivot_val;
    __shared__ int s_singular;

    const int t = threadIdx.x;
    const int h = blockIdx.x;
    const int64_t col0 = (int64_t)h * n;

    // ---- basis block and its scale --------------------------------------------------------------
    double part = 0.0;
    for (int e = t; e < n * n; e += kPrepThreads) {
        const int i = e / n, j = e % n;
        const double v = load_as_double<WT>(a.W, (int64_t)(a.off + i) * a.ldw + col0 + j);
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
    const int row = t % kPrepMaxDh, half = t / kPrepMaxDh;       // thread -> (row, half of the columns)
    const int jn = (n + 1) / 2;
    const int j_lo = half * jn, j_hi = (half == 0) ? jn : n;
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
            for (int j = j_lo; j < j_hi; ++j) {
                const double cur = (j == k) ? 0.0 : A[row * ld + j];
                A[row * ld + j] = cur - f * A[k * ld + j];
            }
        }
        __syncthreads();
    }
    if (s_singular) {
        if (t == 0 && a.status) atomicMax(a.status, h + 1);
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
    const int K = a.d_c - n;
    const int j = t % kPrepMaxDh, rg = t / kPrepMaxDh;            // output column, row parity
    for (int r0 = 0; r0 < K; r0 += kPrepRows) {
        for (int e = t; e < kPrepRows * n; e += kPrepThreads) {
            const int i = e / n, c = e % n;
            const int r = r0 + i;
            const int src = r < a.off ? r : r + n;                 // rows outside the window, ascending
            R[i * n + c] = r < K ? load_as_double<WT>(a.W, (int64_t)src * a.ldw + col0 + c) : 0.0;
        }
        __syncthreads();
        if (j < n) {
            double acc[kPrepRows / 2];
#pragma unroll
            for (int m = 0; m < kPrepRows / 2; ++m) acc[m] = 0.0;
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
        }
        __syncthreads();
    }
}

template <typename WT, typename CT>
int launch_prepare(const PrepArgs& a, hipStream_t st)
{
    const int n = a.d_h;
    const size_t lds = ((size_t)n * (n + 1) + (size_t)(kPrepRows * n > kPrepThreads ? kPrepRows * n : kPrepThreads)) * sizeof(double);
    auto kern = prepare_kernel<WT, CT>;
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return fail(BDA_EHIP, "bda_prepare_device: LDS size %zu: %s", lds, hipGetErrorString(err));
    hipLaunchKernelGGL(kern, dim3(a.H), dim3(kPrepThreads), lds, st, a);
    err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "bda_prepare_device: kernel launch: %s", hipGetErrorString(err));
}

template <typename WT>
int dispatch_c(const PrepArgs& a, int c_dtype, hipStream_t st)
{
    switch (c_dtype) {
    case BDA_F64: return launch_prepare<WT, double>(a, st);
    case BDA_F32: return launch_prepare<WT, float>(a, st);
    case BDA_F16: return launch_prepare<WT, _Float16>(a, st);
    case BDA_BF16: return launch_prepare<WT, __bf16>(a, st);
    default: return fail(BDA_EDTYPE, "bda_prepare_device: bad c_dtype %d", c_dtype);
    }
}

}  // namespace
}  // namespace bda

using namespace bda;

extern "C" int bda_prepare_device(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                                  int basis_offset, void* C, int64_t ldC, bda_dtype c_dtype,
                                  int* singular_head, void* stream)
{
    clear_error();
    if (!W || !C) return fail(BDA_EINVAL, "bda_prepare_device: NULL pointer");
    if (d_h <= 0 || d_c <= d_h || H <= 0) return fail(BDA_EINVAL, "bda_prepare_device: need 0 < d_h < d_c and H > 0");
    if (d_h > kPrepMaxDh) return fail(BDA_EINVAL, "bda_prepare_device: d_h = %d exceeds %d (use bda_prepare)", d_h, kPrepMaxDh);
    const int64_t N = (int64_t)H * d_h;
    if (ldw < N || ldC < N) return fail(BDA_EINVAL, "bda_prepare_device: leading dimension smaller than H d_h = %lld", (long long)N);
    if (basis_offset < 0 || basis_offset > d_c - d_h) return fail(BDA_EINVAL, "bda_prepare_device: basis_offset %d out of range", basis_offset);
    PrepArgs a{W, C, singular_head, ldw, ldC, d_c, H, d_h, basis_offset};
    hipStream_t st = (hipStream_t)stream;
    switch (w_dtype) {
    case BDA_F64: return dispatch_c<double>(a, c_dtype, st);
    case BDA_F32: return dispatch_c<float>(a, c_dtype, st);
    case BDA_F16: return dispatch_c<_Float16>(a, c_dtype, st);
    case BDA_BF16: return dispatch_c<__bf16>(a, c_dtype, st);
    default: return fail(BDA_EDTYPE, "bda_prepare_device: bad w_dtype %d", w_dtype);
    }
}
