/*
 * TEST INFRASTRUCTURE -- fp64 CPU oracle for the run-time operators of BD Attention.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may call this.  It shares no code
 * with the GPU library.  Everything is written as the defining formula, one output element at a
 * time, in double precision, with no blocking or reordering; OpenMP only splits independent token
 * rows over host threads.
 *
 * Notation follows the paper: X (here `c`, the MLA latent) is L x d (here T x d_c), n heads of
 * width d_h, C_qk / C_vo are (d - d_h) x (n d_h) with head i in columns [i d_h, (i+1) d_h).
 */
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Steps 2-3 of Algorithm "BD Attention Inference" and the merged form of Eq. (qk_bd_merge) /
 * Appendix "BD for VO in MHA":
 *
 *     K' = [X_{:, B}]^{x n} + X_{:, Bbar} C
 *
 * generalised from "first d_h columns" to a contiguous basis window B = [off, off + d_h) (first:
 * off = 0; last: off = d - d_h; Appendix "Residual-Min with Offset Search": any offset), Bbar = the
 * remaining columns in ascending order.  Several groups (K blocks, then V blocks) each carry their
 * own window offset; group g owns H[g] heads and its output columns follow those of group g-1.
 *
 *   c   : T x d_c, row stride ldc
 *   C   : (d_c - d_h) x N, row stride ldC, N = sum_g H[g] d_h
 *   out : T x N, row stride ld_out
 */
void oracle_kv_project(const double *c, int64_t ldc, int64_t T, int d_c, int d_h,
                       int G, const int *H, const int *basis_offset,
                       const double *C, int64_t ldC, double *out, int64_t ld_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *x = c + t * ldc;
        int64_t col0 = 0;                       /* first output column of the current group */
        for (int g = 0; g < G; ++g) {
            const int off = basis_offset[g];
            for (int h = 0; h < H[g]; ++h) {
                for (int j = 0; j < d_h; ++j) {
                    const int64_t n = col0 + (int64_t)h * d_h + j;
                    double s = x[off + j];      /* the repeated identity slice X_{:, B} */
                    int kk = 0;                 /* row of C = rank of the latent column in Bbar */
                    for (int k = 0; k < d_c; ++k) {
                        if (k >= off && k < off + d_h)
                            continue;           /* basis columns are not multiplied */
                        s += x[k] * C[(int64_t)kk * ldC + n];
                        ++kk;
                    }
                    out[t * ld_out + n] = s;
                }
            }
            col0 += (int64_t)H[g] * d_h;
        }
    }
}

/*
 * Step 2 / 3 of Algorithm "MHA Inference": K = X W_k, the dense comparator.
 *   c : T x d_c (ldc),  W : d_c x N (ldW),  out : T x N (ld_out)
 */
void oracle_dense_project(const double *c, int64_t ldc, int64_t T, int d_c,
                          const double *W, int64_t ldW, int64_t N, double *out, int64_t ld_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int k = 0; k < d_c; ++k)
                s += c[t * ldc + k] * W[(int64_t)k * ldW + n];
            out[t * ld_out + n] = s;
        }
    }
}

/*
 * Section "BD for Linear Layer":  h <- x B,  y <- [h, h C]   (first-r), or y <- [h C, h] (last-r).
 *   x : T x d_in (ldx),  Bm : d_in x r,  C : r x (d_out - r),  out : T x d_out (ld_out)
 * basis_offset is the first output column that holds h (0 = first-r, d_out - r = last-r); the
 * other columns are filled, in ascending order, by the columns of h C.  h stays in double.
 * `hbuf` is caller-provided scratch of T x r doubles.
 */
void oracle_lowrank_linear(const double *x, int64_t ldx, int64_t T, int d_in, int r, int d_out,
                           int basis_offset, const double *Bm, const double *C,
                           double *out, int64_t ld_out, double *hbuf)
{
    const int64_t nc = (int64_t)d_out - r;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double *h = hbuf + t * (int64_t)r;
        for (int j = 0; j < r; ++j) {
            double s = 0.0;
            for (int k = 0; k < d_in; ++k)
                s += x[t * ldx + k] * Bm[(int64_t)k * r + j];
            h[j] = s;
        }
        for (int j = 0; j < r; ++j)
            out[t * ld_out + basis_offset + j] = h[j];
        for (int64_t m = 0; m < nc; ++m) {
            double s = 0.0;
            for (int j = 0; j < r; ++j)
                s += h[j] * C[(int64_t)j * nc + m];
            const int64_t col = (m < basis_offset) ? m : m + r;
            out[t * ld_out + col] = s;
        }
    }
}
