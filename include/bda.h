/*
 * bda.h -- C ABI of the Basis-Decomposed (BD) key/value up-projection library for AMD MI355X.
 *
 * BD Attention ("Accelerating Attention with Basis Decomposition") replaces, per attention head h,
 * the d_c x d_h key (or value) projection W_h by W_h W_h[B,:]^{-1}, where B is a contiguous window
 * of d_h latent dimensions shared by all heads.  The d_h basis rows become the identity, so only
 * the (d_c - d_h) x d_h block C_h is stored; the inverse is absorbed by the query (or output) side.
 * At run time each head computes  out_h = c[:, B] + c[:, Bbar] C_h.
 *
 * Conventions
 *   - All matrices are row-major; every leading dimension (ld*) counts ELEMENTS, not bytes.
 *   - "host" pointers are read/written by the CPU inside the call; "device" pointers are HIP device
 *     memory owned by the caller (for example PyTorch tensors).  The device entry points enqueue
 *     work on `stream` (a hipStream_t passed as void*, NULL = the default stream), never
 *     synchronise, never allocate and never free.  Small host arrays (H, basis_offset) are copied
 *     into the kernel arguments before the call returns.
 *   - Return value: BDA_OK (0) or a negative bda_status; bda_last_error() then describes the
 *     failure (thread-local).  No exception or abort crosses this boundary.
 *   - T = 0 (no tokens) is a successful no-op.  Outputs must not overlap inputs, except where a
 *     function says otherwise.
 */
#ifndef BDA_H
#define BDA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BDA_F32 = 0,
    BDA_F16 = 1,
    BDA_BF16 = 2,
    BDA_F64 = 3 /* only as store_dtype of the prepare calls: "do not round" */
} bda_dtype;

typedef enum {
    BDA_BASIS_FIRST = 0,         /* B = first d_h latent dimensions (row-first / col-first BD) */
    BDA_BASIS_LAST = 1,          /* B = last d_h latent dimensions */
    BDA_BASIS_RESIDUAL_MIN = 2,  /* first or last, whichever has the smaller mean residual */
    BDA_BASIS_OFFSET_SEARCH = 3, /* any window starting at a multiple of 16, or the last window */
    BDA_BASIS_EXPLICIT = 4       /* the caller names the window start */
} bda_basis_mode;

typedef enum {
    BDA_SIDE_NONE = 0,
    BDA_SIDE_Q = 1, /* companion is W_q (d_side x H d_h): head block h becomes W_q^h W_h[B,:]^T */
    BDA_SIDE_O = 2  /* companion is W_o (H d_h x d_side): head block h becomes W_h[B,:] W_o^h   */
} bda_side;

typedef enum {
    BDA_OK = 0,
    BDA_EINVAL = -1,    /* NULL pointer, bad dimension, ld too small, offset out of range, overlap */
    BDA_EALIGN = -2,    /* reserved: every alignment is currently served (slow path if needed)    */
    BDA_EDTYPE = -3,    /* dtype / out_dtype combination not supported                             */
    BDA_ESINGULAR = -4, /* a basis block W_h[B,:] is numerically singular (prepare only)           */
    BDA_EHIP = -5       /* a HIP runtime call failed                                               */
} bda_status;

#define BDA_MAX_GROUPS 8

/*
 * Offline preparation of one projection (Algorithm "BD Attention Preparation (QK)" for keys with
 * its query companion; Appendix "BD for VO in MHA" for values with their output companion;
 * Algorithm "BD Decomposition (Row)" for the window choice).  Host, float64, synchronous.
 *
 *   W         host, d_c x (H d_h), ld = ldw: dense projection, head h in columns [h d_h, (h+1) d_h).
 *   side      host or NULL: companion weight (see bda_side); d_side = its free dimension
 *             (rows of W_q, columns of W_o); ld = ld_side.
 *   mode, explicit_offset   how the basis window B = [offset, offset + d_h) is chosen.  The
 *             residual that ranks windows is the Frobenius reconstruction error of the BD form
 *             after C (and the companion) have been rounded to `store_dtype`, averaged over
 *             heads; ties keep the earlier candidate (first before last); NaN counts as +inf.
 *             With a companion the reconstructed matrix is the per-head product (W_q^h W_h^T or
 *             W_h W_o^h); without one it is W_h itself.
 *   C_out     host, (d_c - d_h) x (H d_h) contiguous float64: C_h = W_h[Bbar,:] W_h[B,:]^{-1},
 *             heads side by side (the layout of C_qk / C_vo in Algorithm "BD Attention Inference").
 *   side_out  host or NULL, same shape as `side`, contiguous float64.
 *   basis_offset_out   the chosen window start (0 = first, d_c - d_h = last).
 *   resid_out NULL or 3 doubles: mean residual of the first window, of the last window, and of
 *             the chosen window (NaN where a window was not evaluated).
 * Errors: BDA_EINVAL, BDA_ESINGULAR (message names the head and window).
 */
int bda_prepare(const double* W, int64_t ldw, int d_c, int H, int d_h,
                const double* side, int64_t ld_side, int d_side, bda_side side_kind,
                bda_basis_mode mode, int explicit_offset, bda_dtype store_dtype,
                double* C_out, double* side_out, int* basis_offset_out, double* resid_out);

/*
 * Offline preparation of a BD linear layer (Section "BD for Linear Layer"): column BD of
 * W = U V with U d_in x r, V r x d_out (both host, contiguous float64).
 *   Uprime_out  d_in x r:        U V[:, B]                    (replaces U)
 *   C_out       r x (d_out - r): V[:, B]^{-1} V[:, Bbar]      (replaces V)
 * mode: FIRST, LAST or RESIDUAL_MIN (B = first or last r output columns).  resid_out as above.
 */
int bda_prepare_lowrank(const double* U, const double* V, int d_in, int r, int d_out,
                        bda_basis_mode mode, bda_dtype store_dtype,
                        double* Uprime_out, double* C_out, int* basis_offset_out,
                        double* resid_out);

/*
 * bda_prepare on the GPU (Algorithm "BD Attention Preparation (QK)", Appendix "BD for VO in MHA",
 * Algorithm "BD Decomposition (Row)" and Appendix "Residual-Min with Offset Search" for the window
 * choice): C_h = W_h[Bbar,:] W_h[B,:]^{-1}, the companion blocks W_q^h W_h[B,:]^T or W_h[B,:] W_o^h,
 * and the window that minimises the mean residual of the stored form.  One workgroup per head,
 * float64 arithmetic (Gauss-Jordan inverse of the basis block with partial pivoting, then the
 * products); a search prepares every candidate window in turn into the outputs, measures the
 * reconstruction error of what was stored, selects on the device, and prepares the chosen window once
 * more.  Asynchronous on `stream`; nothing comes back to the host and nothing is allocated.
 *   W        device, d_c x (H d_h), ld = ldw, element type w_dtype (any bda_dtype).
 *   side     device or NULL: companion weight as in bda_prepare (W_q: d_side x H d_h; W_o: H d_h x
 *            d_side), ld = ld_side, element type w_dtype.
 *   mode, explicit_offset   as in bda_prepare (candidate windows, ranking, ties, NaN); a window with a
 *            numerically singular basis block in any head (pivot below d_h * 2^-52 * ||W_h[B,:]||_F)
 *            ranks last and is never chosen by a search.
 *   C        device, (d_c - d_h) x (H d_h), ld = ldC, element type c_dtype (any bda_dtype); every
 *            element is rounded once, to nearest even, from the float64 result - ready for
 *            bda_kv_project.
 *   side_out device (NULL without a companion), shape of `side`, ld = ld_side_out, element type
 *            c_dtype, rounded the same way.
 *   basis_offset_out   device int (may be NULL for a single-window mode without resid_out): the
 *            chosen window start once the call has run, or -1 if every candidate was singular (C
 *            and side_out then hold no result).
 *   resid_out   device, NULL or 3 doubles: mean residual of the first, the last and the chosen window
 *            (NaN where a window was not a candidate, +inf for a singular one).
 *   singular_head   device int or NULL; the caller zeroes it; after the call has run it holds
 *            1 + the largest index of a head whose basis block was singular in the window that was
 *            finally prepared, or stays 0.  C of such a head is not written.
 *   workspace, workspace_bytes   device memory for the call's partial results, 16-byte aligned: one
 *            flag per candidate window, the per-head partial sums of the residuals, and - for d_h >
 *            128, whose basis block does not fit the LDS - one d_h x d_h float64 block per head
 *            prepared at a time.  bda_prepare_device_workspace_bytes() gives a sufficient size
 *            (0: none needed, which is the case for a single-window mode without resid_out and d_h
 *            <= 128; workspace may then be NULL); any size from one block upwards works for d_h >
 *            128, more blocks meaning more heads per launch.  Contents before and after are
 *            meaningless; calls that share a workspace must not overlap.
 * d_h <= 256, at most 256 candidate windows.  Agrees with bda_prepare to a small multiple of
 * cond(W_h[B,:]) * 2^-53 (a different elimination order), not bit for bit; the chosen window agrees
 * unless two candidates' residuals are that close.
 * Errors: BDA_EINVAL (also: workspace too small, message says how much is needed), BDA_EDTYPE,
 * BDA_EHIP.
 */
size_t bda_prepare_device_workspace_bytes(int d_c, int H, int d_h, bda_basis_mode mode, int want_residuals);
int bda_prepare_device_ex(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                          const void* side, int64_t ld_side, int d_side, bda_side side_kind,
                          bda_basis_mode mode, int explicit_offset,
                          void* C, int64_t ldC, void* side_out, int64_t ld_side_out, bda_dtype c_dtype,
                          int* basis_offset_out, double* resid_out, int* singular_head,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * bda_prepare_device_ex for callers that cannot allocate device memory and have no workspace to pass
 * (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc): same arguments without
 * the workspace, same kernels, same results.  The call's partial results live in a fixed 8 MiB array
 * that is part of the library's device code: every GPU the library runs on holds it from the moment the
 * library's code is loaded there until the process ends.  The call allocates and frees nothing.
 * Limits: what bda_prepare_device_ex would need with one basis block (1 KiB + 8 bytes x candidate windows
 * x H x min(16, 1024 / H) + 8 d_h^2 for d_h > 128) must fit the 8 MiB; beyond that the call fails with
 * BDA_EINVAL and a message that names both sizes.  For d_h > 128 as many heads are prepared per launch as
 * basis blocks fit the rest of the array.  Every call on a GPU shares that GPU's array (it clears what it
 * needs cleared): calls that overlap on one GPU - two streams, two threads - race; keep them in order.
 */
int bda_prepare_device_static(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                              const void* side, int64_t ld_side, int d_side, bda_side side_kind,
                              bda_basis_mode mode, int explicit_offset,
                              void* C, int64_t ldC, void* side_out, int64_t ld_side_out, bda_dtype c_dtype,
                              int* basis_offset_out, double* resid_out, int* singular_head, void* stream);

/*
 * The short form: C only, for an explicit window (0 = first, d_c - d_h = last, or the offset a search
 * returned), d_h <= 128, no workspace.  Arguments as above.
 */
int bda_prepare_device(const void* W, int64_t ldw, bda_dtype w_dtype, int d_c, int H, int d_h,
                       int basis_offset, void* C, int64_t ldC, bda_dtype c_dtype,
                       int* singular_head, void* stream);

/*
 * Run-time BD projection, steps 2-3 of Algorithm "BD Attention Inference" (Eq. qk_bd_merge and
 * the V' equation of Appendix "BD for VO in MHA"), all heads of all groups in one launch:
 *
 *     out[t, col0_g + h d_h + j] = c[t, off_g + j] + sum_{k in Bbar_g} c[t, k] C[rank(k), col]
 *
 *   c       device, T x d_c, ld = ldc, element type `dtype`.
 *   G, H, basis_offset   host: G <= BDA_MAX_GROUPS groups (for example K blocks then V blocks);
 *           group g has H[g] heads and its own window start basis_offset[g] in [0, d_c - d_h];
 *           groups occupy consecutive output columns.
 *   C       device, (d_c - d_h) x N, N = sum_g H[g] d_h, ld = ldC, element type `dtype`;
 *           row i multiplies the i-th latent dimension outside the group's window (ascending).
 *   out     device, T x N, ld = ld_out, element type `out_dtype` (= dtype, or BDA_F32).
 * Products are accumulated in float32 (fp16/bf16 inputs use MFMA), the identity slice is added in
 * float32, and each output is rounded once (nearest even) when stored.  The MFMA path needs 16-byte
 * aligned pointers, ld's and basis offsets that are multiples of 8 elements, d_c a multiple of 8
 * and d_h a multiple of 32; anything else (and BDA_F32 inputs) runs a slower general kernel with
 * the same result contract.
 * Errors: BDA_EINVAL, BDA_EDTYPE, BDA_EHIP.
 */
int bda_kv_project(const void* c, int64_t ldc, int64_t T, int d_c, int d_h,
                   int G, const int* H, const int* basis_offset,
                   const void* C, int64_t ldC, void* out, int64_t ld_out,
                   bda_dtype dtype, bda_dtype out_dtype, void* stream);

/*
 * Dense comparator, steps 2-3 of Algorithm "MHA Inference": out = c W with the full d_c-long
 * contraction, from the same kernel family.  W: device, d_c x N, ld = ldW.
 */
int bda_dense_project(const void* c, int64_t ldc, int64_t T, int d_c,
                      const void* W, int64_t ldW, int64_t N,
                      void* out, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype,
                      void* stream);

/*
 * BD linear layer (Section "BD for Linear Layer"):  h = x Uprime,  out = [h, h C]  (basis_offset
 * = 0) or out = [h C, h] (basis_offset = d_out - r).  h is written to its r output columns in
 * `dtype` and the second product reads it back from there, so no workspace is needed.
 *   x device T x d_in (ldx); Uprime device d_in x r contiguous; C device r x (d_out - r)
 *   contiguous; out device T x d_out (ld_out); all of element type `dtype`.
 */
int bda_lowrank_linear(const void* x, int64_t ldx, int64_t T, int d_in, int r, int d_out,
                       int basis_offset, const void* Uprime, const void* C,
                       void* out, int64_t ld_out, bda_dtype dtype, void* stream);

/*
 * Gradients of bda_kv_project for BDA training (Section "BDA Training Evaluation": C replaces the
 * projection as the learnable parameter and gradients flow through steps 2-3 of Algorithm "BD
 * Attention Inference").  With d_out = dL/d out (T x N):
 *
 *     grad_c[t, l] = sum_g ( [l in window g] sum_h d_out[t, col0_g + h d_h + l - off_g]
 *                          + [l outside it]   sum_{n in group g} d_out[t, n] C[rank_g(l), n] )
 *     grad_C[i, n] = sum_t c[t, Bbar_g(i)] d_out[t, n]          (g = the group that owns column n)
 *
 *   c, C, G, H, basis_offset, T, d_c, d_h   as in bda_kv_project (element type `dtype`).
 *   d_out    device, T x N, ld = ld_dout, element type `dtype`.
 *   grad_c   device or NULL (skip; then C may be NULL), T x d_c, ld = ld_gc.
 *   grad_C   device or NULL (skip; then c may be NULL), (d_c - d_h) x N, ld = ld_gC.
 *            Both are OVERWRITTEN (not accumulated into), element type `grad_dtype` (= dtype, or
 *            BDA_F32).  With T = 0, grad_C is written with zeros and grad_c is not touched.
 * Each gradient is one launch on `stream`; products are accumulated in float32 (fp16/bf16 inputs use
 * MFMA; the head sum on the window is part of the same accumulation) and rounded once when stored.
 * The MFMA path needs 16-byte aligned pointers, ld's, d_c and basis offsets that are multiples of 8
 * and d_h a multiple of 32; anything else (and BDA_F32 inputs) runs slower general kernels with
 * the same result contract.  Gradients must not overlap the inputs or each other.
 * Errors: BDA_EINVAL, BDA_EDTYPE, BDA_EHIP.
 */
int bda_kv_project_backward(const void* c, int64_t ldc, const void* d_out, int64_t ld_dout,
                            const void* C, int64_t ldC, int64_t T, int d_c, int d_h,
                            int G, const int* H, const int* basis_offset,
                            void* grad_c, int64_t ld_gc, void* grad_C, int64_t ld_gC,
                            bda_dtype dtype, bda_dtype grad_dtype, void* stream);

/*
 * Optional packed layout of C for launches with a few tokens (Algorithm "BD Attention Inference", steps
 * 2-3, in the decode regime, where the call is a stream over the weights).  The canonical C - heads side
 * by side, the layout of C_qk / C_vo in the paper - stays the documented input of every other call;
 * packing is done once, when the weights are loaded.
 *   Layout: the N = sum_g H[g] d_h output columns are cut into slices of 32; slice s holds columns
 *   [32 s, 32 s + 32) of all d_c - d_h rows, row after row: element (k, j) of slice s is 16-bit element
 *   ((s (d_c - d_h) + k) * 32 + j) of the packed buffer.  A workgroup's part of C is then one contiguous
 *   block instead of a 64-byte piece out of every row.  Every group's width H[g] d_h must be a multiple
 *   of 32 (slices do not straddle groups); dtype BDA_F16 or BDA_BF16.
 * bda_packed_weights_bytes: size of the packed buffer ((d_c - d_h) N 2), 0 on bad arguments.
 * bda_pack_weights: device -> device, asynchronous on `stream`, allocates nothing; C and packed 16-byte
 *   aligned, ldC a multiple of 8, no overlap.
 * bda_kv_project_packed: bda_kv_project with `packed` in place of (C, ldC), for T <= 64 and shapes the
 *   few-token kernels take (16-byte aligned buffers; ldc, ld_out, d_c - d_h and the window starts multiples
 *   of 8; d_c - d_h <= 1536); same results as bda_kv_project bit for bit.  BDA_EINVAL otherwise (the
 *   message says to use the canonical call).
 */
size_t bda_packed_weights_bytes(int d_c, int d_h, int G, const int* H, bda_dtype dtype);
int bda_pack_weights(const void* C, int64_t ldC, int d_c, int d_h, int G, const int* H, bda_dtype dtype,
                     void* packed, void* stream);
int bda_kv_project_packed(const void* c, int64_t ldc, int64_t T, int d_c, int d_h,
                          int G, const int* H, const int* basis_offset, const void* packed,
                          void* out, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype, void* stream);

/*
 * The same three device calls with an explicit tile policy for this one call (tests, tuning and
 * benchmarks of the individual kernels; the plain entry points are these with policy 0).  Nothing
 * about the policy outlives the call and other threads' calls are unaffected.
 *   0 = automatic (the largest tile that still fills the chip),
 *   1 = 128 x 128 tokens x columns (register-staged MFMA kernel),
 *   2 = 256 x 256 streaming tiles, lean variant where it applies,
 *   3 = 256 x 256 with the general streaming kernel even where its lean variant would apply,
 *   4 = 128 x 256 with the lean streaming kernel where it applies (else as 2),
 *   5 = automatic, except that up to 128 tokens always take the wide-slice small-T kernel (128
 *       columns per workgroup up to 64 tokens, 64 columns above) wherever it applies
 *       (contraction d_c - d_h <= 384), whatever the output width,
 *   6 = 128 x 256 tiles with the two-workgroups-per-compute-unit streaming kernel wherever it
 *       applies (16-bit types, every group's width a multiple of 256, d_c - d_h a multiple of 32,
 *       d_h 64 or 128), else automatic,
 *   7 = 64 x 256 with the lean streaming kernel where it applies (else as 0 without the small-T
 *       kernels).
 * bda_kv_project_backward_ex honours 1 (128 x 128 output tiles) and treats the rest as automatic.
 * Results do not depend on the policy beyond which kernel computes them (the order of the float32
 * summation over k is the same for every tile shape).  Errors: as the plain call, plus BDA_EINVAL
 * for a policy outside 0 .. 7.
 */
int bda_kv_project_ex(const void* c, int64_t ldc, int64_t T, int d_c, int d_h,
                      int G, const int* H, const int* basis_offset,
                      const void* C, int64_t ldC, void* out, int64_t ld_out,
                      bda_dtype dtype, bda_dtype out_dtype, void* stream, int tile_policy);
int bda_dense_project_ex(const void* c, int64_t ldc, int64_t T, int d_c,
                         const void* W, int64_t ldW, int64_t N,
                         void* out, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype,
                         void* stream, int tile_policy);
int bda_kv_project_backward_ex(const void* c, int64_t ldc, const void* d_out, int64_t ld_dout,
                               const void* C, int64_t ldC, int64_t T, int d_c, int d_h,
                               int G, const int* H, const int* basis_offset,
                               void* grad_c, int64_t ld_gc, void* grad_C, int64_t ld_gC,
                               bda_dtype dtype, bda_dtype grad_dtype, void* stream, int tile_policy);

/*
 * Launch description: which kernel, tile shape and schedule bda_kv_project / bda_dense_project
 * would use for a problem, from the same validation and tile choice as the real calls.  Runs on the
 * host only (no GPU needed, nothing is launched); pointers are assumed 16-byte aligned.  For
 * tests, tuning and documentation of the launch-shape rules; `tile_policy` as in the *_ex calls.
 */
typedef enum {
    BDA_KERNEL_NONE = 0,    /* nothing to launch (T = 0) */
    BDA_KERNEL_GENERAL = 1, /* any type / shape / alignment: 64 x 64 tiles, float32 FMA */
    BDA_KERNEL_MFMA = 2,    /* register-staged MFMA kernel, 128 x 128 or 256 x 256 tiles */
    BDA_KERNEL_STREAM = 3,  /* streaming MFMA kernel (LDS DMA ring), general variant */
    BDA_KERNEL_LEAN = 4,    /* streaming MFMA kernel, lean variant (256-, 128- or 64-token tiles) */
    BDA_KERNEL_DECODE = 5,  /* few tokens (token tiles of up to 128): weight-streaming kernels; tile_columns tells 32-, 64- and 128-column slices apart */
    BDA_KERNEL_DUO = 6      /* streaming MFMA kernel, two 4-wave workgroups per compute unit, 128 x 256 tiles */
} bda_kernel_id;

typedef struct {
    int kernel;        /* bda_kernel_id */
    int tile_tokens;   /* output tile: tokens x columns */
    int tile_columns;
    int token_tiles;   /* tile grid */
    int column_tiles;
    int workgroups;    /* grid size */
    int threads;       /* per workgroup */
    int lds_bytes;     /* per workgroup */
    int rounds;        /* tiles (or super-tiles) a persistent workgroup works through at most */
    int tile_by_tile;  /* 1: dies take runs of single tiles; 0: super-tiles of super_m x super_n tiles */
    int super_m;
    int super_n;
} bda_launch_plan;

int bda_kv_project_plan(int64_t T, int d_c, int d_h, int G, const int* H, const int* basis_offset,
                        int64_t ldc, int64_t ldC, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype,
                        int tile_policy, bda_launch_plan* plan);

int bda_dense_project_plan(int64_t T, int d_c, int64_t N, int64_t ldc, int64_t ldW, int64_t ld_out,
                           bda_dtype dtype, bda_dtype out_dtype, int tile_policy, bda_launch_plan* plan);

/* Message of the last failing call on this thread; never NULL ("" if none). */
const char* bda_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int bda_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BDA_H */
