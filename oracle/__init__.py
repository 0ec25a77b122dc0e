"""TEST INFRASTRUCTURE -- plain fp64 CPU oracle for BD Attention's K/V up-projection path.

Nothing in the product may import this package: only `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py` do.  It shares no code with the GPU library and never calls it.

Two layers, both float64:

* Basis Decomposition on explicit matrices with numpy (`bd_window`: one candidate window, solve
  plus residual; `bd_assemble`: the matrix a BD pair stands for; `bd_decompose`: the best of the
  candidate windows; `attention_prepare_qk`, `attention_prepare_vo`: one window for all heads by
  the mean residual), covering Eq. bd_identity, Algorithms "BD Decomposition (Row)", "BD
  Reconstruction (Row)", "BD Attention Preparation (QK)" and Appendix "BD for VO in MHA".  They
  work on the d x d product matrices, so they are for small and medium sizes.
* The per-head closed form the product path is specified by (`prepare`, `prepare_lowrank`):
  C_h = W_h[Bbar,:] W_h[B,:]^{-1}, which follows from the column-first BD of W_q^h (W_k^h)^T
  (Eq. qk_bd_single) and the row-first BD of W_v^h W_o^h (Appendix "BD for VO in MHA"), and the
  run-time operators (`kv_project`, `dense_project`, `lowrank_linear`), which are C loops over the
  defining formulas in `bd_project.c`.
* The gradients of the K/V projection for BDA training (`kv_project_backward`): the chain rule
  applied head by head to steps 2-3 of Algorithm "BD Attention Inference", with numpy products.

Readings of the paper that the text leaves open are listed where they are applied.
All pins of this oracle live in tests/test_oracle_*.py; no function here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32, F16, BF16, F64 = 0, 1, 2, 3
FIRST, LAST, RESIDUAL_MIN, OFFSET_SEARCH, EXPLICIT = 0, 1, 2, 3, 4
SIDE_NONE, SIDE_Q, SIDE_O = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


# ------------------------------------------------------------------------------------------------
# building / loading the C part
# ------------------------------------------------------------------------------------------------
def build(force: bool = True) -> str:
    """Compile bd_project.c with gcc (OpenMP over token rows only)."""
    if force or not os.path.exists(_LIB_PATH):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
               os.path.join(_HERE, "bd_project.c"), "-o", _LIB_PATH]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB_PATH)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        i64 = ctypes.c_int64
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_kv_project.restype = None
        lib.oracle_kv_project.argtypes = [dp, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ip, ip, dp, i64, dp, i64]
        lib.oracle_dense_project.restype = None
        lib.oracle_dense_project.argtypes = [dp, i64, i64, ctypes.c_int, dp, i64, i64, dp, i64]
        lib.oracle_lowrank_linear.restype = None
        lib.oracle_lowrank_linear.argtypes = [dp, i64, i64, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, dp, dp, dp, i64, dp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


# ------------------------------------------------------------------------------------------------
# storage rounding used when a residual is evaluated "as stored" (the oracle's own copy)
# ------------------------------------------------------------------------------------------------
def round_store(x: np.ndarray, dtype: int) -> np.ndarray:
    """Value of x after one round-to-nearest-even conversion to `dtype`, as float64."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == F64:
        return x
    if dtype == F32:
        with np.errstate(over="ignore"):
            return x.astype(np.float32).astype(np.float64)
    if dtype == F16:
        with np.errstate(over="ignore"):                  # out-of-range values become +-inf
            return x.astype(np.float16).astype(np.float64)
    if dtype == BF16:
        _, e = np.frexp(x)
        s = np.maximum(e - 8, -133)
        y = np.ldexp(np.rint(np.ldexp(x, -s)), s)
        y = np.where(np.abs(y) >= 2.0 ** 128, np.copysign(np.inf, x), y)   # past the largest finite value: +-inf, as IEEE rounding overflows
        return np.where(np.isfinite(x), y, x)
    raise ValueError("dtype")


# ------------------------------------------------------------------------------------------------
# Basis Decomposition of a matrix for one candidate window, and the choice among candidates
# ------------------------------------------------------------------------------------------------
# Eq. bd_identity has four forms (row/column basis, first/last); all are "a contiguous window of r
# rows (columns) is the basis B, every other row (column) is a combination C of it".  One routine
# handles a window at any start; first-r is start 0, last-r is start m - r.  Algorithms "BD
# Decomposition (Row)" / "BD Reconstruction (Row)" and their column twins are this routine looped
# over the two (or more) candidate windows with the smallest Frobenius residual kept.
ROWS, COLS = 0, 1


def _combine(Bm: np.ndarray, R: np.ndarray) -> np.ndarray:
    """C with C @ Bm = R, Bm of full row rank (r x n, n >= r): least squares on the transposed
    system; exact when R lies in the row space of Bm, which BD guarantees."""
    sol, *_ = np.linalg.lstsq(Bm.T, R.T, rcond=None)
    return sol.T


def bd_assemble(Bm: np.ndarray, C: np.ndarray, off: int, axis: int) -> np.ndarray:
    """The matrix a BD pair stands for: window rows = B and the others = C B (axis ROWS), or window
    columns = B and the others = B C (axis COLS), the others keeping their ascending order."""
    r = Bm.shape[axis]
    total = r + C.shape[axis]
    rest = window_complement(total, r, off)
    if axis == ROWS:
        out = np.empty((total, Bm.shape[1]))
        out[off:off + r] = Bm
        out[rest] = C @ Bm
    else:
        out = np.empty((Bm.shape[0], total))
        out[:, off:off + r] = Bm
        out[:, rest] = Bm @ C
    return out


def bd_window(M: np.ndarray, r: int, off: int, axis: int):
    """BD of M with the r rows (columns) starting at `off` as basis.
    Returns (B, C, R): the basis, the coefficients of the other rows (columns), and the Frobenius
    residual ||M - assemble(B, C)|| -- zero in exact arithmetic when rank(M) <= r and the window
    is a basis (theorem of Section "Selection of Basis"), rounding noise scaled by the window's
    conditioning otherwise: the quantity Residual-min ranks windows by."""
    M = _c64(M)
    rest = window_complement(M.shape[axis], r, off)
    if axis == ROWS:
        Bm = M[off:off + r].copy()
        C = _combine(Bm, M[rest])
    else:
        Bm = M[:, off:off + r].copy()
        C = _combine(Bm.T, M[:, rest].T).T
    return Bm, C, float(np.linalg.norm(M - bd_assemble(Bm, C, off, axis)))


def first_last(total: int, r: int) -> List[int]:
    return [0, total - r]


def bd_decompose(M: np.ndarray, r: int, axis: int, offsets: Optional[Sequence[int]] = None):
    """Residual-min BD of one matrix: the candidate window (default: first-r and last-r) with the
    smallest residual; ties keep the earlier candidate (R_F <= R_L -> first).
    Returns (off, B, C, {off: R})."""
    M = _c64(M)
    offsets = first_last(M.shape[axis], r) if offsets is None else list(offsets)
    cands = {off: bd_window(M, r, off, axis) for off in offsets}
    best = min(offsets, key=lambda o: (cands[o][2], offsets.index(o)))
    return best, cands[best][0], cands[best][1], {o: cands[o][2] for o in offsets}


def _shared_window(mats: Sequence[np.ndarray], r: int, axis: int, offsets: Sequence[int]):
    """One window for all heads (Algorithm "BD Attention Preparation (QK)"): every head's matrix is
    decomposed for every candidate, the residuals are averaged over heads per candidate, and the
    candidate with the smallest mean is used by all heads (earlier candidate on ties).
    Returns (off, [(B, C) per head], {off: mean residual})."""
    per = {off: [bd_window(M, r, off, axis) for M in mats] for off in offsets}
    mean = {off: float(np.mean([p[2] for p in per[off]])) for off in offsets}
    best = min(offsets, key=lambda o: (mean[o], list(offsets).index(o)))
    return best, [(p[0], p[1]) for p in per[best]], mean


def attention_prepare_qk(Wq: np.ndarray, Wk: np.ndarray, n: int, offsets: Optional[Sequence[int]] = None):
    """QK preparation on the product matrices (Algorithm "BD Attention Preparation (QK)", Eq.
    qk_bd_single): head i's W_q^i (W_k^i)^T (d_q x d) gets a column BD B^i [I, C^i]; B^i replaces
    W_q^i and (C^i)^T replaces W_k^i.
    Wq: d_q x (n d_h) (the query side may read a different tensor, so its row count is its own),
    Wk: d x (n d_h).  Returns off, B_qk (d_q x n d_h), C_qk ((d - d_h) x n d_h, heads side by side),
    {off: mean residual}."""
    Wq, Wk = _c64(Wq), _c64(Wk)
    d_h = Wk.shape[1] // n
    d = Wk.shape[0]
    heads = [slice(i * d_h, (i + 1) * d_h) for i in range(n)]
    mats = [Wq[:, h] @ Wk[:, h].T for h in heads]
    offsets = first_last(d, d_h) if offsets is None else list(offsets)
    off, pairs, mean = _shared_window(mats, d_h, COLS, offsets)
    return off, np.hstack([Bm for Bm, _ in pairs]), np.hstack([C.T for _, C in pairs]), mean


def attention_prepare_vo(Wv: np.ndarray, Wo: np.ndarray, n: int, offsets: Optional[Sequence[int]] = None):
    """VO preparation (Appendix "BD for VO in MHA"): head i's W_v^i W_o^i (d x d_model) gets a row
    BD [I; C^i] B^i; C^i replaces W_v^i and B^i replaces W_o^i.
    Returns off, C_vo ((d - d_h) x n d_h), B_vo (n d_h x d_model), {off: mean residual}."""
    Wv, Wo = _c64(Wv), _c64(Wo)
    d_h = Wv.shape[1] // n
    d = Wv.shape[0]
    heads = [slice(i * d_h, (i + 1) * d_h) for i in range(n)]
    mats = [Wv[:, h] @ Wo[h, :] for h in heads]
    offsets = first_last(d, d_h) if offsets is None else list(offsets)
    off, pairs, mean = _shared_window(mats, d_h, ROWS, offsets)
    return off, np.hstack([C for _, C in pairs]), np.vstack([Bm for Bm, _ in pairs]), mean


# ------------------------------------------------------------------------------------------------
# per-head closed form (what the product's prepare call is specified to return)
# ------------------------------------------------------------------------------------------------
def window_complement(d_c: int, d_h: int, off: int) -> np.ndarray:
    """Bbar: latent columns outside the basis window [off, off + d_h), ascending."""
    return np.concatenate([np.arange(0, off), np.arange(off + d_h, d_c)]).astype(np.int64)


def candidate_offsets(mode: int, d_c: int, d_h: int, explicit_offset: int = 0) -> List[int]:
    """Basis windows a mode examines.  Offset search (Appendix "Residual-Min with Offset Search"):
    contiguous windows whose start is a multiple of 16; reading: no wrap-around, and the last-r
    window is always among the candidates so the search can only improve on Residual-min."""
    last = d_c - d_h
    if mode == FIRST:
        return [0]
    if mode == LAST:
        return [last]
    if mode == RESIDUAL_MIN:
        return [0, last]
    if mode == OFFSET_SEARCH:
        offs = list(range(0, last + 1, 16))
        if last not in offs:
            offs.append(last)
        return offs
    if mode == EXPLICIT:
        return [int(explicit_offset)]
    raise ValueError("mode")


def _prepare_window(W, d_c, n_heads, d_h, off, side, side_kind, store_dtype):
    """C, side_out and the mean stored-form residual for one basis window."""
    with np.errstate(invalid="ignore", over="ignore"):    # inf - inf in a residual -> NaN -> +inf
        return _prepare_window_impl(W, d_c, n_heads, d_h, off, side, side_kind, store_dtype)


def _prepare_window_impl(W, d_c, n_heads, d_h, off, side, side_kind, store_dtype):
    bbar = window_complement(d_c, d_h, off)
    K = d_c - d_h
    C = np.empty((K, n_heads * d_h))
    side_out = None if side is None else np.empty_like(side)
    resid = []
    for h in range(n_heads):
        cols = slice(h * d_h, (h + 1) * d_h)
        Wh = W[:, cols]
        A = Wh[off:off + d_h, :]                       # W_h[B, :], d_h x d_h
        Ch = np.linalg.solve(A.T, Wh[bbar, :].T).T     # C_h A = W_h[Bbar, :]
        C[:, cols] = Ch
        Chat = round_store(Ch, store_dtype)
        if side_kind == SIDE_Q:
            Wq = side[:, cols]                         # d_side x d_h
            Bq = Wq @ A.T                              # first-r columns of W_q^h (W_h)^T
            side_out[:, cols] = Bq
            Bhat = round_store(Bq, store_dtype)
            M = Wq @ Wh.T                              # d_side x d_c
            rec = np.empty_like(M)
            rec[:, off:off + d_h] = Bhat
            rec[:, bbar] = Bhat @ Chat.T
            resid.append(np.linalg.norm(M - rec))
        elif side_kind == SIDE_O:
            Wo = side[cols, :]                         # d_h x d_model
            Bo = A @ Wo                                # basis rows of W_h W_o^h
            side_out[cols, :] = Bo
            Bhat = round_store(Bo, store_dtype)
            M = Wh @ Wo
            rec = np.empty_like(M)
            rec[off:off + d_h, :] = Bhat
            rec[bbar, :] = Chat @ Bhat
            resid.append(np.linalg.norm(M - rec))
        else:
            # Algorithm "BD Decomposition (Row)" applied to W_h itself with r = d_h: the basis rows
            # reproduce themselves, the others are Chat A.
            resid.append(np.linalg.norm(Wh[bbar, :] - Chat @ A))
    r = float(np.mean(resid))
    if np.isnan(r):
        r = float("inf")
    return C, side_out, r


def prepare(W: np.ndarray, d_c: int, n_heads: int, d_h: int, side: Optional[np.ndarray] = None,
            side_kind: int = SIDE_NONE, mode: int = FIRST, explicit_offset: int = 0,
            store_dtype: int = F64):
    """Offline preparation of one projection (all heads share one basis window).

    W: d_c x (n_heads d_h) dense projection (W_k or W_v slices side by side).
    side: optional companion weight that absorbs the inverse: SIDE_Q -> W_q (d_side x n_heads d_h),
    replaced per head by W_q^h W_h[B,:]^T (= B_qk^h); SIDE_O -> W_o (n_heads d_h x d_model),
    replaced per head by W_h[B,:] W_o^h (= B_vo^h).

    Readings: (i) the residual that ranks windows is evaluated on what will be stored: C (and the
    side weight) rounded to `store_dtype`, the reconstruction error measured in float64 -- in pure
    float64 every window's residual is rounding noise and the choice would be arbitrary; (ii) with
    a side weight the residual is that of the product matrix, as in the preparation algorithm;
    without one it is that of W_h under the row algorithm; (iii) ties keep the earlier candidate
    (R_F <= R_L -> FIRST); a NaN residual counts as +inf.

    Returns C ((d_c - d_h) x n_heads d_h), side_out (or None), basis offset, {offset: residual}.
    """
    W = _c64(W)
    if side is not None:
        side = _c64(side)
    if side is None:
        side_kind = SIDE_NONE
    offs = candidate_offsets(mode, d_c, d_h, explicit_offset)
    best = None
    resid = {}
    for off in offs:
        C, s_out, r = _prepare_window(W, d_c, n_heads, d_h, off, side, side_kind, store_dtype)
        resid[off] = r
        if best is None or r < best[3]:
            best = (C, s_out, off, r)
    return best[0], best[1], best[2], resid


def prepare_lowrank(U: np.ndarray, V: np.ndarray, mode: int = FIRST, store_dtype: int = F64):
    """Section "BD for Linear Layer": column BD of W = U V (d_in x d_out, rank r).
    B = W[:, window] = U V[:, window] (d_in x r) replaces U; C = V[:, window]^{-1} V[:, rest]
    (r x (d_out - r)) replaces V.  Windows: first-r (offset 0) or last-r (offset d_out - r).
    The residual compares U V with B_hat [I, C_hat] (window-arranged), stored-form as in `prepare`.
    Returns Uprime, C, offset, {offset: residual}."""
    U, V = _c64(U), _c64(V)
    r, d_out = V.shape
    offs = candidate_offsets(mode if mode != OFFSET_SEARCH else RESIDUAL_MIN, d_out, r)
    best = None
    resid = {}
    for off in offs:
        rest = window_complement(d_out, r, off)
        Vb = V[:, off:off + r]
        Up = U @ Vb
        C = np.linalg.solve(Vb, V[:, rest])
        if len(offs) > 1:
            Uh, Ch = round_store(Up, store_dtype), round_store(C, store_dtype)
            Wfull = U @ V
            rec = np.empty_like(Wfull)
            rec[:, off:off + r] = Uh
            with np.errstate(invalid="ignore", over="ignore"):
                rec[:, rest] = Uh @ Ch
                res = float(np.linalg.norm(Wfull - rec))
            if np.isnan(res):
                res = float("inf")
        else:
            res = 0.0
        resid[off] = res
        if best is None or res < best[3]:
            best = (Up, C, off, res)
    return best[0], best[1], best[2], resid


# ------------------------------------------------------------------------------------------------
# run-time operators (C loops)
# ------------------------------------------------------------------------------------------------
def kv_project(c: np.ndarray, C: np.ndarray, d_h: int, H: Sequence[int],
               basis_offset: Sequence[int]) -> np.ndarray:
    """K' / V' for all heads of all groups: out = [c[:, B]]^{x n} + c[:, Bbar] C per group."""
    c, C = _c64(c), _c64(C)
    T, d_c = c.shape
    N = int(sum(H)) * d_h
    assert C.shape == (d_c - d_h, N), (C.shape, d_c, d_h, N)
    G = len(H)
    Ha = (ctypes.c_int * G)(*[int(v) for v in H])
    Oa = (ctypes.c_int * G)(*[int(v) for v in basis_offset])
    for o in basis_offset:
        assert 0 <= o <= d_c - d_h
    out = np.empty((T, N), dtype=np.float64)
    if T:
        _load().oracle_kv_project(_dptr(c), d_c, T, d_c, d_h, G, Ha, Oa, _dptr(C), N,
                                  _dptr(out), N)
    return out


def dense_project(c: np.ndarray, W: np.ndarray) -> np.ndarray:
    """K = X W_k (Algorithm "MHA Inference", steps 2-3)."""
    c, W = _c64(c), _c64(W)
    T, d_c = c.shape
    N = W.shape[1]
    assert W.shape[0] == d_c
    out = np.empty((T, N), dtype=np.float64)
    if T:
        _load().oracle_dense_project(_dptr(c), d_c, T, d_c, _dptr(W), N, N, _dptr(out), N)
    return out


def lowrank_linear(x: np.ndarray, Uprime: np.ndarray, C: np.ndarray,
                   basis_offset: int = 0) -> np.ndarray:
    """h = x B, y = [h, h C] (first-r) or [h C, h] (last-r); h is not rounded."""
    x, Uprime, C = _c64(x), _c64(Uprime), _c64(C)
    T, d_in = x.shape
    r = Uprime.shape[1]
    d_out = r + C.shape[1]
    assert Uprime.shape[0] == d_in and C.shape[0] == r
    assert basis_offset in (0, d_out - r)
    out = np.empty((T, d_out), dtype=np.float64)
    hbuf = np.empty((max(T, 1), r), dtype=np.float64)
    if T:
        _load().oracle_lowrank_linear(_dptr(x), d_in, T, d_in, r, d_out, int(basis_offset),
                                      _dptr(Uprime), _dptr(C), _dptr(out), d_out, _dptr(hbuf))
    return out


# ------------------------------------------------------------------------------------------------
# training: gradients of the K/V projection
# ------------------------------------------------------------------------------------------------
def kv_project_backward(c: np.ndarray, d_out: np.ndarray, C: np.ndarray, d_h: int,
                        H: Sequence[int], basis_offset: Sequence[int]
                        ) -> Tuple[np.ndarray, np.ndarray]:
    """Gradients of a loss through `kv_project` (Section "BDA Training Evaluation": C is a learnable
    parameter and gradients flow through the forward of Algorithm "BD Attention Inference").

    With out_h = c[:, B] + c[:, Bbar] C_h (steps 2-3) and d_out = dL/d out, head by head:
        dL/dC_h        = c[:, Bbar]^T d_out_h
        dL/dc[:, Bbar] += d_out_h C_h^T
        dL/dc[:, B]    += d_out_h            (the repeated basis slice: one copy per head)
    Returns (d_c, d_C) in float64, shaped like c and C."""
    c, d_out, C = _c64(c), _c64(d_out), _c64(C)
    T, d_c = c.shape
    N = int(sum(H)) * d_h
    assert C.shape == (d_c - d_h, N) and d_out.shape == (T, N)
    grad_c = np.zeros((T, d_c), dtype=np.float64)
    grad_C = np.zeros((d_c - d_h, N), dtype=np.float64)
    col = 0
    for n_heads, off in zip(H, basis_offset):
        assert 0 <= off <= d_c - d_h
        bbar = window_complement(d_c, d_h, int(off))
        c_bbar = c[:, bbar]
        for _ in range(int(n_heads)):
            head = slice(col, col + d_h)
            g_h = d_out[:, head]
            grad_C[:, head] = c_bbar.T @ g_h
            grad_c[:, bbar] += g_h @ C[:, head].T
            grad_c[:, off:off + d_h] += g_h
            col += d_h
    return grad_c, grad_C
