"""Pins of the fp64 oracle against what the paper and the mathematics fix (CPU only).

Each test names the statement it checks.  The pins are chosen so that a plausible mistake in the
oracle (dropped identity term, wrong sign, transposed operand, wrong window complement, wrong head
column range) fails at least one of them; test_planted_mistakes_are_caught shows that for a few.
"""
import itertools

import numpy as np
import pytest

import oracle
from conftest import read_golden

RNG = np.random.default_rng(1234)


def _rank_r(m, n, r, rng=RNG):
    return rng.standard_normal((m, r)) @ rng.standard_normal((r, n))


# ---------------------------------------------------------------- worked example / closed forms
def test_hand_example_3x2():
    g = read_golden("hand_example_3x2.txt")
    W = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    m = W.shape[0]
    _, C_F, _ = oracle.bd_window(W, 2, 0, oracle.ROWS)
    _, C_L, _ = oracle.bd_window(W, 2, m - 2, oracle.ROWS)
    np.testing.assert_allclose(C_F, [[g["first_c0"], g["first_c1"]]], atol=1e-12)
    np.testing.assert_allclose(C_L, [[g["last_c0"], g["last_c1"]]], atol=1e-12)
    # and through the per-head closed form with d_c = 3, d_h = 2, one head
    C, _, off, _ = oracle.prepare(W, 3, 1, 2, mode=oracle.FIRST)
    np.testing.assert_allclose(C, [[g["first_c0"], g["first_c1"]]], atol=1e-12)
    C, _, off, _ = oracle.prepare(W, 3, 1, 2, mode=oracle.LAST)
    assert off == 1
    np.testing.assert_allclose(C, [[g["last_c0"], g["last_c1"]]], atol=1e-12)


def test_memory_and_flop_closed_forms():
    """Paragraphs "Memory cost of BD" / "Computational cost of BD reconstruction"."""
    g = read_golden("paper_closed_forms.txt")
    m, n, r = 6, 5, 2
    W = _rank_r(m, n, r)
    _, B, C, _ = oracle.bd_decompose(W, r, oracle.ROWS)
    assert B.size + C.size == g["bd_memory_m6_n5_r2"] == r * (m + n - r)
    assert r * (m + n) == g["lowrank_memory_m6_n5_r2"]
    # count the multiply-adds the reconstruction performs: C (m-r x r) times B (r x n)
    assert 2 * C.shape[0] * C.shape[1] * B.shape[1] == g["bd_recon_flops_m6_n5_r2"]
    assert 2 * r * m * n == g["lowrank_recon_flops_m6_n5_r2"]


def test_kv_parameter_saving_25_percent():
    """Stored K/V parameters fall by d_h^2 per head; 25% at d_c = 512, d_h = 128."""
    g = read_golden("paper_closed_forms.txt")
    d_c, d_h, H = 512, 128, 3
    W = RNG.standard_normal((d_c, H * d_h)) * 0.02
    C, _, _, _ = oracle.prepare(W, d_c, H, d_h)
    assert W.size - C.size == H * d_h * d_h
    assert (W.size - C.size) / W.size == g["kv_param_saving_512_128"]


def test_flop_ratio_closed_form():
    g = read_golden("paper_closed_forms.txt")
    d, d_h = 512, 128
    dense = d_h * (2 * d - 1)
    bd = d_h * 2 * (d - d_h)
    assert dense == g["dense_flops_per_token_head_512_128"]
    assert bd == g["bd_flops_per_token_head_512_128"]
    assert dense / bd == g["flop_speedup_512_128"]
    assert round(dense / bd, 2) == g["flop_speedup_printed"]
    # the oracle's kv_project really multiplies (d - d_h) terms per output: count via C's shape
    C, _, _, _ = oracle.prepare(RNG.standard_normal((d, d_h)), d, 1, d_h)
    assert C.shape == (d - d_h, d_h)


def test_lowrank_linear_saving():
    g = read_golden("paper_closed_forms.txt")
    d_in, r, d_out = 4096, 1024, 11008
    low = r * (d_in + d_out)
    bd = d_in * r + r * (d_out - r)
    assert (low - bd) / low == pytest.approx(g["lowrank_linear_saving_4096_1024_11008"], rel=1e-15)
    U = RNG.standard_normal((12, 4))
    V = RNG.standard_normal((4, 9))
    Up, C, off, _ = oracle.prepare_lowrank(U, V)
    assert U.size + V.size - (Up.size + C.size) == 4 * 4


# ---------------------------------------------------------------- BD identities (Eq. bd_identity)
@pytest.mark.parametrize("m,n,r", [(7, 5, 2), (20, 33, 6), (64, 64, 16)])
def test_row_identities_and_reconstruction(m, n, r):
    W = _rank_r(m, n, r)
    off, B, C, resid = oracle.bd_decompose(W, r, oracle.ROWS)
    R_F, R_L = resid[0], resid[m - r]
    assert off in (0, m - r) and list(resid) == [0, m - r]
    assert R_F < 1e-10 * np.linalg.norm(W) and R_L < 1e-10 * np.linalg.norm(W)
    np.testing.assert_allclose(oracle.bd_assemble(B, C, off, oracle.ROWS), W, atol=1e-10 * np.linalg.norm(W))
    # explicit [I; C] B and [C; I] B forms
    I = np.eye(r)
    _, C_F, _ = oracle.bd_window(W, r, 0, oracle.ROWS)
    _, C_L, _ = oracle.bd_window(W, r, m - r, oracle.ROWS)
    np.testing.assert_allclose(np.vstack([I, C_F]) @ W[:r], W, atol=1e-9)
    np.testing.assert_allclose(np.vstack([C_L, I]) @ W[m - r:], W, atol=1e-9)


@pytest.mark.parametrize("m,n,r", [(5, 7, 2), (33, 20, 6)])
def test_col_identities(m, n, r):
    W = _rank_r(m, n, r)
    B_F, C_F, R_F = oracle.bd_window(W, r, 0, oracle.COLS)
    B_L, C_L, R_L = oracle.bd_window(W, r, n - r, oracle.COLS)
    I = np.eye(r)
    np.testing.assert_allclose(B_F @ np.hstack([I, C_F]), W, atol=1e-9)
    np.testing.assert_allclose(B_L @ np.hstack([C_L, I]), W, atol=1e-9)
    assert R_F < 1e-9 and R_L < 1e-9


@pytest.mark.parametrize("axis", [0, 1])
def test_interior_window_identity(axis):
    """A window inside the matrix (Appendix "Residual-Min with Offset Search"): the window's rows
    (columns) of the assembled matrix are B itself, the others are combinations of it, in ascending
    order around the window -- checked against an explicit permutation to the first-r form."""
    m, n, r, off = 11, 9, 3, 4
    W = _rank_r(m, n, r)
    B, C, R = oracle.bd_window(W, r, off, axis)
    assert R < 1e-10
    Wp = W if axis == 0 else W.T
    perm = np.concatenate([np.arange(off, off + r), np.arange(0, off), np.arange(off + r, Wp.shape[0])])
    Bp, Cp, _ = oracle.bd_window(Wp[perm], r, 0, 0)              # first-r form of the permuted matrix
    np.testing.assert_allclose(B if axis == 0 else B.T, Bp, atol=0)
    np.testing.assert_allclose(C if axis == 0 else C.T, Cp, atol=1e-10)


# ---------------------------------------------------------------- prepare: closed form vs literal
@pytest.mark.parametrize("mode", [oracle.FIRST, oracle.LAST])
def test_prepare_matches_literal_qk_algorithm(mode):
    d, n, d_h, d_q = 48, 3, 8, 40
    Wq = RNG.standard_normal((d_q, n * d_h))
    Wk = RNG.standard_normal((d, n * d_h))
    off = 0 if mode == oracle.FIRST else d - d_h
    C, Bq, got_off, _ = oracle.prepare(Wk, d, n, d_h, side=Wq, side_kind=oracle.SIDE_Q, mode=mode)
    assert got_off == off
    # literal: column BD of each product matrix
    for i in range(n):
        M = Wq[:, i * d_h:(i + 1) * d_h] @ Wk[:, i * d_h:(i + 1) * d_h].T
        B_lit, C_lit, _ = oracle.bd_window(M, d_h, off, oracle.COLS)
        np.testing.assert_allclose(Bq[:, i * d_h:(i + 1) * d_h], B_lit, rtol=1e-9, atol=1e-9)
        np.testing.assert_allclose(C[:, i * d_h:(i + 1) * d_h], C_lit.T, rtol=1e-7, atol=1e-8)


def test_prepare_matches_literal_vo_algorithm():
    d, n, d_h, d_model = 40, 2, 8, 56
    Wv = RNG.standard_normal((d, n * d_h))
    Wo = RNG.standard_normal((n * d_h, d_model))
    off_vo, C_vo, B_vo, _ = oracle.attention_prepare_vo(Wv, Wo, n)
    assert off_vo in (0, d - d_h)
    mode = oracle.FIRST if off_vo == 0 else oracle.LAST
    C, Bo, off, _ = oracle.prepare(Wv, d, n, d_h, side=Wo, side_kind=oracle.SIDE_O, mode=mode)
    assert off == off_vo
    np.testing.assert_allclose(C, C_vo, rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(Bo, B_vo, rtol=1e-9, atol=1e-9)


def _near_singular_window(Wk, heads, d_h, off, eps, rng):
    """Makes row off+1 of the given heads' blocks almost a copy of row off: the window at `off`
    becomes ill-conditioned (condition ~ 1/eps) for those heads only."""
    for h in heads:
        blk = Wk[:, h * d_h:(h + 1) * d_h]
        blk[off + 1] = blk[off] * (1 + eps) + eps * rng.standard_normal(d_h)


def test_qk_preparation_on_product_matrices():
    """Algorithm "BD Attention Preparation (QK)" as the oracle implements it on W_q^i (W_k^i)^T:
    outputs head by head against an independent per-head decomposition and against the per-head
    closed form (`prepare`), mean residuals against residuals recomputed here, the defining
    invariant Q'_i K'_i^T = Q_i K_i^T from its outputs alone, and the layouts of B_qk / C_qk."""
    rng = np.random.default_rng(77)
    d, n, d_h, d_q, T = 40, 3, 8, 28, 9
    Wq = rng.standard_normal((d_q, n * d_h))
    Wk = rng.standard_normal((d, n * d_h))
    off, B_qk, C_qk, mean = oracle.attention_prepare_qk(Wq, Wk, n)
    assert B_qk.shape == (d_q, n * d_h) and C_qk.shape == (d - d_h, n * d_h)
    assert list(mean) == [0, d - d_h] and off in mean
    bbar = [k for k in range(d) if not off <= k < off + d_h]
    resid = {0: [], d - d_h: []}
    for i in range(n):
        s = slice(i * d_h, (i + 1) * d_h)
        M = Wq[:, s] @ Wk[:, s].T
        # head i's block of the outputs, heads side by side in head order
        B_i, C_i, _ = oracle.bd_window(M, d_h, off, oracle.COLS)
        assert np.array_equal(B_qk[:, s], B_i) and np.array_equal(B_qk[:, s], M[:, off:off + d_h])
        assert np.array_equal(C_qk[:, s], C_i.T)
        # residuals of both windows, recomputed from the definition M ~ B [I, C] with a plain solve
        for o in resid:
            rest = [k for k in range(d) if not o <= k < o + d_h]
            Bm = M[:, o:o + d_h]
            Cm = np.linalg.lstsq(Bm, M[:, rest], rcond=None)[0]
            rec = np.empty_like(M)
            rec[:, o:o + d_h] = Bm
            rec[:, rest] = Bm @ Cm
            resid[o].append(np.linalg.norm(M - rec))
    for o in resid:
        assert mean[o] == pytest.approx(np.mean(resid[o]), rel=0.5, abs=1e-13)     # (noise-level values)
        assert mean[o] < 1e-10
    # the closed form agrees (same window)
    C, Bq, off2, _ = oracle.prepare(Wk, d, n, d_h, side=Wq, side_kind=oracle.SIDE_Q, mode=oracle.EXPLICIT, explicit_offset=off)
    np.testing.assert_allclose(B_qk, Bq, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(C_qk, C, rtol=1e-7, atol=1e-8)
    # and the scores are those of MHA
    X, Xq = rng.standard_normal((T, d)), rng.standard_normal((T, d_q))
    for i in range(n):
        s = slice(i * d_h, (i + 1) * d_h)
        Kp = X[:, off:off + d_h] + X[:, bbar] @ C_qk[:, s]
        got = (Xq @ B_qk[:, s]) @ Kp.T
        ref = (Xq @ Wq[:, s]) @ (X @ Wk[:, s]).T
        assert np.max(np.abs(got - ref)) <= 1e-9 * np.max(np.abs(ref))


def test_qk_preparation_window_is_chosen_by_the_mean_over_heads():
    """One window for all heads, by the MEAN residual: head 0's first window is made very
    ill-conditioned, the last windows of heads 1 and 2 mildly so.  Two of three heads prefer the
    first window and the last head does too, yet the mean prefers the last one; with the roles
    swapped the first one.  (A vote, the first head alone or the last head alone would each fail
    one of the two cases.)"""
    rng = np.random.default_rng(78)
    d, n, d_h = 40, 3, 8
    Wq = rng.standard_normal((d, n * d_h))
    for bad_strong, bad_mild in ((0, d - d_h), (d - d_h, 0)):
        Wk = rng.standard_normal((d, n * d_h))
        _near_singular_window(Wk, [0], d_h, bad_strong, 1e-11, rng)
        _near_singular_window(Wk, [1, 2], d_h, bad_mild, 1e-5, rng)
        off, _, _, mean = oracle.attention_prepare_qk(Wq, Wk, n)
        per_head = []
        for i in range(n):
            M = Wq[:, i * d_h:(i + 1) * d_h] @ Wk[:, i * d_h:(i + 1) * d_h].T
            per_head.append({o: oracle.bd_window(M, d_h, o, oracle.COLS)[2] for o in (0, d - d_h)})
        # the construction does what it says: head 0 is off by orders of magnitude, 1 and 2 mildly
        assert per_head[0][bad_strong] > 1e3 * max(per_head[1][bad_mild], per_head[2][bad_mild])
        assert per_head[1][bad_mild] > 10 * per_head[1][bad_strong]
        assert per_head[2][bad_mild] > 10 * per_head[2][bad_strong]
        assert off == bad_mild                       # the window that is only mildly bad wins on the mean
        assert mean[bad_mild] < mean[bad_strong]
        # the same through the VO twin (row BD of W_v^i W_o^i)
        Wo = rng.standard_normal((n * d_h, d))
        off_vo, _, _, mean_vo = oracle.attention_prepare_vo(Wk, Wo, n)
        assert off_vo == bad_mild and mean_vo[bad_mild] < mean_vo[bad_strong]


def test_preparation_tie_keeps_first_window_for_all_heads():
    # exact arithmetic on small integers: identity blocks at both ends of every head -> residuals 0
    d, n, d_h = 7, 2, 2
    mid = np.arange(6, dtype=np.float64).reshape(3, 2)
    Wk = np.hstack([np.vstack([np.eye(d_h), mid + h, np.eye(d_h)]) for h in range(n)])
    Wq = np.hstack([np.eye(d_h)] * n)
    off, B_qk, C_qk, mean = oracle.attention_prepare_qk(Wq, Wk, n)
    assert mean[0] == 0.0 and mean[d - d_h] == 0.0 and off == 0


# ---------------------------------------------------------------- prepare: what the maths fixes
@pytest.mark.parametrize("off", [0, 16, 48])
def test_basis_rows_become_identity(off):
    d_c, d_h, H = 64, 16, 2
    W = RNG.standard_normal((d_c, H * d_h)) * 0.125
    C, _, got, _ = oracle.prepare(W, d_c, H, d_h, mode=oracle.EXPLICIT, explicit_offset=off)
    assert got == off
    bbar = oracle.window_complement(d_c, d_h, off)
    for h in range(H):
        Wh = W[:, h * d_h:(h + 1) * d_h]
        A = Wh[off:off + d_h]
        full = Wh @ np.linalg.inv(A)            # transformed weight, all d_c rows
        np.testing.assert_allclose(full[off:off + d_h], np.eye(d_h), atol=1e-10)
        np.testing.assert_allclose(full[bbar], C[:, h * d_h:(h + 1) * d_h], atol=1e-9)
        # reconstruction [I; C] A = W_h
        rec = np.empty_like(Wh)
        rec[off:off + d_h] = A
        rec[bbar] = C[:, h * d_h:(h + 1) * d_h] @ A
        assert np.linalg.norm(rec - Wh) <= 1e-12 * max(1.0, np.linalg.norm(Wh)) * 1e2


def test_prepare_special_cases():
    d_c, d_h = 12, 4
    C0 = RNG.standard_normal((d_c - d_h, d_h))
    W = np.vstack([np.eye(d_h), C0])
    C, _, _, _ = oracle.prepare(W, d_c, 1, d_h)
    assert np.array_equal(C, C0)                 # W_h already [I; C0]
    alpha = 4.0
    W2 = np.vstack([alpha * np.eye(d_h), C0])
    C2, _, _, _ = oracle.prepare(W2, d_c, 1, d_h)
    np.testing.assert_allclose(C2, C0 / alpha, rtol=0, atol=1e-15)
    # last-r window with the identity at the bottom
    W3 = np.vstack([C0, np.eye(d_h)])
    C3, _, off, _ = oracle.prepare(W3, d_c, 1, d_h, mode=oracle.LAST)
    assert off == d_c - d_h and np.array_equal(C3, C0)


def test_window_complement_and_candidates():
    assert list(oracle.window_complement(8, 3, 0)) == [3, 4, 5, 6, 7]
    assert list(oracle.window_complement(8, 3, 5)) == [0, 1, 2, 3, 4]
    assert list(oracle.window_complement(8, 3, 2)) == [0, 1, 5, 6, 7]
    assert oracle.candidate_offsets(oracle.RESIDUAL_MIN, 512, 128) == [0, 384]
    offs = oracle.candidate_offsets(oracle.OFFSET_SEARCH, 512, 128)
    assert offs == list(range(0, 385, 16))
    assert oracle.candidate_offsets(oracle.OFFSET_SEARCH, 72, 16) == [0, 16, 32, 48, 56]


# ---------------------------------------------------------------- tag selection
def test_tag_tie_goes_to_first():
    # integer weights with identity blocks at both ends: both solves are exact, both residuals 0
    d_c, d_h = 10, 3
    mid = np.arange(12, dtype=np.float64).reshape(4, 3)
    W = np.vstack([np.eye(d_h), mid, np.eye(d_h)])
    C, _, off, resid = oracle.prepare(W, d_c, 1, d_h, mode=oracle.RESIDUAL_MIN, store_dtype=oracle.F64)
    assert resid[0] == 0.0 and resid[d_c - d_h] == 0.0
    assert off == 0
    off_m, _, _, r_m = oracle.bd_decompose(W, d_h, oracle.ROWS)
    assert r_m[0] <= r_m[d_c - d_h] and off_m == 0


@pytest.mark.parametrize("bad", ["first", "last"])
def test_ill_conditioned_window_loses(bad):
    d_c, d_h, H = 64, 16, 3
    W = RNG.standard_normal((d_c, H * d_h))
    # make the `bad` window nearly singular in every head: two almost equal basis rows
    r0 = 0 if bad == "first" else d_c - d_h
    for h in range(H):
        blk = W[:, h * d_h:(h + 1) * d_h]
        blk[r0 + 1] = blk[r0] * (1 + 1e-6) + 1e-7 * RNG.standard_normal(d_h)
    C, _, off, resid = oracle.prepare(W, d_c, H, d_h, mode=oracle.RESIDUAL_MIN, store_dtype=oracle.F16)
    assert off == (d_c - d_h if bad == "first" else 0)
    assert resid[r0] > 10 * resid[off]
    # offset search can only do as well or better
    _, _, off2, resid2 = oracle.prepare(W, d_c, H, d_h, mode=oracle.OFFSET_SEARCH, store_dtype=oracle.F16)
    assert resid2[off2] <= resid[off]
    assert off2 % 16 == 0 or off2 == d_c - d_h


def test_nan_residual_counts_as_inf():
    d_c, d_h = 8, 2
    W = RNG.standard_normal((d_c, d_h))
    W[3, 0] = np.nan            # a non-basis row for FIRST, also non-basis for LAST -> both inf -> FIRST
    _, _, off, resid = oracle.prepare(W, d_c, 1, d_h, mode=oracle.RESIDUAL_MIN)
    assert off == 0 and all(np.isinf(v) for v in resid.values())


# ---------------------------------------------------------------- inner-product preservation
@pytest.mark.parametrize("mode", [oracle.FIRST, oracle.LAST, oracle.EXPLICIT])
def test_scores_and_vo_preserved_tiny(mode):
    """Q'_h K'_h^T = Q_h K_h^T and V'_h B_vo^h = V_h W_o^h, brute force in float64 (tiny config)."""
    T, d_c, H, d_h, d_q, d_model = 64, 64, 2, 16, 24, 40
    rng = np.random.default_rng(0)
    c = rng.standard_normal((T, d_c))
    xq = rng.standard_normal((T, d_q))
    Wk = rng.standard_normal((d_c, H * d_h)) * 0.125
    Wv = rng.standard_normal((d_c, H * d_h)) * 0.125
    Wq = rng.standard_normal((d_q, H * d_h))
    Wo = rng.standard_normal((H * d_h, d_model))
    eo = 32
    Ck, Bq, offk, _ = oracle.prepare(Wk, d_c, H, d_h, Wq, oracle.SIDE_Q, mode, eo)
    Cv, Bo, offv, _ = oracle.prepare(Wv, d_c, H, d_h, Wo, oracle.SIDE_O, mode, eo)
    out = oracle.kv_project(c, np.hstack([Ck, Cv]), d_h, [H, H], [offk, offv])
    Kp, Vp = out[:, :H * d_h], out[:, H * d_h:]
    Qp = xq @ Bq
    Q, K, V = xq @ Wq, c @ Wk, c @ Wv
    for h in range(H):
        s = slice(h * d_h, (h + 1) * d_h)
        ref = Q[:, s] @ K[:, s].T
        got = Qp[:, s] @ Kp[:, s].T
        assert np.max(np.abs(got - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))
        ref_vo = V[:, s] @ Wo[s, :]
        got_vo = Vp[:, s] @ Bo[s, :]
        assert np.max(np.abs(got_vo - ref_vo)) <= 1e-10 * max(1.0, np.max(np.abs(ref_vo)))


# ---------------------------------------------------------------- kv_project
def _kv_reference_python(c, C, d_h, H, offs):
    """Pure-Python loops (tiny inputs only)."""
    T, d_c = c.shape
    N = sum(H) * d_h
    out = [[0.0] * N for _ in range(T)]
    col0 = 0
    for g, Hg in enumerate(H):
        off = offs[g]
        bbar = [k for k in range(d_c) if not (off <= k < off + d_h)]
        for t in range(T):
            for h in range(Hg):
                for j in range(d_h):
                    n = col0 + h * d_h + j
                    s = float(c[t, off + j])
                    for kk, k in enumerate(bbar):
                        s += float(c[t, k]) * float(C[kk, n])
                    out[t][n] = s
        col0 += Hg * d_h
    return np.array(out)


def test_kv_project_brute_force_tiny():
    rng = np.random.default_rng(5)
    T, d_c, d_h = 5, 11, 3
    H, offs = [2, 1], [0, 4]
    c = rng.standard_normal((T, d_c))
    C = rng.standard_normal((d_c - d_h, sum(H) * d_h))
    got = oracle.kv_project(c, C, d_h, H, offs)
    ref = _kv_reference_python(c, C, d_h, H, offs)
    np.testing.assert_allclose(got, ref, rtol=1e-14, atol=1e-14)


def test_kv_project_hand_computable():
    # H = 1, d_h = 1, d_c = 3: out = c[off] + sum of the other two times C
    c = np.array([[2.0, 3.0, 5.0]])
    C = np.array([[7.0], [11.0]])
    assert oracle.kv_project(c, C, 1, [1], [0])[0, 0] == 2 + 3 * 7 + 5 * 11
    assert oracle.kv_project(c, C, 1, [1], [1])[0, 0] == 3 + 2 * 7 + 5 * 11
    assert oracle.kv_project(c, C, 1, [1], [2])[0, 0] == 5 + 2 * 7 + 3 * 11


@pytest.mark.parametrize("offs", [[0, 0], [48, 0], [16, 32]])
def test_kv_project_reduces_to_dense_gemm(offs):
    """out_h W_h[B,:] = c W_h: the BD projection is the dense projection in another basis."""
    rng = np.random.default_rng(7)
    T, d_c, d_h, H = 33, 64, 16, [2, 3]
    c = rng.standard_normal((T, d_c))
    Ws, Cs = [], []
    for g in range(2):
        W = rng.standard_normal((d_c, H[g] * d_h)) * 0.125
        C, _, off, _ = oracle.prepare(W, d_c, H[g], d_h, mode=oracle.EXPLICIT, explicit_offset=offs[g])
        Ws.append(W)
        Cs.append(C)
    W_all = np.hstack(Ws)
    out = oracle.kv_project(c, np.hstack(Cs), d_h, H, offs)
    dense = np.matmul(c, W_all)                       # library routine
    col = 0
    for g in range(2):
        for h in range(H[g]):
            s = slice(col, col + d_h)
            A = W_all[offs[g]:offs[g] + d_h, s]
            back = np.matmul(out[:, s], A)
            assert np.max(np.abs(back - dense[:, s])) <= 1e-10 * max(1.0, np.max(np.abs(dense[:, s])))
            col += d_h


def test_kv_project_zero_C_is_tiled_copy():
    rng = np.random.default_rng(8)
    T, d_c, d_h, H, offs = 9, 32, 8, [3, 2], [24, 8]
    c = rng.standard_normal((T, d_c))
    out = oracle.kv_project(c, np.zeros((d_c - d_h, 5 * d_h)), d_h, H, offs)
    for i in range(5):
        off = offs[0] if i < 3 else offs[1]
        assert np.array_equal(out[:, i * d_h:(i + 1) * d_h], c[:, off:off + d_h])


def test_kv_project_zero_basis_slice_is_pure_gemm():
    rng = np.random.default_rng(9)
    T, d_c, d_h, H, off = 6, 20, 4, [2], [8]
    c = rng.standard_normal((T, d_c))
    c[:, 8:12] = 0.0
    C = rng.standard_normal((d_c - d_h, 2 * d_h))
    bbar = oracle.window_complement(d_c, d_h, 8)
    np.testing.assert_allclose(oracle.kv_project(c, C, d_h, H, off), c[:, bbar] @ C, rtol=1e-13, atol=1e-13)


def test_kv_project_empty():
    out = oracle.kv_project(np.zeros((0, 8)), np.zeros((6, 4)), 2, [2], [0])
    assert out.shape == (0, 4)


# ---------------------------------------------------------------- dense / low-rank linear
def test_dense_project_is_matmul():
    rng = np.random.default_rng(10)
    c = rng.standard_normal((17, 23))
    W = rng.standard_normal((23, 29))
    np.testing.assert_allclose(oracle.dense_project(c, W), np.matmul(c, W), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("mode", [oracle.FIRST, oracle.LAST])
def test_lowrank_linear_equals_xUV(mode):
    rng = np.random.default_rng(11)
    T, d_in, r, d_out = 13, 24, 6, 31
    x = rng.standard_normal((T, d_in))
    U = rng.standard_normal((d_in, r))
    V = rng.standard_normal((r, d_out))
    Up, C, off, _ = oracle.prepare_lowrank(U, V, mode=mode)
    assert off == (0 if mode == oracle.FIRST else d_out - r)
    y = oracle.lowrank_linear(x, Up, C, off)
    ref = np.matmul(np.matmul(x, U), V)
    assert np.max(np.abs(y - ref)) <= 1e-10 * np.max(np.abs(ref))
    # literal column BD of the product agrees with the closed form
    B_lit, C_lit, _ = oracle.bd_window(U @ V, r, off, oracle.COLS)
    np.testing.assert_allclose(Up, B_lit, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(C, C_lit, rtol=1e-7, atol=1e-8)


def test_lowrank_residual_min_picks_better_window():
    rng = np.random.default_rng(12)
    d_in, r, d_out = 20, 5, 17
    U = rng.standard_normal((d_in, r))
    V = rng.standard_normal((r, d_out))
    V[:, 1] = V[:, 0] * (1 + 1e-6)               # first-r window nearly singular
    _, _, off, resid = oracle.prepare_lowrank(U, V, mode=oracle.RESIDUAL_MIN, store_dtype=oracle.F16)
    assert off == d_out - r and resid[0] > resid[off]


# ---------------------------------------------------------------- storage rounding
def _bf16_cases():
    """float32-representable values (so that a float64 -> float32 -> bfloat16 conversion rounds
    once): random normals and subnormals, exact ties between two bfloat16 neighbours with even and
    odd lower neighbour, values one float32 ulp either side of a tie, powers of two, signed zeros,
    the largest finite bfloat16 and the tie above it (rounds to infinity)."""
    rng = np.random.default_rng(99)
    bits = [rng.integers(0, 2 ** 32, 20000, dtype=np.uint64).astype(np.uint32)]
    bits.append(rng.integers(0, 2 ** 23, 2000, dtype=np.uint64).astype(np.uint32))               # float32 subnormals
    hi = rng.integers(0, 0x7F80, 4000, dtype=np.uint64).astype(np.uint32) << np.uint32(16)       # finite bf16 patterns
    for low in (0x8000, 0x7FFF, 0x8001, 0x0001, 0xFFFF):
        bits.append(hi | np.uint32(low))
        bits.append(hi | np.uint32(low) | np.uint32(0x80000000))
    bits.append(np.array([0x00000000, 0x80000000, 0x7F7F0000, 0x7F7F8000, 0x7F7F7FFF, 0x00008000, 0x00018000,
                          0x00010000, 0x3F800000, 0x3F808000, 0x3F818000], dtype=np.uint32))
    b = np.concatenate(bits)
    v = b.view(np.float32)
    return v[np.isfinite(v)].astype(np.float64)


def test_bf16_rounding_matches_a_library_cast():
    """`round_store(x, BF16)` (ranks windows for bf16 storage) and the input generator's own bf16
    rounding against torch's CPU float32 -> bfloat16 cast (round to nearest even), bit for bit."""
    torch = pytest.importorskip("torch")
    import bda_workloads as wl
    x = _bf16_cases()
    ref_t = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)
    ref = ref_t.to(torch.float32).numpy().astype(np.float64)
    got = oracle.round_store(x, oracle.BF16)
    fin = np.isfinite(ref)
    assert np.array_equal(got, ref) and np.array_equal(np.signbit(got), np.signbit(ref))
    assert (~fin).sum() >= 2                                  # the overflow cases are among them
    stored, val = wl.to_storage(x, wl.BF16)
    ref_bits = ref_t.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(stored, ref_bits)
    assert np.array_equal(val[fin], ref[fin])


def test_f16_and_f32_rounding_match_library_casts():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(98)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-9, 5, 5000), [0.0, -0.0, 65504.0, 65519.0, 6e-8, 3e-8]])
    ref16 = torch.from_numpy(x).to(torch.float16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_store(x, oracle.F16), ref16)
    ref32 = torch.from_numpy(x).to(torch.float32).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_store(x, oracle.F32), ref32)


# ---------------------------------------------------------------- the pins catch planted mistakes
def test_planted_mistakes_are_caught():
    """Plant typical mistakes in a copy of the projection formula (on the CPU) and check that the
    pins above would reject each: the dense-GEMM reduction and the zero-C copy."""
    rng = np.random.default_rng(13)
    T, d_c, d_h, Hn, off = 7, 24, 4, 2, 8
    c = rng.standard_normal((T, d_c))
    W = rng.standard_normal((d_c, Hn * d_h))
    C, _, _, _ = oracle.prepare(W, d_c, Hn, d_h, mode=oracle.EXPLICIT, explicit_offset=off)
    bbar = oracle.window_complement(d_c, d_h, off)
    dense = c @ W

    def check(out):
        for h in range(Hn):
            s = slice(h * d_h, (h + 1) * d_h)
            if np.max(np.abs(out[:, s] @ W[off:off + d_h, s] - dense[:, s])) > 1e-10:
                return False
        return True

    good = np.hstack([c[:, off:off + d_h]] * Hn) + c[:, bbar] @ C
    assert check(good) and check(oracle.kv_project(c, C, d_h, [Hn], [off]))
    wrong_bbar = np.concatenate([np.arange(d_h, d_c)])                       # ignores the offset
    mistakes = {
        "dropped identity": c[:, bbar] @ C,
        "wrong sign": np.hstack([c[:, off:off + d_h]] * Hn) - c[:, bbar] @ C,
        "wrong window": np.hstack([c[:, 0:d_h]] * Hn) + c[:, bbar] @ C,
        "wrong complement": np.hstack([c[:, off:off + d_h]] * Hn) + c[:, wrong_bbar] @ C,
        "heads swapped": (np.hstack([c[:, off:off + d_h]] * Hn) + c[:, bbar] @ C)[:, ::-1],
    }
    for name, out in mistakes.items():
        assert not check(out), name
