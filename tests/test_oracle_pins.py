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
    C_F = oracle._solve_right(W[:2], W[2:])
    C_L = oracle._solve_right(W[m - 2:], W[:m - 2])
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
    tag, B, C, _ = oracle.bd_decompose_row(W, r)
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
    tag, B, C, (R_F, R_L) = oracle.bd_decompose_row(W, r)
    assert R_F < 1e-10 * np.linalg.norm(W) and R_L < 1e-10 * np.linalg.norm(W)
    np.testing.assert_allclose(oracle.bd_reconstruct_row(tag, B, C), W, atol=1e-10 * np.linalg.norm(W))
    # explicit [I; C] B and [C; I] B forms
    I = np.eye(r)
    C_F = oracle._solve_right(W[:r], W[r:])
    C_L = oracle._solve_right(W[m - r:], W[:m - r])
    np.testing.assert_allclose(np.vstack([I, C_F]) @ W[:r], W, atol=1e-9)
    np.testing.assert_allclose(np.vstack([C_L, I]) @ W[m - r:], W, atol=1e-9)


@pytest.mark.parametrize("m,n,r", [(5, 7, 2), (33, 20, 6)])
def test_col_identities(m, n, r):
    W = _rank_r(m, n, r)
    (R_F, B_F, C_F), (R_L, B_L, C_L) = oracle.bd_decompose_col_both(W, r)
    I = np.eye(r)
    np.testing.assert_allclose(B_F @ np.hstack([I, C_F]), W, atol=1e-9)
    np.testing.assert_allclose(B_L @ np.hstack([C_L, I]), W, atol=1e-9)
    assert R_F < 1e-9 and R_L < 1e-9


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
        (R_F, B_F, C_F), (R_L, B_L, C_L) = oracle.bd_decompose_col_both(M, d_h)
        B_lit, C_lit = (B_F, C_F) if mode == oracle.FIRST else (B_L, C_L)
        np.testing.assert_allclose(Bq[:, i * d_h:(i + 1) * d_h], B_lit, rtol=1e-9, atol=1e-9)
        np.testing.assert_allclose(C[:, i * d_h:(i + 1) * d_h], C_lit.T, rtol=1e-7, atol=1e-8)


def test_prepare_matches_literal_vo_algorithm():
    d, n, d_h, d_model = 40, 2, 8, 56
    Wv = RNG.standard_normal((d, n * d_h))
    Wo = RNG.standard_normal((n * d_h, d_model))
    tag, C_vo, B_vo, _ = oracle.attention_prepare_vo(Wv, Wo, n)
    mode = oracle.FIRST if tag == oracle.FIRST else oracle.LAST
    C, Bo, off, _ = oracle.prepare(Wv, d, n, d_h, side=Wo, side_kind=oracle.SIDE_O, mode=mode)
    np.testing.assert_allclose(C, C_vo, rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(Bo, B_vo, rtol=1e-9, atol=1e-9)


def test_literal_qk_prepare_shapes_and_shared_tag():
    """One tag for all heads; C_qk is (d - d_h) x n d_h (input line of the inference algorithm)."""
    d, n, d_h = 32, 4, 8
    Wq = RNG.standard_normal((d, n * d_h))
    Wk = RNG.standard_normal((d, n * d_h))
    tag, B_qk, C_qk, (R_F, R_L) = oracle.attention_prepare_qk(Wq, Wk, n)
    assert B_qk.shape == (d, n * d_h) and C_qk.shape == (d - d_h, n * d_h)
    assert tag == (oracle.FIRST if R_F <= R_L else oracle.LAST)


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
    tag, _, _, (R_F, R_L) = oracle.bd_decompose_row(W, d_h)
    assert R_F <= R_L and tag == oracle.FIRST


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
    (R_F, B_F, C_F), (R_L, B_L, C_L) = oracle.bd_decompose_col_both(U @ V, r)
    B_lit, C_lit = (B_F, C_F) if mode == oracle.FIRST else (B_L, C_L)
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
