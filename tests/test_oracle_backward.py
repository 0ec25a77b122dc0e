"""Pins of the oracle's K/V projection gradients (not gpu).

The forward oracle (C loops, pinned on its own in test_oracle_pins.py) is bilinear in (c, C), so a
difference quotient of L = <d_out, forward(c, C)> with ANY step equals the partial derivative up to
rounding: the gradients are checked entry by entry against it, against autograd through a dense
formulation that never mentions B / Bbar, against the adjoint identity, and in the special cases
that have a closed form.  Planted mistakes must fail."""
import numpy as np
import pytest
import torch

import oracle


def _problem(seed, T, d_c, d_h, H, offs):
    rng = np.random.default_rng(seed)
    N = sum(H) * d_h
    return (rng.standard_normal((T, d_c)), rng.standard_normal((T, N)),
            rng.standard_normal((d_c - d_h, N)))


def _loss(c, C, g, d_h, H, offs):
    return float(np.sum(g * oracle.kv_project(c, C, d_h, H, offs)))


CASES = [(3, 12, 4, [2], [0]), (4, 12, 4, [1, 2], [8, 4]), (2, 20, 4, [3], [16]), (5, 16, 8, [1, 1], [0, 8])]


@pytest.mark.parametrize("T,d_c,d_h,H,offs", CASES)
def test_backward_equals_difference_quotients(T, d_c, d_h, H, offs):
    c, g, C = _problem(1, T, d_c, d_h, H, offs)
    dc, dC = oracle.kv_project_backward(c, g, C, d_h, H, offs)
    base = _loss(c, C, g, d_h, H, offs)
    for i in range(T):
        for j in range(d_c):
            cp = c.copy()
            cp[i, j] += 0.5
            assert abs((_loss(cp, C, g, d_h, H, offs) - base) / 0.5 - dc[i, j]) < 1e-9, (i, j)
    for i in range(C.shape[0]):
        for j in range(C.shape[1]):
            Cp = C.copy()
            Cp[i, j] += 2.0
            assert abs((_loss(c, Cp, g, d_h, H, offs) - base) / 2.0 - dC[i, j]) < 1e-9, (i, j)


def _head_layout(d_c, d_h, H, offs):
    """Per head: the latent rows outside its window, the window start, its first output column."""
    col = 0
    rows = []
    for n_heads, off in zip(H, offs):
        keep = [k for k in range(d_c) if not (off <= k < off + d_h)]
        for _ in range(n_heads):
            rows.append((keep, off, col))
            col += d_h
    return rows


@pytest.mark.parametrize("T,d_c,d_h,H,offs", CASES + [(33, 96, 16, [3, 2], [32, 80])])
def test_backward_equals_autograd_of_dense_form(T, d_c, d_h, H, offs):
    c, g, C = _problem(2, T, d_c, d_h, H, offs)
    ct = torch.tensor(c, requires_grad=True)
    Ct = torch.tensor(C, requires_grad=True)
    # the d_c x N matrix whose basis rows are identity blocks and whose other rows are C
    # (Eq. qk_bd_merge read as one dense product)
    blocks = []
    for keep, off, col in _head_layout(d_c, d_h, H, offs):
        Wh = torch.zeros((d_c, d_h), dtype=torch.float64)
        Wh[off:off + d_h, :] = torch.eye(d_h, dtype=torch.float64)
        Wh = Wh.index_put((torch.tensor(keep),), Ct[:, col:col + d_h])
        blocks.append(Wh)
    out = ct @ torch.cat(blocks, dim=1)
    assert np.allclose(out.detach().numpy(), oracle.kv_project(c, C, d_h, H, offs), atol=1e-12)
    out.backward(torch.tensor(g))
    dc, dC = oracle.kv_project_backward(c, g, C, d_h, H, offs)
    assert np.max(np.abs(ct.grad.numpy() - dc)) < 1e-11
    assert np.max(np.abs(Ct.grad.numpy() - dC)) < 1e-11


def test_backward_adjoint_identity_medium():
    T, d_c, d_h, H, offs = 70, 192, 32, [3, 2], [48, 160]
    c, g, C = _problem(3, T, d_c, d_h, H, offs)
    rng = np.random.default_rng(4)
    dc, dC = oracle.kv_project_backward(c, g, C, d_h, H, offs)
    for _ in range(3):
        u = rng.standard_normal(c.shape)
        V = rng.standard_normal(C.shape)
        lhs_c = _loss(c + u, C, g, d_h, H, offs) - _loss(c, C, g, d_h, H, offs)
        lhs_C = _loss(c, C + V, g, d_h, H, offs) - _loss(c, C, g, d_h, H, offs)
        assert abs(lhs_c - np.sum(dc * u)) < 1e-8 * (1 + abs(lhs_c))
        assert abs(lhs_C - np.sum(dC * V)) < 1e-8 * (1 + abs(lhs_C))


def test_backward_closed_form_special_cases():
    T, d_c, d_h, H, offs = 6, 24, 8, [2, 1], [8, 16]
    c, g, C = _problem(5, T, d_c, d_h, H, offs)
    # C = 0: the forward is a tiled copy of the basis slice, so d_c is the sum of the heads'
    # gradients on the window and zero elsewhere; d_C does not depend on C at all
    dc0, dC0 = oracle.kv_project_backward(c, g, np.zeros_like(C), d_h, H, offs)
    want = np.zeros_like(c)
    want[:, 8:16] += g[:, 0:8] + g[:, 8:16]
    want[:, 16:24] += g[:, 16:24]
    assert np.array_equal(dc0, want)
    _, dC = oracle.kv_project_backward(c, g, C, d_h, H, offs)
    assert np.array_equal(dC, dC0)
    # one token, one head, d_out = e_j: d_C is the outer product of the non-basis latent with e_j
    c1 = c[:1]
    e = np.zeros((1, 8))
    e[0, 3] = 1.0
    dc1, dC1 = oracle.kv_project_backward(c1, e, C[:, :8], d_h, [1], [8])
    bbar = oracle.window_complement(d_c, d_h, 8)
    assert np.array_equal(dC1[:, 3], c1[0, bbar]) and np.count_nonzero(dC1) == np.count_nonzero(dC1[:, 3])
    assert np.array_equal(dc1[0, bbar], C[:, 3]) and dc1[0, 8 + 3] == 1.0
    # no tokens
    dce, dCe = oracle.kv_project_backward(c[:0], g[:0], C, d_h, H, offs)
    assert dce.shape == (0, d_c) and not dCe.any()


def test_backward_planted_mistakes_are_caught():
    """Typical slips, planted in a copy of the formulas on the CPU, must fail the
    difference-quotient pin."""
    T, d_c, d_h, H, offs = 3, 12, 4, [2], [4]
    c, g, C = _problem(6, T, d_c, d_h, H, offs)
    bbar = oracle.window_complement(d_c, d_h, 4)
    base = _loss(c, C, g, d_h, H, offs)

    def quotient_c():
        q = np.zeros_like(c)
        for i in range(T):
            for j in range(d_c):
                cp = c.copy()
                cp[i, j] += 1.0
                q[i, j] = _loss(cp, C, g, d_h, H, offs) - base
        return q

    q = quotient_c()
    good, _ = oracle.kv_project_backward(c, g, C, d_h, H, offs)
    assert np.max(np.abs(good - q)) < 1e-9
    no_head_sum = np.zeros_like(c)
    no_head_sum[:, bbar] = g @ C.T
    last_head_only = no_head_sum.copy()
    last_head_only[:, 4:8] = g[:, 4:8]
    wrong_window = no_head_sum.copy()
    wrong_window[:, 0:4] += g[:, 0:4] + g[:, 4:8]
    for name, bad in {"no head sum": no_head_sum, "last head only": last_head_only,
                      "wrong window": wrong_window}.items():
        assert np.max(np.abs(bad - q)) > 1e-3, name
