"""GPU parity of the K/V projection's gradients (bda_kv_project_backward through the C ABI) against
the fp64 oracle, element by element on the same seeded inputs.

Tolerance: |g - o| <= tol * max(|o|, RMS of o's column) (+ half a bf16 ulp for bf16 storage), with
tol 2e-3 for fp16 / bf16 and 1e-5 for fp32 -- the forward's bar with the per-head floor replaced
by a per-column one: the window columns of grad_c (a sum of a few heads) and its other columns (a
contraction over all output columns) differ in scale by an order of magnitude."""
import numpy as np
import pytest

import bda_workloads as wl
import oracle
from helpers import assert_parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import gpu_harness as gh          # noqa: E402
import paper_2510_01718_amd as bda  # noqa: E402


def _inputs(seed, T, d_c, d_h, H, dtype, c_scale=1.0, C_scale=0.25):
    """Latent rows, upstream gradient and coefficients: independent Gaussians rounded to the
    storage type (the gradient formulas do not care whether C came from a preparation)."""
    rng = np.random.default_rng([seed, T, d_c])
    N = sum(H) * d_h
    c_s, c64 = wl.to_storage(c_scale * rng.standard_normal((T, d_c)), dtype)
    g_s, g64 = wl.to_storage(rng.standard_normal((T, N)), dtype)
    C_s, C64 = wl.to_storage(C_scale * rng.standard_normal((d_c - d_h, N)), dtype)
    return (c_s, c64), (g_s, g64), (C_s, C64)


def _backward(c_s, g_s, C_s, T, d_c, d_h, H, offs, dtype, grad_dtype=None, pad=0, want=(True, True), fill=None, policy=0):
    grad_dtype = dtype if grad_dtype is None else grad_dtype
    N = sum(H) * d_h
    K = d_c - d_h
    ldc, ldg, ldC, ld_gc, ld_gC = d_c + pad, N + pad, N + 2 * pad, d_c + 3 * pad, N + pad
    c_d = gh.to_device(c_s, dtype, ldc) if T else gh.new_out(1, ldc, dtype)
    g_d = gh.to_device(g_s, dtype, ldg) if T else gh.new_out(1, ldg, dtype)
    C_d = gh.to_device(C_s, dtype, ldC)
    gc_d = gh.new_out(max(T, 1), ld_gc, grad_dtype, fill) if want[0] else None
    gC_d = gh.new_out(K, ld_gC, grad_dtype, fill) if want[1] else None
    if policy:
        bda.bda_kv_project_backward_ex(c_d if want[1] else None, ldc, g_d, ldg, C_d if want[0] else None, ldC,
                                       T, d_c, d_h, H, offs, gc_d, ld_gc, gC_d, ld_gC, dtype, grad_dtype, gh.stream(), policy)
    else:
        bda.bda_kv_project_backward(c_d if want[1] else None, ldc, g_d, ldg, C_d if want[0] else None, ldC,
                                    T, d_c, d_h, H, offs, gc_d, ld_gc, gC_d, ld_gC, dtype, grad_dtype, gh.stream())
    torch.cuda.synchronize()
    gc = gh.to_host64(gc_d[:T], grad_dtype, d_c) if want[0] else None
    gC = gh.to_host64(gC_d, grad_dtype, N) if want[1] else None
    return gc, gC, gc_d, gC_d


def _check(T, d_c, d_h, H, offs, dtype, grad_dtype=None, pad=0, policy=0, seed=5, what=""):
    (c_s, c64), (g_s, g64), (C_s, C64) = _inputs(seed, T, d_c, d_h, H, dtype)
    ref_c, ref_C = oracle.kv_project_backward(c64, g64, C64, d_h, H, offs)
    gc, gC, _, _ = _backward(c_s, g_s, C_s, T, d_c, d_h, H, offs, dtype, grad_dtype, pad, policy=policy)
    gd = dtype if grad_dtype is None else grad_dtype
    tag = f"{what} T={T} d_c={d_c} d_h={d_h} H={H} offs={offs} dtype={dtype}/{gd} policy={policy}"
    if T:
        assert_parity(gc, ref_c, 1, dtype, gd, "grad_c " + tag)
    assert_parity(gC, ref_C, 1, dtype, gd, "grad_C " + tag)


SHAPES = [
    (300, 512, 128, [3, 2], [0, 384]),     # first / last window, ragged token tail
    (130, 256, 64, [2, 3], [64, 192]),     # interior and last window, two groups with different windows
    (77, 192, 32, [5], [40]),              # window start a multiple of 8 only
    (64, 128, 32, [1], [96]),              # a single tile
    (200, 320, 96, [2, 1], [16, 224]),     # d_h not a power of two: chunks of 64 straddle heads
]


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("T,d_c,d_h,H,offs", SHAPES)
@pytest.mark.parametrize("policy", [0, 1])
def test_backward_mfma_matches_oracle(T, d_c, d_h, H, offs, dtype, policy):
    _check(T, d_c, d_h, H, offs, dtype, policy=policy)


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_backward_float32_gradients_and_padded_rows(dtype):
    _check(150, 256, 64, [2, 2], [0, 128], dtype, grad_dtype=wl.F32, pad=8)
    _check(150, 256, 64, [2, 2], [192, 64], dtype, grad_dtype=wl.F32, pad=16, policy=1)


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_backward_general_kernels(dtype):
    # fp32 inputs, and 16-bit inputs whose head width / window start / row pitch rule out MFMA tiles
    _check(50, 72, 24, [2, 1], [3, 48], dtype)
    _check(70, 96, 32, [3], [20], dtype, pad=3)
    if dtype != wl.F32:
        _check(33, 64, 16, [2], [8], dtype, grad_dtype=wl.F32)


def test_backward_tile_shapes_chosen_by_size():
    # many 64 x 64 tiles (two per compute unit): 65 x 8 for the latent gradient ...
    _check(4100, 512, 128, [1, 1], [0, 384], wl.F16)
    # ... and 6 x 86 for the weight gradient
    _check(100, 512, 128, [22, 21], [384, 0], wl.BF16)
    # 128 x 128 tiles by size: 65 x 4 latent tiles
    _check(8200, 512, 128, [1], [128], wl.BF16)


def test_backward_each_gradient_alone_and_no_tokens():
    T, d_c, d_h, H, offs, dtype = 90, 256, 64, [2, 1], [0, 192], wl.F16
    (c_s, c64), (g_s, g64), (C_s, C64) = _inputs(9, T, d_c, d_h, H, dtype)
    ref_c, ref_C = oracle.kv_project_backward(c64, g64, C64, d_h, H, offs)
    gc, none, _, _ = _backward(c_s, g_s, C_s, T, d_c, d_h, H, offs, dtype, want=(True, False))
    assert none is None
    assert_parity(gc, ref_c, 1, dtype, dtype, "grad_c alone")
    none, gC, _, _ = _backward(c_s, g_s, C_s, T, d_c, d_h, H, offs, dtype, want=(False, True))
    assert none is None
    assert_parity(gC, ref_C, 1, dtype, dtype, "grad_C alone")
    # no tokens: the weight gradient is an empty sum
    _, gC0, _, _ = _backward(c_s[:0], g_s[:0], C_s, 0, d_c, d_h, H, offs, dtype, fill=7.0)
    assert gC0.shape == ref_C.shape and not gC0.any()
    (c_s, _), (g_s, _), (C_s, _) = _inputs(9, 0, 72, 24, [2, 1], wl.F32)
    _, gC0, _, _ = _backward(c_s, g_s, C_s, 0, 72, 24, [2, 1], [3, 48], wl.F32, fill=7.0)
    assert gC0.shape == (48, 72) and not gC0.any()


def test_backward_writes_nothing_outside_its_matrices():
    T, d_c, d_h, H, offs, dtype, pad = 70, 128, 32, [2, 1], [32, 96], wl.F16, 8
    (c_s, _), (g_s, _), (C_s, _) = _inputs(11, T, d_c, d_h, H, dtype)
    N = sum(H) * d_h
    _, _, gc_d, gC_d = _backward(c_s, g_s, C_s, T, d_c, d_h, H, offs, dtype, pad=pad, fill=3.0)
    assert torch.all(gc_d[:, d_c:] == 3.0) and torch.all(gC_d[:, N:] == 3.0)


def test_backward_benchmark_shape_full():
    """The V2-Lite-shaped training step (T = 4096, 16 + 16 heads, fp16): every element."""
    _check(4096, 512, 128, [16, 16], [0, 0], wl.F16, what="v2lite")


def test_backward_v3_shape_sampled():
    """The V3-shaped training step (T = 8192, 128 + 128 heads, bf16, two different windows), the
    shape the largest forward configuration has: grad_c on 264 sampled token rows (its rows are
    independent, so the oracle computes exactly those), grad_C on 10 sampled heads (all tokens, all
    rows of C; the oracle is given the reduced problem made of those heads' columns).  Gradients
    start as NaN patterns and must be finite everywhere."""
    T, d_c, d_h, H, offs, dtype = 8192, 512, 128, [128, 128], [0, 384], wl.BF16
    N, K = sum(H) * d_h, d_c - d_h
    rng = np.random.default_rng([31, T, d_c])
    c_s, c64 = wl.to_storage(rng.standard_normal((T, d_c)), dtype)
    C_s, C64 = wl.to_storage(0.25 * rng.standard_normal((K, N)), dtype)
    g_s = np.empty((T, N), dtype=np.uint16)
    for r0 in range(0, T, 512):                                   # chunked: the float64 draw of the whole matrix is 2 GiB
        g_s[r0:r0 + 512], _ = wl.to_storage(rng.standard_normal((512, N)), dtype)
    c_d, g_d, C_d = gh.to_device(c_s, dtype), gh.to_device(g_s, dtype), gh.to_device(C_s, dtype)
    gc_d = gh.new_out(T, d_c, dtype, fill=0x7FC0)
    gC_d = gh.new_out(K, N, dtype, fill=0x7FC0)
    bda.bda_kv_project_backward(c_d, d_c, g_d, N, C_d, N, T, d_c, d_h, H, offs, gc_d, d_c, gC_d, N, dtype, dtype, gh.stream())
    torch.cuda.synchronize()
    gc, gC = gh.to_host64(gc_d, dtype), gh.to_host64(gC_d, dtype)
    assert np.all(np.isfinite(gc)) and np.all(np.isfinite(gC))
    # grad_c: first / last rows, one row per 128-token tile, random rows
    rows = set(range(4)) | set(range(T - 4, T)) | {128 * b + (37 * b + 5) % 128 for b in range(T // 128)}
    rows |= set(int(r) for r in rng.integers(0, T, 192))
    rows = np.array(sorted(rows))
    assert len(rows) >= 256
    ref_c, _ = oracle.kv_project_backward(c64[rows], wl.from_storage(g_s[rows], dtype), C64, d_h, H, offs)
    rel_c = assert_parity(gc[rows], ref_c, 1, dtype, dtype, "v3 grad_c, sampled rows")
    # grad_C: sampled heads of both groups
    heads = sorted({0, 1, 127, 128, 129, 255} | set(int(h) for h in rng.integers(0, 256, 4)))
    cols = np.concatenate([np.arange(h * d_h, (h + 1) * d_h) for h in heads])
    H_sub = [sum(1 for h in heads if h < 128), sum(1 for h in heads if h >= 128)]
    g_sub = wl.from_storage(np.ascontiguousarray(g_s[:, cols]), dtype)
    _, ref_C = oracle.kv_project_backward(c64, g_sub, C64[:, cols], d_h, H_sub, offs)
    rel_C = assert_parity(gC[:, cols], ref_C, 1, dtype, dtype, "v3 grad_C, sampled heads")
    print(f"v3 backward: grad_c {len(rows)} rows {rel_c:.2e}; grad_C {len(heads)} heads {rel_C:.2e}")


@pytest.mark.parametrize("seed", [1, 2])
def test_backward_random_shapes(seed):
    """Seeded random shapes (head widths 32 .. 128 incl. 96, contraction 32 .. 448 in steps of 8 with
    windows anywhere on the multiples of 8, one to three groups, 1 .. 700 tokens, padded rows) through
    both tile shapes of the gradient kernels."""
    rng = np.random.default_rng(3000 + seed)
    for case in range(14):
        d_h = int(rng.choice([32, 64, 96, 128]))
        K = 8 * int(rng.integers(4, 57))
        d_c = K + d_h
        G = int(rng.integers(1, 4))
        H = [int(rng.integers(1, 5)) for _ in range(G)]
        offs = [8 * int(rng.integers(0, K // 8 + 1)) for _ in range(G)]
        T = int(rng.choice([1, 33, 64, 100, 129, 256, 300, 700]))
        dtype = wl.F16 if rng.integers(0, 2) else wl.BF16
        grad_dtype = wl.F32 if rng.integers(0, 3) == 0 else None
        pad = 8 * int(rng.integers(0, 3))
        for policy in (0, 1):
            _check(T, d_c, d_h, H, offs, dtype, grad_dtype=grad_dtype, pad=pad, policy=policy, seed=seed * 100 + case,
                   what=f"seed {seed} case {case}")
