"""Shared test helpers: error metric and tolerances for GPU-vs-oracle parity.

Tolerance (float outputs): with o the oracle value and RMS_h the root mean square of the oracle
output over the head block (all tokens, d_h columns) that o belongs to,

    |g - o| <= tol * max(|o|, RMS_h)                       fp16 (tol 2e-3), fp32 (tol 1e-5)
    |g - o| <= tol * max(|o|, RMS_h) + half_ulp_bf16(o)    bf16 stored outputs (tol 2e-3)

The RMS floor is needed because an output that cancels to nearly zero has no meaningful
element-wise relative error; the extra half ulp for bf16 is needed because bf16's own storage
rounding (up to 2^-8 relative) exceeds 2e-3 -- the same kernel with float32 outputs is held to the
plain 2e-3 in a separate test.
"""
import numpy as np

import bda_workloads as wl

TOL = {wl.F32: 1e-5, wl.F16: 2e-3, wl.BF16: 2e-3}


def head_rms(o: np.ndarray, d_h: int) -> np.ndarray:
    """RMS of the oracle output per head block, broadcast back to o's shape."""
    T, N = o.shape
    blocks = o.reshape(T, N // d_h, d_h)
    rms = np.sqrt(np.mean(blocks * blocks, axis=(0, 2), keepdims=True))
    return np.broadcast_to(rms, blocks.shape).reshape(T, N)


def parity_error(g: np.ndarray, o: np.ndarray, d_h: int, in_dtype: int, out_dtype: int,
                 extra_allow=None):
    """Returns (worst ratio of |g-o| to its allowance, plain max relative error).
    `extra_allow` (same shape as o, or None) is an additional absolute allowance that the caller
    derives from the arithmetic of the operator under test."""
    g = np.asarray(g, dtype=np.float64)
    scale = np.maximum(np.abs(o), head_rms(o, d_h))
    scale = np.maximum(scale, np.finfo(np.float64).tiny)
    allow = TOL[in_dtype] * scale
    if out_dtype == wl.BF16:
        allow = allow + wl.half_ulp(o, wl.BF16)
    if extra_allow is not None:
        allow = allow + extra_allow
    diff = np.abs(g - o)
    return float(np.max(diff / allow)), float(np.max(diff / scale))


def lowrank_h_rounding_allowance(ref, C64, r, off, dtype):
    """BD linear layer: the library stores h = x B in `dtype` inside the output and the second
    product reads it back, while the oracle keeps h in float64.  One rounding of h_j moves the
    output column m by at most half_ulp(h_j) |C_jm|; summed over j this bounds the difference.
    Computed from oracle values only."""
    h = ref[:, off:off + r]
    extra = np.zeros_like(ref)
    rest = np.concatenate([np.arange(0, off), np.arange(off + r, ref.shape[1])])
    extra[:, rest] = wl.half_ulp(h, dtype) @ np.abs(C64)
    return extra


def assert_parity(g, o, d_h, in_dtype, out_dtype, what="", extra_allow=None):
    assert g.shape == o.shape, (g.shape, o.shape)
    assert np.all(np.isfinite(g)), f"{what}: non-finite GPU output"
    worst, rel = parity_error(g, o, d_h, in_dtype, out_dtype, extra_allow)
    assert worst <= 1.0, f"{what}: error {rel:.3e} exceeds tolerance (ratio {worst:.3f})"
    return rel
