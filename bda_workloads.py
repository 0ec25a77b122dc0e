"""Seeded synthetic inputs for the BD key/value up-projection and the BD low-rank linear.

This module only draws random numbers, normalises latent rows and rounds values to a storage
dtype.  It holds none of the method's arithmetic (no basis decomposition, no projection), so both
the CPU oracle's tests and the GPU library's tests/bench can take their inputs from it without
sharing any code of the method itself.

The shapes follow the attention shape the paper benchmarks (n heads, latent width d = d_c = 512,
head width d_h = 128; throughput tables of the appendix) and the low-rank LLaMA-style linear of the
low-rank pruning experiment.  Real model weights are not available, so Gaussian weights stand in
for them; by the almost-sure full-rank theorem (section "Selection of Basis") any contiguous
d_h x d_h block of such weights is a valid basis.

Draw order (fixed, part of the recipe):
  latent stream   : Generator(PCG64([seed, 0, T]))  -> c (T x d_c), row-major draw
  weight stream   : Generator(PCG64([seed, 1]))     -> for each group (K then V), for each head,
                    a d_c x d_h block, row-major draw
so the weights of a configuration do not depend on the number of tokens T.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

# dtype tags (same integer values as the C ABI's bda_dtype; plain data, no arithmetic)
F32, F16, BF16, F64 = 0, 1, 2, 3
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16", F64: "f64"}
DTYPE_BYTES = {F32: 4, F16: 2, BF16: 2, F64: 8}


# --------------------------------------------------------------------------------------------
# storage rounding (round-to-nearest-even from float64)
# --------------------------------------------------------------------------------------------
def _bf16_bits_from_f64(x: np.ndarray) -> np.ndarray:
    """float64 -> bfloat16 bit patterns (uint16), one round-to-nearest-even step from float64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    m, e = np.frexp(x)                                  # x = m * 2**e, 0.5 <= |m| < 1
    step_exp = np.maximum(e - 8, -133)                  # 8 significant bits; subnormal floor
    q = np.ldexp(np.rint(np.ldexp(x, -step_exp)), step_exp)   # np.rint rounds half to even
    q = np.where(np.isfinite(x), q, x)
    f32 = q.astype(np.float32)                          # exact (or overflow to inf)
    bits = (f32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return np.where(np.isnan(x), np.uint16(0x7FC0), bits).astype(np.uint16)


def _f64_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def to_storage(x: np.ndarray, dtype: int) -> Tuple[np.ndarray, np.ndarray]:
    """Round float64 values to `dtype`.

    Returns (stored, value64): `stored` is the array a device buffer is filled from (float32,
    float16, or uint16 bit patterns for bf16); `value64` is exactly what those stored numbers
    mean, as float64 -- the oracle computes on `value64`, the GPU library on `stored`.
    """
    x = np.ascontiguousarray(x, dtype=np.float64)
    if dtype == F32:
        s = x.astype(np.float32)
        return s, s.astype(np.float64)
    if dtype == F16:
        s = x.astype(np.float16)
        return s, s.astype(np.float64)
    if dtype == BF16:
        s = _bf16_bits_from_f64(x)
        return s, _f64_from_bf16_bits(s)
    if dtype == F64:
        return x.copy(), x.copy()
    raise ValueError(f"unknown dtype tag {dtype}")


def from_storage(stored: np.ndarray, dtype: int) -> np.ndarray:
    """Exact float64 meaning of a stored array (inverse view of `to_storage`)."""
    if dtype == BF16:
        return _f64_from_bf16_bits(stored)
    return np.asarray(stored).astype(np.float64)


def half_ulp(value64: np.ndarray, dtype: int) -> np.ndarray:
    """Half a unit in the last place of `dtype` at the magnitude of each value (normal range)."""
    mant = {F32: 24, F16: 11, BF16: 8}[dtype]
    min_exp = {F32: -126, F16: -14, BF16: -126}[dtype]
    a = np.abs(np.asarray(value64, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** min_exp)))
    return 0.5 * np.exp2(e - (mant - 1))


# --------------------------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------------------------
@dataclass
class KVWorkload:
    """One K/V up-projection problem: latent c and the dense per-head projection weights."""
    name: str
    seed: int
    dtype: int
    T: int
    d_c: int
    d_h: int
    H: List[int]                      # heads per group (group 0 = K_nope blocks, group 1 = V blocks)
    c_stored: np.ndarray              # T x d_c in storage dtype
    c: np.ndarray                     # same numbers as float64
    W: np.ndarray                     # d_c x (sum(H)*d_h) float64, dense weights (unrounded)
    meta: Dict[str, object] = field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(sum(self.H)) * self.d_h


@dataclass
class LowRankWorkload:
    """One low-rank linear problem W = U.V with input x."""
    name: str
    seed: int
    dtype: int
    T: int
    d_in: int
    r: int
    d_out: int
    x_stored: np.ndarray
    x: np.ndarray
    U: np.ndarray                     # d_in x r float64
    V: np.ndarray                     # r x d_out float64


def _latent(seed: int, T: int, d_c: int, rms_norm: bool) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64([seed, 0, T]))
    c = rng.standard_normal((T, d_c))
    if rms_norm:
        c = c / np.sqrt(np.mean(c * c, axis=1, keepdims=True) + 1e-6)
    return c


def _head_weights(seed: int, d_c: int, d_h: int, H: List[int], std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64([seed, 1]))
    n_heads = int(sum(H))
    W = np.empty((d_c, n_heads * d_h), dtype=np.float64)
    for h in range(n_heads):
        W[:, h * d_h:(h + 1) * d_h] = std * rng.standard_normal((d_c, d_h))
    return W


def kv_workload(name: str, T: Optional[int] = None, seed: Optional[int] = None,
                dtype: Optional[int] = None) -> KVWorkload:
    """Named K/V workloads.

    tiny     : T=64, d_c=64, 2 heads of 16, N(0,1) latent, weights of variance 1/64, fp32, seed 0
    v2lite   : DeepSeek-V2-Lite-shaped, d_c=512, 16 K_nope + 16 V heads of 128, weights of std
               0.02, RMS-normalised latent, fp16, T=4096, seed 1
    decode   : the v2lite weights with T tokens (T in {1, 8, 32, 64})
    v3       : DeepSeek-V3-shaped, 128 K_nope + 128 V heads of 128, bf16, T=8192, seed 2
    """
    if name == "tiny":
        p = dict(T=64, d_c=64, d_h=16, H=[2], std=0.125, rms=False, dtype=F32, seed=0)
    elif name == "v2lite":
        p = dict(T=4096, d_c=512, d_h=128, H=[16, 16], std=0.02, rms=True, dtype=F16, seed=1)
    elif name == "decode":
        p = dict(T=1, d_c=512, d_h=128, H=[16, 16], std=0.02, rms=True, dtype=F16, seed=1)
    elif name == "v3":
        p = dict(T=8192, d_c=512, d_h=128, H=[128, 128], std=0.02, rms=True, dtype=BF16, seed=2)
    else:
        raise ValueError(f"unknown K/V workload {name!r}")
    if T is not None:
        p["T"] = int(T)
    if seed is not None:
        p["seed"] = int(seed)
    if dtype is not None:
        p["dtype"] = int(dtype)
    return custom_kv_workload(name, p["T"], p["d_c"], p["d_h"], p["H"], p["std"], p["rms"],
                              p["dtype"], p["seed"])


def custom_kv_workload(name: str, T: int, d_c: int, d_h: int, H: List[int], std: float,
                       rms_norm: bool, dtype: int, seed: int) -> KVWorkload:
    c = _latent(seed, T, d_c, rms_norm)
    c_stored, c64 = to_storage(c, dtype)
    W = _head_weights(seed, d_c, d_h, list(H), std)
    return KVWorkload(name=name, seed=seed, dtype=dtype, T=T, d_c=d_c, d_h=d_h, H=list(H),
                      c_stored=c_stored, c=c64, W=W)


def lowrank_workload(name: str = "lowrank", T: Optional[int] = None, seed: Optional[int] = None,
                     d_in: Optional[int] = None, r: Optional[int] = None,
                     d_out: Optional[int] = None, dtype: Optional[int] = None) -> LowRankWorkload:
    """Low-rank linear W = U.V: d_in=4096, r=1024, d_out=11008, U and V of std 0.02, x ~ N(0,1),
    fp16, T=8192, seed 3.  Draw order: x, then U, then V (separate streams for x and weights)."""
    p = dict(T=8192, d_in=4096, r=1024, d_out=11008, dtype=F16, seed=3)
    for k, v in dict(T=T, seed=seed, d_in=d_in, r=r, d_out=d_out, dtype=dtype).items():
        if v is not None:
            p[k] = int(v)
    rng_x = np.random.Generator(np.random.PCG64([p["seed"], 0, p["T"]]))
    rng_w = np.random.Generator(np.random.PCG64([p["seed"], 1]))
    x = rng_x.standard_normal((p["T"], p["d_in"]))
    U = 0.02 * rng_w.standard_normal((p["d_in"], p["r"]))
    V = 0.02 * rng_w.standard_normal((p["r"], p["d_out"]))
    x_stored, x64 = to_storage(x, p["dtype"])
    return LowRankWorkload(name=name, seed=p["seed"], dtype=p["dtype"], T=p["T"], d_in=p["d_in"],
                           r=p["r"], d_out=p["d_out"], x_stored=x_stored, x=x64, U=U, V=V)
