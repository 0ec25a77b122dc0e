"""ctypes binding of libbda.so: same names as the C ABI (include/bda.h), argument marshalling only.

Host calls (`bda_prepare*`) take and return numpy float64 arrays.  Device calls take anything that
exposes `data_ptr()` (PyTorch tensors on the GPU) or a raw integer device address, plus explicit
sizes; they enqueue on the given stream (an integer hipStream_t, e.g.
`torch.cuda.current_stream().cuda_stream`; 0 = default stream) and return nothing.
A non-zero status raises BdaError with the library's message.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

BDA_F32, BDA_F16, BDA_BF16, BDA_F64 = 0, 1, 2, 3
BASIS_FIRST, BASIS_LAST, BASIS_RESIDUAL_MIN, BASIS_OFFSET_SEARCH, BASIS_EXPLICIT = 0, 1, 2, 3, 4
SIDE_NONE, SIDE_Q, SIDE_O = 0, 1, 2

EXPORTS = ("bda_prepare", "bda_prepare_lowrank", "bda_prepare_device", "bda_prepare_device_ex",
           "bda_prepare_device_workspace_bytes", "bda_prepare_device_static", "bda_packed_weights_bytes",
           "bda_pack_weights", "bda_kv_project_packed", "bda_kv_project", "bda_dense_project",
           "bda_lowrank_linear", "bda_kv_project_backward", "bda_kv_project_ex", "bda_dense_project_ex",
           "bda_kv_project_backward_ex", "bda_kv_project_plan", "bda_dense_project_plan", "bda_last_error", "bda_version")

_PKG = os.path.dirname(os.path.abspath(__file__))
_lib = None


KERNEL_NONE, KERNEL_GENERAL, KERNEL_MFMA, KERNEL_STREAM, KERNEL_LEAN, KERNEL_DECODE, KERNEL_DUO = 0, 1, 2, 3, 4, 5, 6


class LaunchPlan(ctypes.Structure):
    """Mirror of bda_launch_plan."""
    _fields_ = [(n, ctypes.c_int) for n in ("kernel", "tile_tokens", "tile_columns", "token_tiles", "column_tiles",
                                            "workgroups", "threads", "lds_bytes", "rounds", "tile_by_tile",
                                            "super_m", "super_n")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class BdaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"bda status {status}: {message}")
        self.status = status
        self.message = message


def lib_path() -> str:
    return os.path.join(_PKG, "libbda.so")


def load():
    """Loads libbda.so; fails loudly if it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is not built; run `python -m paper_2510_01718_amd.build` (needs hipcc)")
    lib = ctypes.CDLL(path)
    c_int, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int)
    lib.bda_prepare.restype = c_int
    lib.bda_prepare.argtypes = [dp, i64, c_int, c_int, c_int, dp, i64, c_int, c_int, c_int, c_int,
                                c_int, dp, dp, ip, dp]
    lib.bda_prepare_lowrank.restype = c_int
    lib.bda_prepare_lowrank.argtypes = [dp, dp, c_int, c_int, c_int, c_int, c_int, dp, dp, ip, dp]
    lib.bda_prepare_device.restype = c_int
    lib.bda_prepare_device.argtypes = [vp, i64, c_int, c_int, c_int, c_int, c_int, vp, i64, c_int, vp, vp]
    lib.bda_prepare_device_workspace_bytes.restype = ctypes.c_size_t
    lib.bda_prepare_device_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int]
    lib.bda_prepare_device_ex.restype = c_int
    lib.bda_prepare_device_ex.argtypes = [vp, i64, c_int, c_int, c_int, c_int, vp, i64, c_int, c_int, c_int, c_int,
                                          vp, i64, vp, i64, c_int, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.bda_prepare_device_static.restype = c_int
    lib.bda_prepare_device_static.argtypes = [vp, i64, c_int, c_int, c_int, c_int, vp, i64, c_int, c_int, c_int, c_int,
                                              vp, i64, vp, i64, c_int, vp, vp, vp, vp]
    lib.bda_packed_weights_bytes.restype = ctypes.c_size_t
    lib.bda_packed_weights_bytes.argtypes = [c_int, c_int, c_int, ip, c_int]
    lib.bda_pack_weights.restype = c_int
    lib.bda_pack_weights.argtypes = [vp, i64, c_int, c_int, c_int, ip, c_int, vp, vp]
    lib.bda_kv_project_packed.restype = c_int
    lib.bda_kv_project_packed.argtypes = [vp, i64, i64, c_int, c_int, c_int, ip, ip, vp, vp, i64, c_int, c_int, vp]
    lib.bda_kv_project.restype = c_int
    lib.bda_kv_project.argtypes = [vp, i64, i64, c_int, c_int, c_int, ip, ip, vp, i64, vp, i64,
                                   c_int, c_int, vp]
    lib.bda_dense_project.restype = c_int
    lib.bda_dense_project.argtypes = [vp, i64, i64, c_int, vp, i64, i64, vp, i64, c_int, c_int, vp]
    lib.bda_lowrank_linear.restype = c_int
    lib.bda_lowrank_linear.argtypes = [vp, i64, i64, c_int, c_int, c_int, c_int, vp, vp, vp, i64,
                                       c_int, vp]
    lib.bda_kv_project_backward.restype = c_int
    lib.bda_kv_project_backward.argtypes = [vp, i64, vp, i64, vp, i64, i64, c_int, c_int, c_int, ip, ip,
                                            vp, i64, vp, i64, c_int, c_int, vp]
    lib.bda_kv_project_plan.restype = c_int
    lib.bda_kv_project_plan.argtypes = [i64, c_int, c_int, c_int, ip, ip, i64, i64, i64, c_int, c_int, c_int,
                                        ctypes.POINTER(LaunchPlan)]
    lib.bda_dense_project_plan.restype = c_int
    lib.bda_dense_project_plan.argtypes = [i64, c_int, i64, i64, i64, i64, c_int, c_int, c_int, ctypes.POINTER(LaunchPlan)]
    lib.bda_kv_project_ex.restype = c_int
    lib.bda_kv_project_ex.argtypes = lib.bda_kv_project.argtypes + [c_int]
    lib.bda_dense_project_ex.restype = c_int
    lib.bda_dense_project_ex.argtypes = lib.bda_dense_project.argtypes + [c_int]
    lib.bda_kv_project_backward_ex.restype = c_int
    lib.bda_kv_project_backward_ex.argtypes = lib.bda_kv_project_backward.argtypes + [c_int]
    lib.bda_last_error.restype = ctypes.c_char_p
    lib.bda_last_error.argtypes = []
    lib.bda_version.restype = c_int
    lib.bda_version.argtypes = []
    _lib = lib
    return lib


def exported_symbols() -> Tuple[str, ...]:
    lib = load()
    return tuple(name for name in EXPORTS if hasattr(lib, name))


def bda_last_error() -> str:
    return load().bda_last_error().decode()


def bda_version() -> int:
    return int(load().bda_version())


def _check(status: int) -> None:
    if status != 0:
        raise BdaError(status, bda_last_error())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _dp(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr()) or None
    return int(x) or None


def _int_array(v: Sequence[int]):
    return (ctypes.c_int * len(v))(*[int(i) for i in v])


def bda_prepare(W: np.ndarray, d_c: int, H: int, d_h: int, side: Optional[np.ndarray] = None,
                side_kind: int = SIDE_NONE, mode: int = BASIS_FIRST, explicit_offset: int = 0,
                store_dtype: int = BDA_F64, want_resid: bool = False):
    """Returns (C, side_out or None, basis_offset, resid or None); see include/bda.h."""
    lib = load()
    W = _f64(W)
    K, N = d_c - d_h, H * d_h
    C = np.empty((max(K, 0), N), dtype=np.float64)
    side_c, side_out, d_side, ld_side = None, None, 0, 0
    if side is not None:
        side_c = _f64(side)
        side_out = np.empty_like(side_c)
        d_side = side_c.shape[0] if side_kind == SIDE_Q else side_c.shape[1]
        ld_side = side_c.shape[1]
    off = ctypes.c_int(-1)
    resid = np.full(3, np.nan) if want_resid else None
    _check(lib.bda_prepare(_dp(W), W.shape[1] if W.ndim == 2 else 0, d_c, H, d_h, _dp(side_c),
                           ld_side, d_side, side_kind, mode, explicit_offset, store_dtype,
                           _dp(C), _dp(side_out), ctypes.byref(off), _dp(resid)))
    return C, side_out, int(off.value), resid


def bda_prepare_lowrank(U: np.ndarray, V: np.ndarray, mode: int = BASIS_FIRST,
                        store_dtype: int = BDA_F64, want_resid: bool = False):
    """Returns (Uprime, C, basis_offset, resid or None)."""
    lib = load()
    U, V = _f64(U), _f64(V)
    d_in, r = U.shape
    d_out = V.shape[1]
    if V.shape[0] != r:
        raise ValueError("U is d_in x r and V must be r x d_out")
    Up = np.empty((d_in, r), dtype=np.float64)
    C = np.empty((r, max(d_out - r, 0)), dtype=np.float64)
    off = ctypes.c_int(-1)
    resid = np.full(3, np.nan) if want_resid else None
    _check(lib.bda_prepare_lowrank(_dp(U), _dp(V), d_in, r, d_out, mode, store_dtype, _dp(Up),
                                   _dp(C), ctypes.byref(off), _dp(resid)))
    return Up, C, int(off.value), resid


def bda_kv_project(c, ldc: int, T: int, d_c: int, d_h: int, H: Sequence[int],
                   basis_offset: Sequence[int], C, ldC: int, out, ld_out: int, dtype: int,
                   out_dtype: Optional[int] = None, stream: int = 0) -> None:
    lib = load()
    G = len(H)
    if len(basis_offset) != G:
        raise ValueError("H and basis_offset must have one entry per group")
    _check(lib.bda_kv_project(_ptr(c), ldc, T, d_c, d_h, G, _int_array(H), _int_array(basis_offset),
                              _ptr(C), ldC, _ptr(out), ld_out, dtype,
                              dtype if out_dtype is None else out_dtype, stream or None))


def bda_packed_weights_bytes(d_c: int, d_h: int, H: Sequence[int], dtype: int) -> int:
    return int(load().bda_packed_weights_bytes(d_c, d_h, len(H), _int_array(H), dtype))


def bda_pack_weights(C, ldC: int, d_c: int, d_h: int, H: Sequence[int], dtype: int, packed, stream: int = 0) -> None:
    _check(load().bda_pack_weights(_ptr(C), ldC, d_c, d_h, len(H), _int_array(H), dtype, _ptr(packed), stream or None))


def bda_kv_project_packed(c, ldc: int, T: int, d_c: int, d_h: int, H: Sequence[int],
                          basis_offset: Sequence[int], packed, out, ld_out: int, dtype: int,
                          out_dtype: Optional[int] = None, stream: int = 0) -> None:
    lib = load()
    G = len(H)
    if len(basis_offset) != G:
        raise ValueError("H and basis_offset must have one entry per group")
    _check(lib.bda_kv_project_packed(_ptr(c), ldc, T, d_c, d_h, G, _int_array(H), _int_array(basis_offset),
                                     _ptr(packed), _ptr(out), ld_out, dtype,
                                     dtype if out_dtype is None else out_dtype, stream or None))


def bda_kv_project_ex(c, ldc: int, T: int, d_c: int, d_h: int, H: Sequence[int],
                      basis_offset: Sequence[int], C, ldC: int, out, ld_out: int, dtype: int,
                      out_dtype: Optional[int] = None, stream: int = 0, tile_policy: int = 0) -> None:
    lib = load()
    G = len(H)
    if len(basis_offset) != G:
        raise ValueError("H and basis_offset must have one entry per group")
    _check(lib.bda_kv_project_ex(_ptr(c), ldc, T, d_c, d_h, G, _int_array(H), _int_array(basis_offset),
                                 _ptr(C), ldC, _ptr(out), ld_out, dtype,
                                 dtype if out_dtype is None else out_dtype, stream or None, int(tile_policy)))


def bda_prepare_device(W, ldw: int, w_dtype: int, d_c: int, H: int, d_h: int, basis_offset: int,
                       C, ldC: int, c_dtype: int, singular_head=None, stream: int = 0) -> None:
    lib = load()
    _check(lib.bda_prepare_device(_ptr(W), ldw, w_dtype, d_c, H, d_h, basis_offset, _ptr(C), ldC, c_dtype,
                                  _ptr(singular_head), stream or None))


def bda_prepare_device_workspace_bytes(d_c: int, H: int, d_h: int, mode: int, want_residuals: bool = False) -> int:
    return int(load().bda_prepare_device_workspace_bytes(d_c, H, d_h, mode, 1 if want_residuals else 0))


def bda_prepare_device_ex(W, ldw: int, w_dtype: int, d_c: int, H: int, d_h: int, C, ldC: int, c_dtype: int,
                          side=None, ld_side: int = 0, d_side: int = 0, side_kind: int = SIDE_NONE,
                          side_out=None, ld_side_out: int = 0, mode: int = BASIS_FIRST, explicit_offset: int = 0,
                          basis_offset_out=None, resid_out=None, singular_head=None,
                          workspace=None, workspace_bytes: int = 0, stream: int = 0) -> None:
    """All array arguments are device arrays (anything with data_ptr()); see include/bda.h."""
    lib = load()
    _check(lib.bda_prepare_device_ex(_ptr(W), ldw, w_dtype, d_c, H, d_h, _ptr(side), ld_side, d_side, side_kind,
                                     mode, explicit_offset, _ptr(C), ldC, _ptr(side_out), ld_side_out, c_dtype,
                                     _ptr(basis_offset_out), _ptr(resid_out), _ptr(singular_head),
                                     _ptr(workspace), int(workspace_bytes), stream or None))


def bda_prepare_device_static(W, ldw: int, w_dtype: int, d_c: int, H: int, d_h: int, C, ldC: int, c_dtype: int,
                              side=None, ld_side: int = 0, d_side: int = 0, side_kind: int = SIDE_NONE,
                              side_out=None, ld_side_out: int = 0, mode: int = BASIS_FIRST, explicit_offset: int = 0,
                              basis_offset_out=None, resid_out=None, singular_head=None, stream: int = 0) -> None:
    """bda_prepare_device_ex without a workspace (the library's built-in scratch); see include/bda.h."""
    lib = load()
    _check(lib.bda_prepare_device_static(_ptr(W), ldw, w_dtype, d_c, H, d_h, _ptr(side), ld_side, d_side, side_kind,
                                         mode, explicit_offset, _ptr(C), ldC, _ptr(side_out), ld_side_out, c_dtype,
                                         _ptr(basis_offset_out), _ptr(resid_out), _ptr(singular_head), stream or None))


def bda_dense_project(c, ldc: int, T: int, d_c: int, W, ldW: int, N: int, out, ld_out: int,
                      dtype: int, out_dtype: Optional[int] = None, stream: int = 0) -> None:
    lib = load()
    _check(lib.bda_dense_project(_ptr(c), ldc, T, d_c, _ptr(W), ldW, N, _ptr(out), ld_out, dtype,
                                 dtype if out_dtype is None else out_dtype, stream or None))


def bda_dense_project_ex(c, ldc: int, T: int, d_c: int, W, ldW: int, N: int, out, ld_out: int,
                         dtype: int, out_dtype: Optional[int] = None, stream: int = 0, tile_policy: int = 0) -> None:
    lib = load()
    _check(lib.bda_dense_project_ex(_ptr(c), ldc, T, d_c, _ptr(W), ldW, N, _ptr(out), ld_out, dtype,
                                    dtype if out_dtype is None else out_dtype, stream or None, int(tile_policy)))


def bda_lowrank_linear(x, ldx: int, T: int, d_in: int, r: int, d_out: int, basis_offset: int,
                       Uprime, C, out, ld_out: int, dtype: int, stream: int = 0) -> None:
    lib = load()
    _check(lib.bda_lowrank_linear(_ptr(x), ldx, T, d_in, r, d_out, basis_offset, _ptr(Uprime),
                                  _ptr(C), _ptr(out), ld_out, dtype, stream or None))


def bda_kv_project_backward(c, ldc: int, d_out, ld_dout: int, C, ldC: int, T: int, d_c: int, d_h: int,
                            H: Sequence[int], basis_offset: Sequence[int], grad_c, ld_gc: int,
                            grad_C, ld_gC: int, dtype: int, grad_dtype: Optional[int] = None,
                            stream: int = 0) -> None:
    lib = load()
    G = len(H)
    if len(basis_offset) != G:
        raise ValueError("H and basis_offset must have one entry per group")
    _check(lib.bda_kv_project_backward(_ptr(c), ldc, _ptr(d_out), ld_dout, _ptr(C), ldC, T, d_c, d_h, G,
                                       _int_array(H), _int_array(basis_offset), _ptr(grad_c), ld_gc,
                                       _ptr(grad_C), ld_gC, dtype,
                                       dtype if grad_dtype is None else grad_dtype, stream or None))


def bda_kv_project_backward_ex(c, ldc: int, d_out, ld_dout: int, C, ldC: int, T: int, d_c: int, d_h: int,
                               H: Sequence[int], basis_offset: Sequence[int], grad_c, ld_gc: int,
                               grad_C, ld_gC: int, dtype: int, grad_dtype: Optional[int] = None,
                               stream: int = 0, tile_policy: int = 0) -> None:
    lib = load()
    G = len(H)
    if len(basis_offset) != G:
        raise ValueError("H and basis_offset must have one entry per group")
    _check(lib.bda_kv_project_backward_ex(_ptr(c), ldc, _ptr(d_out), ld_dout, _ptr(C), ldC, T, d_c, d_h, G,
                                          _int_array(H), _int_array(basis_offset), _ptr(grad_c), ld_gc,
                                          _ptr(grad_C), ld_gC, dtype,
                                          dtype if grad_dtype is None else grad_dtype, stream or None,
                                          int(tile_policy)))


def bda_kv_project_plan(T: int, d_c: int, d_h: int, H: Sequence[int], basis_offset: Sequence[int], dtype: int,
                        out_dtype: Optional[int] = None, ldc: Optional[int] = None, ldC: Optional[int] = None,
                        ld_out: Optional[int] = None, tile_policy: int = 0) -> dict:
    lib = load()
    N = int(sum(H)) * d_h
    plan = LaunchPlan()
    _check(lib.bda_kv_project_plan(T, d_c, d_h, len(H), _int_array(H), _int_array(basis_offset), ldc or d_c, ldC or N,
                                   ld_out or N, dtype, dtype if out_dtype is None else out_dtype, int(tile_policy),
                                   ctypes.byref(plan)))
    return plan.as_dict()


def bda_dense_project_plan(T: int, d_c: int, N: int, dtype: int, out_dtype: Optional[int] = None,
                           ldc: Optional[int] = None, ldW: Optional[int] = None, ld_out: Optional[int] = None,
                           tile_policy: int = 0) -> dict:
    lib = load()
    plan = LaunchPlan()
    _check(lib.bda_dense_project_plan(T, d_c, N, ldc or d_c, ldW or N, ld_out or N, dtype,
                                      dtype if out_dtype is None else out_dtype, int(tile_policy), ctypes.byref(plan)))
    return plan.as_dict()
