"""Device plumbing for the GPU tests: numpy <-> torch device buffers, calls through the C ABI."""
import numpy as np
import torch

import bda_workloads as wl
import paper_2510_01718_amd as bda

_TORCH = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.int16}


def to_device(stored: np.ndarray, dtype: int, ld: int = None, row_pad_value: float = 0.0) -> torch.Tensor:
    """Uploads a 2-D stored array; with `ld` > columns the rows are padded (strided layout)."""
    a = np.ascontiguousarray(stored)
    if dtype == wl.BF16:
        a = a.view(np.int16)
    rows, cols = a.shape
    if ld is None or ld == cols:
        return torch.from_numpy(a.copy()).cuda()
    buf = torch.zeros((rows, ld), dtype=_TORCH[dtype])
    buf[:, :cols] = torch.from_numpy(a.copy())
    return buf.cuda()


def new_out(rows: int, ld: int, dtype: int, fill=None) -> torch.Tensor:
    t = torch.empty((rows, ld), dtype=_TORCH[dtype], device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def to_host64(t: torch.Tensor, dtype: int, cols: int = None) -> np.ndarray:
    a = t.cpu().numpy()
    if cols is not None:
        a = a[:, :cols]
    if dtype == wl.BF16:
        return wl.from_storage(np.ascontiguousarray(a).view(np.uint16), wl.BF16)
    return a.astype(np.float64)


def stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def kv_project(c_stored, C_stored, d_c, d_h, H, offs, dtype, out_dtype=None, ldc=None, ldC=None,
               ld_out=None, fill=None, policy=0, extra_rows=0):
    """Runs bda_kv_project (bda_kv_project_ex for a tile policy other than 0) on stored inputs and
    returns (float64 output, raw device tensor).  `extra_rows` rows are allocated past the T the call
    is given (with `fill`, a guard against writes past the last token)."""
    out_dtype = dtype if out_dtype is None else out_dtype
    T = c_stored.shape[0]
    N = int(sum(H)) * d_h
    ldc = ldc or d_c
    ldC = ldC or N
    ld_out = ld_out or N
    c_d = to_device(c_stored, dtype, ldc)
    C_d = to_device(C_stored, dtype, ldC)
    out_d = new_out(max(T, 1) + extra_rows, ld_out, out_dtype, fill)
    if policy:
        bda.bda_kv_project_ex(c_d, ldc, T, d_c, d_h, H, offs, C_d, ldC, out_d, ld_out, dtype, out_dtype, stream(), policy)
    else:
        bda.bda_kv_project(c_d, ldc, T, d_c, d_h, H, offs, C_d, ldC, out_d, ld_out, dtype, out_dtype, stream())
    torch.cuda.synchronize()
    return to_host64(out_d[:T], out_dtype, N), out_d
