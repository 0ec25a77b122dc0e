"""bda_prepare_device_static (the entry point that allocates nothing: its partial results live in an
array that is part of the library's device code) against bda_prepare_device_ex with a caller's workspace.

Both run the same kernels on the same inputs in the same order, so every output must be equal bit for
bit: C, the companion block, the chosen window, the three residuals, the singular-head flag.  Two calls
in a row share the built-in array; the second is smaller (fewer heads, fewer candidate windows, narrower
heads), so whatever the first left behind must not matter.  Head widths above 128 keep their basis blocks
in the array as well."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import bda_workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402
import paper_2510_01718_amd as bda  # noqa: E402

pytestmark = pytest.mark.gpu

_TDT = {wl.F64: torch.float64, wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.int16}


def _call(static, W_d, side_d, side_kind, d_c, H, d_h, d_side, mode, c_dtype):
    """One preparation straight through the C ABI (ctypes on the loaded library); returns every output."""
    lib = bda.load()
    N = H * d_h
    C_d = torch.full((d_c - d_h, N), -7, dtype=_TDT[c_dtype], device="cuda")
    so_d = torch.full(tuple(side_d.shape), -7, dtype=_TDT[c_dtype], device="cuda")
    off_d = torch.full((1,), -99, dtype=torch.int32, device="cuda")
    res_d = torch.zeros(3, dtype=torch.float64, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    ld_side = side_d.shape[1]
    vp = ctypes.c_void_p
    head = [vp(W_d.data_ptr()), N, wl.F64, d_c, H, d_h, vp(side_d.data_ptr()), ld_side, d_side, side_kind, mode, 0,
            vp(C_d.data_ptr()), N, vp(so_d.data_ptr()), ld_side, c_dtype, vp(off_d.data_ptr()), vp(res_d.data_ptr()), vp(flag.data_ptr())]
    if static:
        rc = lib.bda_prepare_device_static(*head, vp(gh.stream()))
    else:
        nb = int(lib.bda_prepare_device_workspace_bytes(d_c, H, d_h, mode, 1))
        ws = torch.full((nb,), 0xA5, dtype=torch.uint8, device="cuda")
        rc = lib.bda_prepare_device_ex(*head, vp(ws.data_ptr()), nb, vp(gh.stream()))
    assert rc == 0, lib.bda_last_error()
    torch.cuda.synchronize()
    return [C_d.cpu().numpy(), so_d.cpu().numpy(), off_d.cpu().numpy(), res_d.cpu().numpy().view(np.int64), flag.cpu().numpy()]


def _inputs(d_c, H, d_h, d_side, side_kind, seed):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((d_c, H * d_h)) * 0.05
    W[1, :d_h] = W[0, :d_h] + 2e-4 * rng.standard_normal(d_h)          # a weak first window: the search has something to decide
    side = rng.standard_normal((d_side, H * d_h) if side_kind == bda.SIDE_Q else (H * d_h, d_side)) * 0.05
    return torch.from_numpy(W).cuda(), torch.from_numpy(side).cuda()


def test_static_entry_point_equals_workspace_entry_point_on_two_calls_in_a_row():
    cases = [  # the second of each pair is the smaller one
        [(256, 6, 64, 48, bda.SIDE_Q, bda.BASIS_OFFSET_SEARCH, wl.BF16), (128, 3, 32, 20, bda.SIDE_O, bda.BASIS_RESIDUAL_MIN, wl.F16)],
        [(512, 3, 256, 16, bda.SIDE_O, bda.BASIS_RESIDUAL_MIN, wl.F16), (448, 2, 192, 8, bda.SIDE_Q, bda.BASIS_FIRST, wl.BF16)],
    ]
    for pair in cases:
        prepared = []
        for i, (d_c, H, d_h, d_side, side_kind, mode, c_dtype) in enumerate(pair):
            W_d, side_d = _inputs(d_c, H, d_h, d_side, side_kind, seed=900 + i)
            want = _call(False, W_d, side_d, side_kind, d_c, H, d_h, d_side, mode, c_dtype)
            prepared.append((W_d, side_d, side_kind, d_c, H, d_h, d_side, mode, c_dtype, want))
        for args in prepared:                      # the two static calls back to back, nothing in between
            got = _call(True, *args[:-1])
            for g, w, name in zip(got, args[-1], ("C", "companion", "window", "residuals", "singular_head")):
                assert np.array_equal(g, w), (name, args[3:9])
            assert got[2][0] >= 0 and got[4][0] == 0


def test_static_entry_point_rejects_what_does_not_fit_its_array():
    lib = bda.load()
    fake = ctypes.c_void_p(0x1000)
    # 255 candidate windows x 8192 heads x 1 part x 8 bytes of partial sums = 16 MiB: twice the array
    H, d_h, d_c = 8192, 128, 128 + 16 * 254
    rc = lib.bda_prepare_device_static(fake, H * d_h, 3, d_c, H, d_h, None, 0, 0, 0, bda.BASIS_OFFSET_SEARCH, 0,
                                       fake, H * d_h, None, 0, 1, fake, None, None, None)
    assert rc == -1
    msg = lib.bda_last_error()
    assert b"built-in scratch" in msg and b"8388608" in msg and b"bda_prepare_device_ex" in msg
