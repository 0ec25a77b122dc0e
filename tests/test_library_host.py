"""CPU-only tests of libbda: the shared library loads, exports every symbol the header declares,
its host-side prepare agrees with the oracle, and argument errors are reported, not crashed on.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import bda_workloads as wl
import oracle
import paper_2510_01718_amd as bda

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bda.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(bda_[a-z_0-9]+)\s*\(", header))
    assert {"bda_prepare", "bda_kv_project", "bda_lowrank_linear", "bda_dense_project"} <= declared
    lib = ctypes.CDLL(bda.lib_path())
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in bda.h but not exported"
    assert set(bda.exported_symbols()) == declared
    assert bda.bda_version() >= 100


def test_enum_values_match_header():
    header = open(os.path.join(ROOT, "include", "bda.h")).read()
    for name, val in [("BDA_F32", bda.BDA_F32), ("BDA_F16", bda.BDA_F16), ("BDA_BF16", bda.BDA_BF16),
                      ("BDA_F64", bda.BDA_F64), ("BDA_BASIS_FIRST", bda.BASIS_FIRST),
                      ("BDA_BASIS_LAST", bda.BASIS_LAST), ("BDA_BASIS_RESIDUAL_MIN", bda.BASIS_RESIDUAL_MIN),
                      ("BDA_BASIS_OFFSET_SEARCH", bda.BASIS_OFFSET_SEARCH), ("BDA_BASIS_EXPLICIT", bda.BASIS_EXPLICIT),
                      ("BDA_SIDE_NONE", bda.SIDE_NONE), ("BDA_SIDE_Q", bda.SIDE_Q), ("BDA_SIDE_O", bda.SIDE_O)]:
        m = re.search(rf"\b{name}\s*=\s*(-?\d+)", header)
        assert m and int(m.group(1)) == val, name
    # the workload module and the oracle use the same dtype tags (plain data)
    assert (wl.F32, wl.F16, wl.BF16, wl.F64) == (bda.BDA_F32, bda.BDA_F16, bda.BDA_BF16, bda.BDA_F64)
    assert (oracle.F32, oracle.F16, oracle.BF16, oracle.F64) == (wl.F32, wl.F16, wl.BF16, wl.F64)


@pytest.mark.parametrize("mode", [bda.BASIS_FIRST, bda.BASIS_LAST, bda.BASIS_RESIDUAL_MIN,
                                  bda.BASIS_OFFSET_SEARCH, bda.BASIS_EXPLICIT])
@pytest.mark.parametrize("side_kind", [bda.SIDE_NONE, bda.SIDE_Q, bda.SIDE_O])
@pytest.mark.parametrize("store", [bda.BDA_F16, bda.BDA_BF16, bda.BDA_F32])
def test_prepare_matches_oracle(mode, side_kind, store):
    rng = np.random.default_rng(100 + mode * 10 + side_kind)
    d_c, H, d_h = 80, 3, 16
    W = rng.standard_normal((d_c, H * d_h)) * 0.1
    side = None
    if side_kind == bda.SIDE_Q:
        side = rng.standard_normal((24, H * d_h))
    elif side_kind == bda.SIDE_O:
        side = rng.standard_normal((H * d_h, 40))
    C, s_out, off, resid = bda.bda_prepare(W, d_c, H, d_h, side, side_kind, mode, 32, store, want_resid=True)
    Co, so, offo, ro = oracle.prepare(W, d_c, H, d_h, side, side_kind, mode, 32, store)
    assert off == offo                                        # index selection is exact
    scale = np.max(np.abs(Co))
    assert np.max(np.abs(C - Co)) <= 1e-9 * scale
    if side is not None:
        assert np.max(np.abs(s_out - so)) <= 1e-10 * np.max(np.abs(so))
    assert resid[2] == pytest.approx(ro[offo], rel=1e-6)
    if 0 in ro:
        assert resid[0] == pytest.approx(ro[0], rel=1e-6)
    if d_c - d_h in ro:
        assert resid[1] == pytest.approx(ro[d_c - d_h], rel=1e-6)


def test_prepare_tiny_config_basis_rows_identity():
    w = wl.kv_workload("tiny")
    C, _, off, _ = bda.bda_prepare(w.W, w.d_c, 2, w.d_h)
    assert off == 0 and C.shape == (48, 32)
    for h in range(2):
        Wh = w.W[:, h * 16:(h + 1) * 16]
        full = Wh @ np.linalg.inv(Wh[:16])
        assert np.max(np.abs(full[:16] - np.eye(16))) < 1e-10
        assert np.max(np.abs(full[16:] - C[:, h * 16:(h + 1) * 16])) < 1e-9


def test_prepare_picks_other_window_when_first_is_ill_conditioned():
    rng = np.random.default_rng(7)
    d_c, H, d_h = 64, 2, 16
    W = rng.standard_normal((d_c, H * d_h))
    for h in range(H):
        W[1, h * d_h:(h + 1) * d_h] = W[0, h * d_h:(h + 1) * d_h] * (1 + 1e-6)
    _, _, off, resid = bda.bda_prepare(W, d_c, H, d_h, mode=bda.BASIS_RESIDUAL_MIN, store_dtype=bda.BDA_F16, want_resid=True)
    _, _, offo, _ = oracle.prepare(W, d_c, H, d_h, mode=oracle.RESIDUAL_MIN, store_dtype=oracle.F16)
    assert off == offo == d_c - d_h
    assert resid[0] > resid[1]


def test_prepare_tie_keeps_first():
    d_c, d_h = 10, 3
    W = np.vstack([np.eye(d_h), np.arange(12, dtype=np.float64).reshape(4, 3), np.eye(d_h)])
    _, _, off, resid = bda.bda_prepare(W, d_c, 1, d_h, mode=bda.BASIS_RESIDUAL_MIN, store_dtype=bda.BDA_F64, want_resid=True)
    assert off == 0 and resid[0] == resid[1]


def test_prepare_singular_and_invalid():
    with pytest.raises(bda.BdaError) as e:
        bda.bda_prepare(np.zeros((8, 4)), 8, 1, 4)
    assert e.value.status == -4 and "head 0" in e.value.message
    W = np.ones((8, 4))
    W[:4] = np.eye(4)
    W[1] = W[0]                                    # two equal basis rows in the first window
    with pytest.raises(bda.BdaError) as e:
        bda.bda_prepare(W, 8, 1, 4)
    assert e.value.status == -4
    with pytest.raises(bda.BdaError) as e:
        bda.bda_prepare(np.ones((8, 4)), 8, 1, 8)          # d_h >= d_c
    assert e.value.status == -1
    with pytest.raises(bda.BdaError) as e:
        bda.bda_prepare(np.ones((8, 4)), 8, 1, 4, mode=bda.BASIS_EXPLICIT, explicit_offset=5)
    assert e.value.status == -1
    # residual-min skips a singular window instead of failing
    rng = np.random.default_rng(3)
    W = rng.standard_normal((12, 4))
    W[1] = W[0]
    _, _, off, _ = bda.bda_prepare(W, 12, 1, 4, mode=bda.BASIS_RESIDUAL_MIN)
    assert off == 8


@pytest.mark.parametrize("mode", [bda.BASIS_FIRST, bda.BASIS_LAST, bda.BASIS_RESIDUAL_MIN])
def test_prepare_lowrank_matches_oracle(mode):
    rng = np.random.default_rng(21)
    d_in, r, d_out = 40, 8, 29
    U = rng.standard_normal((d_in, r))
    V = rng.standard_normal((r, d_out))
    Up, C, off, resid = bda.bda_prepare_lowrank(U, V, mode, bda.BDA_F16, want_resid=True)
    Upo, Co, offo, ro = oracle.prepare_lowrank(U, V, mode, oracle.F16)
    assert off == offo
    assert np.max(np.abs(Up - Upo)) <= 1e-11 * np.max(np.abs(Upo))
    assert np.max(np.abs(C - Co)) <= 1e-9 * np.max(np.abs(Co))
    if mode == bda.BASIS_RESIDUAL_MIN:
        assert resid[2] == pytest.approx(ro[offo], rel=1e-6)


def test_device_entry_points_reject_bad_arguments_without_a_gpu():
    """Validation happens before any HIP call, so these return an error code on a CPU-only box."""
    lib = bda.load()
    H = (ctypes.c_int * 1)(2)
    off = (ctypes.c_int * 1)(0)
    bad_off = (ctypes.c_int * 1)(49)
    fake = ctypes.c_void_p(0x1000)
    # d_h >= d_c
    assert lib.bda_kv_project(fake, 64, 4, 64, 64, 1, H, off, fake, 32, fake, 32, 1, 1, None) == -1
    # offset out of range
    assert lib.bda_kv_project(fake, 64, 4, 64, 16, 1, H, bad_off, fake, 32, fake, 32, 1, 1, None) == -1
    assert b"basis_offset" in lib.bda_last_error()
    # out_dtype neither dtype nor f32
    assert lib.bda_kv_project(fake, 64, 4, 64, 16, 1, H, off, fake, 32, fake, 32, 1, 2, None) == -3
    # too many groups
    assert lib.bda_kv_project(fake, 64, 4, 64, 16, 9, H, off, fake, 32, fake, 32, 1, 1, None) == -1
    # ld too small
    assert lib.bda_kv_project(fake, 8, 4, 64, 16, 1, H, off, fake, 32, fake, 32, 1, 1, None) == -1
    # NULL pointer with T > 0
    assert lib.bda_kv_project(None, 64, 4, 64, 16, 1, H, off, fake, 32, fake, 32, 1, 1, None) == -1
    # out overlapping c
    assert lib.bda_kv_project(fake, 64, 4, 64, 16, 1, H, off, ctypes.c_void_p(0x100000), 32, fake, 32, 1, 1, None) == -1
    assert b"overlap" in lib.bda_last_error()
    # T = 0 is a successful no-op even with NULL buffers
    assert lib.bda_kv_project(None, 64, 0, 64, 16, 1, H, off, None, 32, None, 32, 1, 1, None) == 0
    assert lib.bda_last_error() == b""
    # GPU preparation: NULL, window out of range, head too wide for the LDS-resident inverse, bad dtype
    assert lib.bda_prepare_device(None, 32, 3, 64, 2, 16, 0, fake, 32, 1, None, None) == -1
    assert lib.bda_prepare_device(fake, 32, 3, 64, 2, 16, 49, fake, 32, 1, None, None) == -1
    assert b"basis_offset" in lib.bda_last_error()
    assert lib.bda_prepare_device(fake, 512, 3, 1024, 2, 256, 0, fake, 512, 1, None, None) == -1
    assert lib.bda_prepare_device(fake, 32, 7, 64, 2, 16, 0, fake, 32, 1, None, None) == -3
    assert lib.bda_prepare_device(fake, 16, 3, 64, 2, 16, 0, fake, 32, 1, None, None) == -1
    # the long form: a search needs a workspace (the message says how much), a companion its output, a
    # search somewhere to put the chosen window; no more than 256 candidate windows; d_h up to 256
    ex = lib.bda_prepare_device_ex
    need = lib.bda_prepare_device_workspace_bytes(64, 2, 16, 2, 0)
    assert need == 1024 + 256 * ((2 * 2 * 64 * 8 + 255) // 256)      # flags + 2 candidates x 2 heads x 64 parts of a sum
    assert lib.bda_prepare_device_workspace_bytes(64, 2, 16, 0, 0) == 0 and lib.bda_prepare_device_workspace_bytes(64, 2, 64, 0, 0) == 0
    assert lib.bda_prepare_device_workspace_bytes(1024, 2, 256, 0, 0) == 1024 + 2 * 256 * 256 * 8
    assert ex(fake, 32, 3, 64, 2, 16, None, 0, 0, 0, 2, 0, fake, 32, None, 0, 1, fake, None, None, None, 0, None) == -1
    assert str(need).encode() in lib.bda_last_error()
    assert ex(fake, 32, 3, 64, 2, 16, None, 0, 0, 0, 2, 0, fake, 32, None, 0, 1, fake, None, None, fake, need - 1, None) == -1
    assert ex(fake, 32, 3, 64, 2, 16, None, 0, 0, 0, 2, 0, fake, 32, None, 0, 1, None, None, None, fake, need, None) == -1
    assert b"basis_offset_out" in lib.bda_last_error()
    assert ex(fake, 32, 3, 64, 2, 16, fake, 32, 8, 1, 0, 0, fake, 32, None, 32, 1, None, None, None, None, 0, None) == -1
    assert b"companion" in lib.bda_last_error()
    assert ex(fake, 32, 3, 64, 2, 16, fake, 16, 8, 1, 0, 0, fake, 32, fake, 32, 1, None, None, None, None, 0, None) == -1
    assert ex(fake, 16, 3, 8192, 1, 16, None, 0, 0, 0, 3, 0, fake, 16, None, 0, 1, fake, None, None, fake, 1 << 30, None) == -1
    assert b"candidate" in lib.bda_last_error()
    assert ex(fake, 1028, 3, 1024, 4, 257, None, 0, 0, 0, 0, 0, fake, 1028, None, 0, 1, None, None, None, None, 0, None) == -1
    assert ex(fake, 512, 3, 1024, 2, 256, None, 0, 0, 0, 0, 0, fake, 512, None, 0, 1, None, None, None, None, 0, None) == -1   # d_h > 128 needs a workspace
    assert ex(fake, 32, 3, 64, 2, 16, None, 0, 0, 0, 9, 0, fake, 32, None, 0, 1, None, None, None, None, 0, None) == -1
    # gradients: bad window, ld too small, a gradient on top of an input, grad dtype, nothing asked for
    far = ctypes.c_void_p(0x900000)
    farther = ctypes.c_void_p(0xA00000)
    bwd = lib.bda_kv_project_backward
    assert bwd(fake, 64, fake, 32, fake, 32, 4, 64, 16, 1, H, bad_off, far, 64, farther, 32, 1, 1, None) == -1
    assert b"basis_offset" in lib.bda_last_error()
    assert bwd(fake, 64, far, 16, fake, 32, 4, 64, 16, 1, H, off, far, 64, farther, 32, 1, 1, None) == -1
    assert bwd(fake, 64, far, 32, fake, 32, 4, 64, 16, 1, H, off, farther, 32, None, 32, 1, 1, None) == -1
    assert bwd(fake, 64, fake, 32, fake, 32, 4, 64, 16, 1, H, off, fake, 64, farther, 32, 1, 1, None) == -1
    assert b"overlaps" in lib.bda_last_error()
    assert bwd(fake, 64, far, 32, fake, 32, 4, 64, 16, 1, H, off, None, 64, farther, 32, 1, 2, None) == -3
    assert bwd(None, 64, far, 32, None, 32, 4, 64, 16, 1, H, off, None, 64, farther, 32, 1, 1, None) == -1
    assert b"needs c" in lib.bda_last_error()
    assert bwd(None, 64, None, 32, None, 32, 4, 64, 16, 1, H, off, None, 64, None, 32, 1, 1, None) == 0
    assert lib.bda_dense_project(fake, 64, 4, 64, fake, 8, 32, fake, 32, 1, 1, None) == -1
    assert lib.bda_lowrank_linear(fake, 64, 4, 64, 8, 40, 3, fake, fake, fake, 40, 1, None) == -1
    # packed weights: 16-bit only, group widths multiples of 32, at most 64 tokens, shapes the few-token kernels take
    H32, H3 = (ctypes.c_int * 1)(2), (ctypes.c_int * 2)(1, 3)
    assert lib.bda_packed_weights_bytes(96, 32, 1, H32, 1) == 64 * 64 * 2
    assert lib.bda_packed_weights_bytes(96, 32, 1, H32, 0) == 0 and b"16-bit" in lib.bda_last_error()
    assert lib.bda_packed_weights_bytes(64, 16, 2, H3, 1) == 0 and b"multiple of 32" in lib.bda_last_error()
    assert lib.bda_packed_weights_bytes(64, 16, 1, H32, 2) == 48 * 32 * 2
    assert lib.bda_pack_weights(fake, 60, 96, 32, 1, H32, 1, far, None) == -1            # ldC < N
    assert lib.bda_pack_weights(fake, 64, 96, 32, 1, H32, 1, ctypes.c_void_p(0x1008), None) == -1
    assert lib.bda_pack_weights(fake, 64, 96, 32, 1, H32, 1, ctypes.c_void_p(0x1100), None) == -1 and b"overlaps" in lib.bda_last_error()
    assert lib.bda_pack_weights(fake, 64, 96, 32, 1, H32, 3, far, None) == -3
    pk = lib.bda_kv_project_packed
    assert pk(fake, 96, 65, 96, 32, 1, H32, off, far, farther, 64, 1, 1, None) == -1 and b"64 tokens" in lib.bda_last_error()
    assert pk(fake, 96, 4, 96, 32, 1, H32, (ctypes.c_int * 1)(65), far, farther, 64, 1, 1, None) == -1 and b"basis_offset" in lib.bda_last_error()
    assert pk(fake, 96, 4, 96, 32, 1, H32, off, far, farther, 64, 0, 0, None) == -3
    assert pk(fake, 96, 4, 96, 32, 1, H32, off, far, fake, 64, 1, 1, None) == -1 and b"overlaps" in lib.bda_last_error()
    assert pk(fake, 100, 4, 96, 32, 1, H32, off, far, farther, 64, 1, 1, None) == -1 and b"canonical" in lib.bda_last_error()
    assert pk(None, 96, 0, 96, 32, 1, H32, off, None, None, 64, 1, 1, None) == 0
    # a tile policy outside 0 .. 7 is refused before anything else is looked at
    assert lib.bda_kv_project_ex(fake, 64, 4, 64, 16, 1, H, off, fake, 32, far, 32, 1, 1, None, 8) == -1
    assert b"tile_policy" in lib.bda_last_error()
    assert lib.bda_dense_project_ex(fake, 64, 4, 64, fake, 32, 32, far, 32, 1, 1, None, -1) == -1
    assert lib.bda_kv_project_backward_ex(None, 64, None, 32, None, 32, 4, 64, 16, 1, H, off, None, 64, None, 32, 1, 1, None, 8) == -1


def test_workload_recipe_is_stable():
    """The seeded generator is part of the test contract: same seed -> same bits."""
    a = wl.kv_workload("tiny")
    b = wl.kv_workload("tiny")
    assert np.array_equal(a.c_stored, b.c_stored) and np.array_equal(a.W, b.W)
    assert a.c_stored.dtype == np.float32 and a.c.shape == (64, 64) and a.W.shape == (64, 32)
    d8 = wl.kv_workload("decode", T=8)
    d1 = wl.kv_workload("decode", T=1)
    assert np.array_equal(d8.W, d1.W)                       # weights do not depend on T
    v = wl.kv_workload("v2lite", T=16)
    assert np.array_equal(v.W, d8.W)
    rms = np.sqrt(np.mean(from64(v.c) ** 2, axis=1))
    assert np.allclose(rms, 1.0, atol=2e-3)


def from64(x):
    return np.asarray(x, dtype=np.float64)


# ------------------------------------------------------------------ launch-shape rules (host logic)
def _plan(T, H, offs, dtype, d_c=512, d_h=128, **kw):
    return bda.bda_kv_project_plan(T, d_c, d_h, H, offs, dtype, **kw)


def test_launch_plan_benchmark_shapes():
    """The tile choice and schedule of the configurations that are benchmarked (no GPU needed)."""
    p = _plan(4096, [16, 16], [0, 0], bda.BDA_F16)                      # main workload: one 256 x 256 tile per CU
    assert (p["kernel"], p["tile_tokens"], p["tile_columns"]) == (bda.KERNEL_LEAN, 256, 256)
    assert (p["token_tiles"], p["column_tiles"], p["workgroups"], p["threads"]) == (16, 16, 256, 512)
    assert (p["rounds"], p["tile_by_tile"], p["super_m"], p["super_n"]) == (1, 0, 4, 8)
    assert p["lds_bytes"] == 160 * 1024
    p = _plan(8192, [128, 128], [0, 0], bda.BDA_BF16)                   # V3 shape: 16 tiles per CU
    assert (p["kernel"], p["tile_tokens"], p["rounds"], p["workgroups"]) == (bda.KERNEL_LEAN, 256, 16, 256)
    for T in (1, 8, 32, 64):                                            # decode: one workgroup per 32 columns
        p = _plan(T, [16, 16], [0, 0], bda.BDA_F16)
        assert (p["kernel"], p["column_tiles"], p["workgroups"]) == (bda.KERNEL_DECODE, 128, 128)
    for T in (65, 128):                                                 # up to 128 tokens while every slice has a CU
        p = _plan(T, [16, 16], [0, 0], bda.BDA_F16)
        assert (p["kernel"], p["tile_tokens"], p["tile_columns"], p["workgroups"]) == (bda.KERNEL_DECODE, 128, 32, 128)
        p = _plan(T, [40, 40], [0, 0], bda.BDA_F16)                     # 320 slices of 32: 160 slices of 64 instead
        assert (p["kernel"], p["tile_columns"], p["workgroups"], p["lds_bytes"]) == (bda.KERNEL_DECODE, 64, 160, 144 * 1024)
        assert _plan(T, [96, 96], [0, 0], bda.BDA_F16)["kernel"] == bda.KERNEL_LEAN      # 384 slices of 64: tiles
        assert _plan(T, [40, 40], [0, 0], bda.BDA_F16, d_c=1024)["kernel"] == bda.KERNEL_LEAN   # K = 896 > 384
    # more than 128 tokens: token tiles of 128 while all the workgroups fit the chip at once
    p = _plan(256, [16, 16], [0, 0], bda.BDA_F16)
    assert (p["kernel"], p["tile_columns"], p["token_tiles"], p["workgroups"]) == (bda.KERNEL_DECODE, 32, 2, 256)
    p = _plan(512, [15, 17], [0, 0], bda.BDA_F16)                       # (group widths off the 256 grid: no lean kernel)
    assert (p["kernel"], p["tile_columns"], p["token_tiles"], p["workgroups"]) == (bda.KERNEL_DECODE, 64, 4, 256)
    p = _plan(512, [16, 16], [0, 0], bda.BDA_F16)                       # where the lean kernel applies: one round of its 64-token tiles
    assert (p["kernel"], p["tile_tokens"], p["tile_columns"], p["token_tiles"], p["workgroups"]) == (bda.KERNEL_LEAN, 64, 256, 8, 128)
    assert _plan(600, [16, 16], [0, 0], bda.BDA_F16)["kernel"] == bda.KERNEL_LEAN
    p = _plan(64, [128, 128], [0, 0], bda.BDA_BF16)                     # wide output: 128-column slices
    assert (p["kernel"], p["tile_columns"], p["workgroups"], p["lds_bytes"]) == (bda.KERNEL_DECODE, 128, 256, 144 * 1024)
    p = _plan(16, [128, 128], [0, 0], bda.BDA_BF16)
    assert (p["kernel"], p["tile_tokens"], p["tile_columns"], p["lds_bytes"]) == (bda.KERNEL_DECODE, 32, 128, 120 * 1024)
    assert _plan(64, [64, 64], [0, 0], bda.BDA_BF16)["tile_columns"] == 32       # 128 slices of 128: stays with 32-column slices
    assert _plan(64, [128, 128], [0, 0], bda.BDA_BF16, d_c=1024)["tile_columns"] == 32   # K = 896 > 384
    p = bda.bda_dense_project_plan(8192, 4096, 1024, bda.BDA_F16)       # BD linear, first GEMM
    assert (p["kernel"], p["tile_tokens"], p["token_tiles"] * p["column_tiles"], p["rounds"]) == (bda.KERNEL_LEAN, 128, 256, 1)
    p = _plan(64, [1], [0], bda.BDA_F32, d_c=64, d_h=32)                # config 1: float32
    assert p["kernel"] == bda.KERNEL_GENERAL
    assert _plan(0, [16, 16], [0, 0], bda.BDA_F16)["kernel"] == bda.KERNEL_NONE


def test_launch_plan_tile_choice_by_rounds():
    """64-token tiles where one round of them covers the launch; 128-token tiles where they need fewer
    than 1/0.56 times the rounds of 256-token tiles; dies take single tiles where whole super-tiles
    would need more rounds."""
    want = {600: (64, 1, 1), 1024: (64, 1, 0), 1536: (128, 1, 1), 2048: (128, 1, 0), 2560: (256, 1, 1),
            3072: (256, 1, 1), 4096: (256, 1, 0), 5120: (128, 3, 0), 8192: (256, 2, 0)}
    for T, (tokens, rounds, by_tile) in want.items():
        p = _plan(T, [16, 16], [0, 0], bda.BDA_F16)
        assert p["kernel"] == bda.KERNEL_LEAN, T
        assert (p["tile_tokens"], p["rounds"], p["tile_by_tile"]) == (tokens, rounds, by_tile), (T, p)
        tiles = p["token_tiles"] * p["column_tiles"]
        per_die = p["workgroups"] // 8
        assert 8 * per_die * p["rounds"] >= tiles                      # every tile has a slot
    p = _plan(1536, [16, 16], [0, 0], bda.BDA_F16)
    assert (p["token_tiles"], p["column_tiles"], p["workgroups"]) == (12, 16, 192)   # 24 tiles per die, one round


def test_launch_plan_preconditions_of_the_lean_kernel():
    lean = bda.KERNEL_LEAN
    assert _plan(4096, [16, 16], [208, 16], bda.BDA_F16)["kernel"] == lean        # windows off the 64 grid
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16, out_dtype=bda.BDA_F32)["kernel"] == lean
    assert _plan(4096, [2, 4, 2], [0, 64, 384], bda.BDA_BF16)["kernel"] == lean   # three groups
    # contraction not a multiple of 64 -> general streaming kernel (tile count >= 96), or register-staged
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16, d_c=520)["kernel"] == bda.KERNEL_STREAM
    assert _plan(512, [16, 16], [0, 0], bda.BDA_F16, d_c=520)["kernel"] == bda.KERNEL_MFMA
    # a group narrower than a 256-column tile
    p = _plan(4096, [1], [0], bda.BDA_F16)
    assert (p["kernel"], p["tile_tokens"], p["tile_columns"]) == (bda.KERNEL_MFMA, 128, 128)
    # window start not a multiple of 8, row pitch not a multiple of 8, head width not a multiple of 32
    assert _plan(4096, [16, 16], [4, 0], bda.BDA_F16)["kernel"] == bda.KERNEL_GENERAL
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16, ldc=516)["kernel"] == bda.KERNEL_GENERAL
    assert _plan(1100, [4], [0], bda.BDA_F16, d_c=96, d_h=24)["kernel"] == bda.KERNEL_GENERAL
    assert _plan(300, [4], [0], bda.BDA_F16, d_c=96, d_h=24)["kernel"] == bda.KERNEL_DECODE   # (few tokens: head width % 8 is enough)
    # the tile policy hook
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16, tile_policy=1)["kernel"] == bda.KERNEL_MFMA
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16, tile_policy=3)["kernel"] == bda.KERNEL_STREAM
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16, tile_policy=4)["tile_tokens"] == 128
    p = _plan(4096, [16, 16], [0, 0], bda.BDA_F16, tile_policy=7)
    assert (p["kernel"], p["tile_tokens"], p["rounds"], p["lds_bytes"]) == (bda.KERNEL_LEAN, 64, 4, 112 * 1024)
    p = _plan(256, [128], [0], bda.BDA_BF16)                                 # V3 k_proj, 256 tokens: one round of 64-token tiles
    assert (p["kernel"], p["tile_tokens"], p["workgroups"], p["rounds"]) == (bda.KERNEL_LEAN, 64, 256, 1)
    duo = _plan(8192, [128, 128], [0, 0], bda.BDA_BF16, tile_policy=6)       # two 4-wave workgroups per compute unit
    assert (duo["kernel"], duo["tile_tokens"], duo["workgroups"], duo["threads"], duo["rounds"]) == (bda.KERNEL_DUO, 128, 512, 256, 16)
    assert (duo["super_m"], duo["super_n"]) == (1, 8)                          # eight column ranges: one die keeps 16 column tiles of weights
    assert _plan(300, [4], [64], bda.BDA_F16, d_c=448, d_h=192, tile_policy=6) == _plan(300, [4], [64], bda.BDA_F16, d_c=448, d_h=192)
    assert _plan(4096, [16, 16], [0, 0], bda.BDA_F16)["kernel"] == lean          # and nothing of it outlives the call
    with pytest.raises(bda.BdaError):
        _plan(4096, [16, 16], [0, 400], bda.BDA_F16)                    # window outside the latent
