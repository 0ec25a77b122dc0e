"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle, element by element
on the same seeded inputs (sizes the oracle finishes in seconds, spanning several tiles and ragged
tails), and on sampled token rows at the full benchmark sizes."""
import numpy as np
import pytest

import bda_workloads as wl
import oracle
from helpers import assert_parity, lowrank_h_rounding_allowance, parity_error

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import gpu_harness as gh          # noqa: E402
import paper_2510_01718_amd as bda  # noqa: E402


def _prepare_stored(W, d_c, H, d_h, offs, dtype):
    """Oracle-side preparation per group, rounded to the storage dtype (the same C feeds both)."""
    Cs, col = [], 0
    for g, Hg in enumerate(H):
        Wg = W[:, col:col + Hg * d_h]
        C, _, off, _ = oracle.prepare(Wg, d_c, Hg, d_h, mode=oracle.EXPLICIT, explicit_offset=offs[g])
        Cs.append(C)
        col += Hg * d_h
    C_stored, C64 = wl.to_storage(np.hstack(Cs), dtype)
    return C_stored, C64


def _run_kv_case(w, offs, out_dtype=None, policy=0, **ld):
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, offs, w.dtype)
    ref = oracle.kv_project(w.c, C64, w.d_h, w.H, offs)
    got, _ = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, w.dtype, out_dtype, policy=policy, **ld)
    od = w.dtype if out_dtype is None else out_dtype
    return assert_parity(got, ref, w.d_h, w.dtype, od, f"{w.name} offs={offs} policy={policy}")


# ------------------------------------------------------------------------------------------- configs
def test_config1_tiny_fp32():
    w = wl.kv_workload("tiny")
    rel = _run_kv_case(w, [0])
    assert rel < 1e-5


@pytest.mark.parametrize("T", [1, 8, 32, 64, 65, 128])
def test_config3_decode_shapes(T):
    w = wl.kv_workload("decode", T=T)
    _run_kv_case(w, [0, 0])


@pytest.mark.parametrize("T", [1, 8, 32, 33, 64])
def test_config3_decode_shapes_wide_slices(T):
    # policy 5: the 128-column small-T kernel, which the library picks by itself only for outputs
    # wider than about 20 k columns
    w = wl.kv_workload("decode", T=T)
    _run_kv_case(w, [0, 0], policy=5)


@pytest.mark.parametrize("T", [65, 100, 128])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, None), (wl.BF16, wl.F32)])
def test_decode_64_column_slices(T, dtype, out_dtype):
    """65 .. 128 tokens through the 64-column variant of the wide-slice kernel (policy 5; automatic
    where 32-column slices would outnumber the compute units): windows off the 64 grid, a group that
    ends inside a slice, the contraction at the limit 384 and a short one."""
    w = wl.custom_kv_workload("dec64_a", T=T, d_c=512, d_h=128, H=[3, 2], std=0.02, rms_norm=True, dtype=dtype, seed=60 + T)
    _run_kv_case(w, [72, 384], out_dtype=out_dtype, policy=5)
    w = wl.custom_kv_workload("dec64_b", T=T, d_c=96, d_h=40, H=[1, 2], std=0.1, rms_norm=True, dtype=dtype, seed=61 + T)
    _run_kv_case(w, [56, 0], out_dtype=out_dtype, policy=5)
    w = wl.custom_kv_workload("dec64_c", T=T, d_c=440, d_h=56, H=[5, 1], std=0.05, rms_norm=True, dtype=dtype, seed=62 + T)
    _run_kv_case(w, [0, 384], out_dtype=out_dtype, policy=5)
    if dtype == wl.BF16 and out_dtype is None:           # automatic choice: 72 heads = 9216 columns = 288 / 144 slices
        w = wl.custom_kv_workload("dec64_auto", T=T, d_c=512, d_h=128, H=[40, 32], std=0.02, rms_norm=True, dtype=dtype, seed=63 + T)
        p = bda.bda_kv_project_plan(T, 512, 128, [40, 32], [0, 200], dtype)
        assert (p["kernel"], p["tile_tokens"], p["tile_columns"], p["workgroups"]) == (bda.KERNEL_DECODE, 128, 64, 144)
        _run_kv_case(w, [0, 200])


@pytest.mark.parametrize("T", [129, 200, 256, 300, 700])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, wl.F32)])
def test_small_T_kernels_with_token_tiles(T, dtype, out_dtype):
    """More than 128 tokens through the small-T kernels: token tiles of 128 (the last one ragged) while
    slices x token tiles <= 256.  640 columns: 32-column slices (20 x 2 .. 6 token tiles); 8192
    columns at up to 256 tokens: 64-column slices (128 x 2)."""
    w = wl.custom_kv_workload("tiles32", T=T, d_c=512, d_h=128, H=[3, 2], std=0.02, rms_norm=True, dtype=dtype, seed=70 + T)
    p = bda.bda_kv_project_plan(T, 512, 128, [3, 2], [72, 384], dtype, out_dtype=out_dtype)
    assert (p["kernel"], p["tile_columns"], p["token_tiles"]) == (bda.KERNEL_DECODE, 32, (T + 127) // 128)
    _run_kv_case(w, [72, 384], out_dtype=out_dtype)
    if T <= 256:
        # (group widths off the 256-column grid; where the lean kernel applies, one round of its 64-token tiles is taken instead)
        w = wl.custom_kv_workload("tiles64", T=T, d_c=512, d_h=128, H=[33, 31], std=0.02, rms_norm=True, dtype=dtype, seed=71 + T)
        p = bda.bda_kv_project_plan(T, 512, 128, [33, 31], [0, 200], dtype, out_dtype=out_dtype)
        assert (p["kernel"], p["tile_columns"], p["token_tiles"], p["workgroups"]) == (bda.KERNEL_DECODE, 64, 2, 256)
        _run_kv_case(w, [0, 200], out_dtype=out_dtype)
        w = wl.custom_kv_workload("tiles64", T=T, d_c=512, d_h=128, H=[34, 30], std=0.02, rms_norm=True, dtype=dtype, seed=71 + T)
        p = bda.bda_kv_project_plan(T, 512, 128, [34, 30], [0, 200], dtype, out_dtype=out_dtype)
        assert (p["kernel"], p["tile_tokens"], p["rounds"]) == (bda.KERNEL_LEAN, 64, 1)
        _run_kv_case(w, [0, 200], out_dtype=out_dtype)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_small_T_kernels_random_shapes(seed):
    """Seeded random small problems (1 .. 500 tokens, head widths 8 .. 128, contraction 8 .. 384, one to
    three groups with windows anywhere on the multiples of 8, padded row pitches) through the
    automatic choice and through policy 5, against the oracle on the same stored numbers; columns
    past N stay untouched."""
    rng = np.random.default_rng(1000 + seed)
    for case in range(40):
        d_h = int(rng.choice([8, 16, 24, 32, 40, 56, 64, 96, 128]))
        K = 8 * int(rng.integers(1, 49))
        d_c = K + d_h
        G = int(rng.integers(1, 4))
        H = [int(rng.integers(1, 6)) for _ in range(G)]
        offs = [8 * int(rng.integers(0, K // 8 + 1)) for _ in range(G)]
        T = int(rng.choice([1, 2, 7, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 200, 256, 257, 300, 500]))
        N = sum(H) * d_h
        dtype = wl.F16 if rng.integers(0, 2) else wl.BF16
        ldc, ldC, ld_out = (v + 8 * int(rng.integers(0, 3)) for v in (d_c, N, N))
        c_stored, c64 = wl.to_storage(rng.standard_normal((T, d_c)), dtype)
        C_stored, C64 = wl.to_storage(rng.standard_normal((K, N)) * 0.2, dtype)
        ref = oracle.kv_project(c64, C64, d_h, H, offs)
        for policy in (0, 5):
            what = f"seed {seed} case {case} policy {policy}: T={T} d_c={d_c} d_h={d_h} H={H} offs={offs} ld=({ldc},{ldC},{ld_out})"
            got, raw = gh.kv_project(c_stored, C_stored, d_c, d_h, H, offs, dtype, ldc=ldc, ldC=ldC, ld_out=ld_out, fill=-7.0,
                                     policy=policy)
            assert_parity(got, ref, d_h, dtype, dtype, what)
            if ld_out > N:
                pad = raw[:, N:].cpu().numpy()
                assert np.all(pad == (np.float16(-7.0) if dtype == wl.F16 else -7)), what + ": columns beyond N were written"


@pytest.mark.parametrize("seed", [1, 2])
def test_tile_kernels_random_shapes(seed):
    """Seeded random mid-size problems (129 .. 2049 tokens, head widths 32 .. 256, contraction on and off
    the multiples of 64, groups that do and do not fill 256-column tiles, windows anywhere on the
    multiples of 8, padded row pitches) through every tile policy, against the oracle."""
    rng = np.random.default_rng(2000 + seed)
    for case in range(12):
        d_h = int(rng.choice([32, 64, 128, 192, 256]))
        K = 64 * int(rng.integers(1, 9)) if rng.integers(0, 4) else 8 * int(rng.integers(4, 60))
        d_c = K + d_h
        G = int(rng.integers(1, 4))
        mult = max(1, 256 // d_h)
        H = [int(rng.integers(1, 5)) * (mult if rng.integers(0, 3) else 1) for _ in range(G)]
        offs = [8 * int(rng.integers(0, K // 8 + 1)) for _ in range(G)]
        T = int(rng.choice([129, 255, 256, 300, 511, 640, 700, 1024, 1300, 2049]))
        N = sum(H) * d_h
        dtype = wl.F16 if rng.integers(0, 2) else wl.BF16
        ldc, ldC, ld_out = (v + 8 * int(rng.integers(0, 2)) for v in (d_c, N, N))
        c_stored, c64 = wl.to_storage(rng.standard_normal((T, d_c)), dtype)
        C_stored, C64 = wl.to_storage(rng.standard_normal((K, N)) * 0.2, dtype)
        ref = oracle.kv_project(c64, C64, d_h, H, offs)
        for policy in (0, 1, 2, 3, 4, 5, 6, 7):
            what = f"seed {seed} case {case} policy {policy}: T={T} d_c={d_c} d_h={d_h} H={H} offs={offs} ld=({ldc},{ldC},{ld_out})"
            got, _ = gh.kv_project(c_stored, C_stored, d_c, d_h, H, offs, dtype, ldc=ldc, ldC=ldC, ld_out=ld_out, fill=-7.0,
                                   policy=policy)
            assert_parity(got, ref, d_h, dtype, dtype, what)


@pytest.mark.parametrize("T", [1, 31, 64])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, wl.F32)])
def test_decode_wide_slices_automatic(T, dtype, out_dtype):
    # 160 slices of 128 columns (two groups, different windows off the 64 grid): the width from which
    # the wide-slice kernel is the automatic choice
    w = wl.custom_kv_workload("dec_wide", T=T, d_c=512, d_h=128, H=[100, 60], std=0.02, rms_norm=True, dtype=dtype, seed=50 + T)
    p = bda.bda_kv_project_plan(T, 512, 128, [100, 60], [72, 384], dtype, out_dtype=out_dtype)
    assert (p["kernel"], p["tile_columns"], p["workgroups"]) == (bda.KERNEL_DECODE, 128, 160)
    _run_kv_case(w, [72, 384], out_dtype=out_dtype)


@pytest.mark.parametrize("T", [1, 7, 33, 64, 65, 97, 128])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, None), (wl.BF16, wl.F32)])
def test_decode_kernel_groups_and_offsets(T, dtype, out_dtype):
    # the small-T kernel: two groups with different windows, a group that ends inside a 32-column
    # slice (40 columns), head width 8 ... and the V2-Lite head shape
    w = wl.custom_kv_workload("dec_a", T=T, d_c=512, d_h=128, H=[3, 2], std=0.02, rms_norm=True, dtype=dtype, seed=40 + T)
    _run_kv_case(w, [64, 384], out_dtype=out_dtype)
    w = wl.custom_kv_workload("dec_b", T=T, d_c=96, d_h=40, H=[1, 2], std=0.1, rms_norm=True, dtype=dtype, seed=41 + T)
    _run_kv_case(w, [56, 0], out_dtype=out_dtype)
    w = wl.custom_kv_workload("dec_c", T=T, d_c=1152, d_h=64, H=[5], std=0.02, rms_norm=True, dtype=dtype, seed=42 + T)
    _run_kv_case(w, [512], out_dtype=out_dtype)
    if T <= 64:                                          # the same through the 128-column kernel (dec_c: K > 384, falls back)
        w = wl.custom_kv_workload("dec_a", T=T, d_c=512, d_h=128, H=[3, 2], std=0.02, rms_norm=True, dtype=dtype, seed=40 + T)
        _run_kv_case(w, [64, 384], out_dtype=out_dtype, policy=5)
        w = wl.custom_kv_workload("dec_b", T=T, d_c=96, d_h=40, H=[1, 2], std=0.1, rms_norm=True, dtype=dtype, seed=41 + T)
        _run_kv_case(w, [56, 0], out_dtype=out_dtype, policy=5)
        w = wl.custom_kv_workload("dec_c", T=T, d_c=1152, d_h=64, H=[5], std=0.02, rms_norm=True, dtype=dtype, seed=42 + T)
        _run_kv_case(w, [512], out_dtype=out_dtype, policy=5)
        w = wl.custom_kv_workload("dec_d", T=T, d_c=440, d_h=56, H=[5, 1], std=0.05, rms_norm=True, dtype=dtype, seed=43 + T)
        _run_kv_case(w, [0, 384], out_dtype=out_dtype, policy=5)   # K = 384 at the limit, ragged last slices (280 and 56 columns)


@pytest.mark.parametrize("policy", [1, 2])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("offs", [[0, 0], [384, 384], [0, 384], [64, 200]])
def test_kv_medium_ragged(policy, dtype, offs):
    # 300 tokens (ragged against 128- and 256-row tiles), 3 + 2 heads (640 columns: the second
    # group ends inside a tile), V2-Lite head shape
    w = wl.custom_kv_workload("medium", T=300, d_c=512, d_h=128, H=[3, 2], std=0.02, rms_norm=True,
                              dtype=dtype, seed=11)
    _run_kv_case(w, offs, policy=policy)


@pytest.mark.parametrize("policy", [2, 3, 4, 6, 7])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, None), (wl.F16, wl.F32)])
@pytest.mark.parametrize("offs", [[0, 0], [384, 384], [64, 192], [16, 208], [8, 376], [120, 72]])
def test_kv_lean_and_general_streaming_kernels(policy, dtype, out_dtype, offs):
    """Full 256-column tiles, windows on and off the multiples of 64 (the stage that holds a window's
    start then shifts part of its lanes): policy 2 runs the lean streaming kernel,
    policy 3 forces the general one on the same launch, policy 4 the lean kernel with 128-token tiles,
    policy 6 the kernel with two 4-wave workgroups per compute unit (128 x 256 tiles, stages of 32);
    700 tokens = three (six) token tiles per workgroup column, the last one ragged."""
    w = wl.custom_kv_workload("lean", T=700, d_c=512, d_h=128, H=[4, 2], std=0.02, rms_norm=True,
                              dtype=dtype, seed=12)
    _run_kv_case(w, offs, out_dtype=out_dtype, policy=policy)


@pytest.mark.parametrize("policy", [2, 4, 6, 7])
def test_kv_lean_three_groups(policy):
    """Three groups with different windows through the lean kernel (group look-up beyond the two
    register-held groups)."""
    w = wl.custom_kv_workload("lean3", T=300, d_c=512, d_h=128, H=[2, 4, 2], std=0.02, rms_norm=True,
                              dtype=wl.BF16, seed=21)
    _run_kv_case(w, [0, 64, 384], policy=policy)


@pytest.mark.parametrize("out_dtype", [None, wl.F32])
@pytest.mark.parametrize("d_c,d_h,H,offs", [(512, 128, [10, 6], [64, 200]),     # seven stages per tile
                                            (256, 64, [20, 12], [0, 192]),      # four
                                            (256, 128, [10, 6], [0, 128])])     # three: the fewest the lean kernel takes
def test_kv_lean_64_token_tiles_over_two_rounds(d_c, d_h, H, offs, out_dtype):
    """Tile policy 7 on 33 x 8 tiles of 64 x 256: two rounds, the second nearly empty, ragged last token tile
    (by itself the library takes 64-token tiles only where one round covers the launch)."""
    w = wl.custom_kv_workload("lean64", T=2100, d_c=d_c, d_h=d_h, H=H, std=0.02, rms_norm=True, dtype=wl.BF16, seed=24)
    p = bda.bda_kv_project_plan(w.T, d_c, d_h, H, offs, w.dtype, out_dtype=out_dtype or w.dtype, tile_policy=7)
    assert (p["kernel"], p["tile_tokens"], p["rounds"]) == (bda.KERNEL_LEAN, 64, 2)
    _run_kv_case(w, offs, out_dtype=out_dtype, policy=7)


def test_kv_lean_tile_by_tile_order_two_rounds():
    """17 x 25 tiles of 128 x 256: whole super-tiles would need three rounds, so the tiles are dealt
    out one by one (54 per die, two rounds, the last die's run shorter); ragged last token tile."""
    w = wl.custom_kv_workload("linear2", T=2100, d_c=512, d_h=128, H=[26, 24], std=0.02, rms_norm=True,
                              dtype=wl.F16, seed=22)
    _run_kv_case(w, [0, 384], policy=4)


@pytest.mark.parametrize("policy", [2, 3, 4, 6, 7])
@pytest.mark.parametrize("d_c,d_h,H,offs", [(256, 64, [8, 4], [0, 192]),        # window narrower than an identity stage
                                            (448, 192, [4], [64]),              # one and a half identity stages
                                            (512, 256, [2, 1], [256, 0]),       # window = tile width: two stages
                                            (1024, 512, [1, 1], [512, 128])])   # tile takes its own 256 columns of the window
def test_kv_lean_head_widths(policy, d_c, d_h, H, offs):
    """Head widths other than 128 through the streaming kernels: the identity slice of a tile is
    64 ... 256 window columns, taken in stages of 128 (lean) or 64 (general)."""
    w = wl.custom_kv_workload("widths", T=300, d_c=d_c, d_h=d_h, H=H, std=0.02, rms_norm=True,
                              dtype=wl.F16, seed=31)
    _run_kv_case(w, offs, policy=policy)


@pytest.mark.parametrize("T,tile", [(600, 64), (1024, 64), (1300, 128), (1536, 128)])
def test_kv_lean_automatic_tile_choice(T, tile):
    """Automatic policy on the V2-Lite shape at token counts that select 64-token tiles (one round of
    them covers the launch) and 128-token tiles (tile-by-tile order at 1536: 12 x 16 tiles)."""
    w = wl.custom_kv_workload("auto", T=T, d_c=512, d_h=128, H=[16, 16], std=0.02, rms_norm=True,
                              dtype=wl.F16, seed=23)
    p = bda.bda_kv_project_plan(T, 512, 128, [16, 16], [0, 0], wl.F16)
    assert (p["kernel"], p["tile_tokens"]) == (bda.KERNEL_LEAN, tile)
    _run_kv_case(w, [0, 0])
    _run_kv_case(w, [64, 200])                               # windows inside the latent, one off the 64-column stage grid


@pytest.mark.parametrize("policy", [2, 3, 4, 6, 7])
def test_dense_many_stages_streaming(policy):
    """A long contraction (K = 1024: 16 stages per tile, no identity slice) through both streaming kernels."""
    rng = np.random.default_rng(13)
    T, K, N = 520, 1024, 512
    x = rng.standard_normal((T, K))
    W = rng.standard_normal((K, N)) * 0.05
    xs, x64 = wl.to_storage(x, wl.F16)
    Ws, W64 = wl.to_storage(W, wl.F16)
    x_d, W_d = gh.to_device(xs, wl.F16), gh.to_device(Ws, wl.F16)
    out_d = gh.new_out(T, N, wl.F16)
    bda.bda_dense_project_ex(x_d, K, T, K, W_d, N, N, out_d, N, wl.F16, stream=gh.stream(), tile_policy=policy)
    torch.cuda.synchronize()
    assert_parity(gh.to_host64(out_d, wl.F16), oracle.dense_project(x64, W64), N, wl.F16, wl.F16, "dense K=1024")


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_kv_fp32_output_meets_plain_tolerance(dtype):
    w = wl.custom_kv_workload("medium32", T=200, d_c=512, d_h=128, H=[2, 2], std=0.02, rms_norm=True,
                              dtype=dtype, seed=12)
    _run_kv_case(w, [0, 384], out_dtype=wl.F32, policy=1)
    _run_kv_case(w, [0, 384], out_dtype=wl.F32, policy=2)


@pytest.mark.parametrize("d_h,d_c,H", [(64, 256, [3, 1]), (32, 96, [5]), (96, 288, [2, 2]), (256, 512, [1, 2])])
def test_kv_other_head_shapes(d_h, d_c, H):
    w = wl.custom_kv_workload("shapes", T=150, d_c=d_c, d_h=d_h, H=H, std=0.05, rms_norm=True,
                              dtype=wl.F16, seed=13)
    last = d_c - d_h
    offs = [0, last][:len(H)] if len(H) > 1 else [32 if last >= 32 else 0]
    for policy in (1, 2):
        _run_kv_case(w, offs, policy=policy)


def test_kv_strided_buffers_and_untouched_padding():
    w = wl.custom_kv_workload("strided", T=130, d_c=512, d_h=128, H=[2, 1], std=0.02, rms_norm=True,
                              dtype=wl.F16, seed=14)
    offs = [0, 384]
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, offs, w.dtype)
    ref = oracle.kv_project(w.c, C64, w.d_h, w.H, offs)
    N = w.N
    for policy in (1, 2):
        got, raw = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, w.dtype,
                                 ldc=w.d_c + 64, ldC=N + 8, ld_out=N + 24, fill=-7.0, policy=policy)
        assert_parity(got, ref, w.d_h, w.dtype, w.dtype, "strided")
        pad = raw[:, N:].cpu().numpy()
        assert np.all(pad == np.float16(-7.0)), "columns beyond N were written"


@pytest.mark.parametrize("T", [8, 50, 100])
@pytest.mark.parametrize("policy", [0, 5])
def test_small_T_kernels_strided_buffers_and_exact_copy(T, policy):
    """The small-T kernels (32-column slices at policy 0, 128- or 64-column slices at policy 5) with
    row pitches larger than the rows: results as with dense buffers, padding untouched; and with
    C = 0 the output is the basis slice bit for bit (float32 identity add, one rounding)."""
    w = wl.custom_kv_workload("strided_small", T=T, d_c=512, d_h=128, H=[2, 1], std=0.02, rms_norm=True,
                              dtype=wl.F16, seed=18 + T)
    offs = [8, 384]
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, offs, w.dtype)
    ref = oracle.kv_project(w.c, C64, w.d_h, w.H, offs)
    N = w.N
    assert bda.bda_kv_project_plan(T, 512, 128, w.H, offs, w.dtype, ldc=w.d_c + 64, ldC=N + 8, ld_out=N + 24,
                                   tile_policy=policy)["kernel"] == bda.KERNEL_DECODE
    got, raw = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, w.dtype,
                             ldc=w.d_c + 64, ldC=N + 8, ld_out=N + 24, fill=-7.0, policy=policy)
    zero_C, _ = wl.to_storage(np.zeros((384, N)), w.dtype)
    copy, _ = gh.kv_project(w.c_stored, zero_C, w.d_c, w.d_h, w.H, offs, w.dtype, policy=policy)
    assert_parity(got, ref, w.d_h, w.dtype, w.dtype, "strided small T")
    pad = raw[:, N:].cpu().numpy()
    assert np.all(pad == np.float16(-7.0)), "columns beyond N were written"
    for h in range(3):
        off = offs[0] if h < 2 else offs[1]
        assert np.array_equal(copy[:, h * 128:(h + 1) * 128], w.c[:, off:off + 128]), (h, policy)


def test_kv_general_kernel_for_unaligned_shapes():
    # d_h = 20 and d_c = 52 satisfy none of the MFMA path's alignment rules
    w = wl.custom_kv_workload("unaligned", T=77, d_c=52, d_h=20, H=[2, 3], std=0.1, rms_norm=False,
                              dtype=wl.F16, seed=15)
    _run_kv_case(w, [3, 32])
    w = wl.custom_kv_workload("unaligned32", T=77, d_c=52, d_h=20, H=[2, 3], std=0.1, rms_norm=False,
                              dtype=wl.F32, seed=15)
    _run_kv_case(w, [3, 32])
    w = wl.custom_kv_workload("unaligned_bf", T=33, d_c=52, d_h=20, H=[1], std=0.1, rms_norm=False,
                              dtype=wl.BF16, seed=16)
    _run_kv_case(w, [32], out_dtype=wl.F32)


# ------------------------------------------------------------------------------------ exact properties
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16, wl.F32])
def test_zero_C_copies_basis_slice_bit_exactly(dtype):
    w = wl.custom_kv_workload("copy", T=200, d_c=512, d_h=128, H=[2, 2], std=0.02, rms_norm=True,
                              dtype=dtype, seed=17)
    C_stored, _ = wl.to_storage(np.zeros((384, w.N)), dtype)
    for policy, offs in ((1, [64, 384]), (2, [64, 384]), (4, [64, 384]), (2, [40, 376]), (4, [8, 200])):
        got, _ = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, dtype, policy=policy)
        for h in range(4):
            off = offs[0] if h < 2 else offs[1]
            assert np.array_equal(got[:, h * 128:(h + 1) * 128], w.c[:, off:off + 128]), (dtype, h, policy)


def test_zero_basis_slice_is_pure_gemm():
    w = wl.custom_kv_workload("puregemm", T=140, d_c=512, d_h=128, H=[3], std=0.02, rms_norm=True,
                              dtype=wl.F16, seed=18)
    c = w.c.copy()
    c[:, 128:256] = 0.0
    c_stored, c64 = wl.to_storage(c, wl.F16)
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, [128], wl.F16)
    ref = oracle.kv_project(c64, C64, 128, [3], [128])
    got, _ = gh.kv_project(c_stored, C_stored, 512, 128, [3], [128], wl.F16)
    assert_parity(got, ref, 128, wl.F16, wl.F16, "pure gemm")


def test_deterministic_across_runs():
    w = wl.custom_kv_workload("det", T=513, d_c=512, d_h=128, H=[4, 4], std=0.02, rms_norm=True,
                              dtype=wl.BF16, seed=19)
    C_stored, _ = _prepare_stored(w.W, w.d_c, w.H, w.d_h, [0, 384], wl.BF16)
    outs = [gh.kv_project(w.c_stored, C_stored, 512, 128, [4, 4], [0, 384], wl.BF16)[0] for _ in range(3)]
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_empty_and_error_paths():
    c = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    C = torch.zeros((48, 32), dtype=torch.float16, device="cuda")
    out = torch.full((4, 32), 3.0, dtype=torch.float16, device="cuda")
    bda.bda_kv_project(c, 64, 0, 64, 16, [2], [0], C, 32, out, 32, bda.BDA_F16)   # T = 0
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)
    with pytest.raises(bda.BdaError) as e:
        bda.bda_kv_project(c, 64, 4, 64, 16, [2], [49], C, 32, out, 32, bda.BDA_F16)
    assert e.value.status == -1
    with pytest.raises(bda.BdaError):
        bda.bda_kv_project(c, 64, 4, 64, 16, [2], [0], C, 32, c, 64, bda.BDA_F16)  # out aliases c
    with pytest.raises(bda.BdaError) as e:
        bda.bda_kv_project(c, 64, 4, 64, 16, [2], [0], C, 32, out, 32, bda.BDA_F16, bda.BDA_BF16)
    assert e.value.status == -3


# ------------------------------------------------------------------------------------ dense and low-rank
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16, wl.F32])
@pytest.mark.parametrize("policy", [1, 2])
def test_dense_project(dtype, policy):
    w = wl.custom_kv_workload("dense", T=270, d_c=512, d_h=128, H=[5], std=0.02, rms_norm=True,
                              dtype=dtype, seed=20)
    W_stored, W64 = wl.to_storage(w.W, dtype)
    ref = oracle.dense_project(w.c, W64)
    c_d, W_d = gh.to_device(w.c_stored, dtype), gh.to_device(W_stored, dtype)
    out_d = gh.new_out(w.T, w.N, dtype)
    bda.bda_dense_project_ex(c_d, 512, w.T, 512, W_d, w.N, w.N, out_d, w.N, dtype, stream=gh.stream(), tile_policy=policy)
    torch.cuda.synchronize()
    assert_parity(gh.to_host64(out_d, dtype), ref, 128, dtype, dtype, "dense")


@pytest.mark.parametrize("T", [1, 40, 64, 100, 300])
@pytest.mark.parametrize("policy", [0, 5])
def test_dense_project_few_tokens(T, policy):
    """The small-T kernels without an identity slice: 32-column slices (policy 0; four token blocks
    at T = 100, three token tiles at T = 300) and 128- / 64-column slices (policy 5), contraction 320."""
    dtype = wl.BF16
    w = wl.custom_kv_workload("dense_few", T=T, d_c=320, d_h=64, H=[9], std=0.05, rms_norm=True, dtype=dtype, seed=23 + T)
    W_stored, W64 = wl.to_storage(w.W, dtype)
    ref = oracle.dense_project(w.c, W64)
    c_d, W_d = gh.to_device(w.c_stored, dtype), gh.to_device(W_stored, dtype)
    out_d = gh.new_out(w.T, w.N, dtype)
    p = bda.bda_dense_project_plan(T, 320, w.N, dtype)
    assert p["kernel"] == bda.KERNEL_DECODE
    if policy == 5 and T <= 64:
        assert bda.bda_dense_project_plan(T, 320, w.N, dtype, tile_policy=policy)["tile_columns"] == 128
    bda.bda_dense_project_ex(c_d, 320, w.T, 320, W_d, w.N, w.N, out_d, w.N, dtype, stream=gh.stream(), tile_policy=policy)
    torch.cuda.synchronize()
    assert_parity(gh.to_host64(out_d, dtype), ref, 64, dtype, dtype, "dense few tokens")


@pytest.mark.parametrize("last", [False, True])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_lowrank_linear_small(last, dtype):
    lw = wl.lowrank_workload(T=200, d_in=256, r=64, d_out=320, dtype=dtype, seed=21)
    Up, C, off, _ = oracle.prepare_lowrank(lw.U, lw.V, mode=oracle.LAST if last else oracle.FIRST)
    Up_s, Up64 = wl.to_storage(Up, dtype)
    C_s, C64 = wl.to_storage(C, dtype)
    ref = oracle.lowrank_linear(lw.x, Up64, C64, off)
    x_d, U_d, C_d = gh.to_device(lw.x_stored, dtype), gh.to_device(Up_s, dtype), gh.to_device(C_s, dtype)
    out_d = gh.new_out(lw.T, lw.d_out + 8, dtype, fill=0)
    bda.bda_lowrank_linear(x_d, lw.d_in, lw.T, lw.d_in, lw.r, lw.d_out, off, U_d, C_d, out_d,
                           lw.d_out + 8, dtype, gh.stream())
    torch.cuda.synchronize()
    got = gh.to_host64(out_d, dtype, lw.d_out)
    # the h block is held to the plain tolerance; the h C block gets the a-priori allowance for
    # the one rounding of h that the library performs and the oracle does not
    extra = lowrank_h_rounding_allowance(ref, C64, lw.r, off, dtype)
    assert_parity(got, ref, lw.d_out, dtype, dtype, "lowrank", extra)
    assert_parity(got[:, off:off + lw.r], ref[:, off:off + lw.r], lw.r, dtype, dtype, "lowrank h block")
    # the second product alone, from the h the GPU stored, at the plain tolerance
    rest = np.concatenate([np.arange(0, off), np.arange(off + lw.r, lw.d_out)])
    ref2 = oracle.dense_project(got[:, off:off + lw.r], C64)
    assert_parity(got[:, rest], ref2, lw.d_out - lw.r, dtype, dtype, "lowrank h C from the stored h")


# ------------------------------------------------------------------------------------ full benchmark sizes
NAN_FILL = {wl.F16: float("nan"), wl.F32: float("nan"), wl.BF16: 0x7FC0}     # bf16 buffers are int16 bit patterns


def _sample_rows(T, n_random, seed, block=32):
    """First and last rows, the rows around the first 256-row tile border, one row inside every
    `block`-row MFMA block of every token tile (its position inside the block varies), and
    `n_random` random rows."""
    rng = np.random.default_rng(seed)
    rows = set(range(0, min(T, 4))) | set(range(max(T - 4, 0), T))
    rows |= {255, 256, 257} & set(range(T))
    rows |= {min(T - 1, b * block + (7 * b + 3) % block) for b in range((T + block - 1) // block)}
    rows |= set(int(r) for r in rng.integers(0, T, n_random))
    return np.array(sorted(rows), dtype=np.int64)


def _whole_output_check(got, c64, C64, d_h, H, offs, in_dtype, out_dtype, what, chunk=1024):
    """Every element of a full-size output against a float64 numpy product of the same stored inputs
    (tile(c[:, B]) + c[:, Bbar] @ C per group, a library GEMM -- not the oracle's loops, which
    check the sampled rows), chunk by chunk; with the output pre-filled with NaN this also shows a
    tile that was skipped."""
    assert np.all(np.isfinite(got)), f"{what}: output holds NaN / inf (an unwritten or doubly damaged tile)"
    d_c = c64.shape[1]
    worst = 0.0
    for r0 in range(0, c64.shape[0], chunk):
        cc = c64[r0:r0 + chunk]
        parts, col = [], 0
        for Hg, off in zip(H, offs):
            bbar = np.concatenate([np.arange(0, off), np.arange(off + d_h, d_c)])
            w = Hg * d_h
            parts.append(np.tile(cc[:, off:off + d_h], (1, Hg)) + np.matmul(cc[:, bbar], C64[:, col:col + w]))
            col += w
        ref = np.hstack(parts)
        worst = max(worst, assert_parity(got[r0:r0 + chunk], ref, d_h, in_dtype, out_dtype, f"{what} rows {r0}.."))
    return worst


def test_full_size_config2_every_element():
    """Config 2 (V2-Lite shape, T = 4096, fp16) in the launch configuration the bench times: every
    element against the oracle's loops; the output starts as NaN."""
    w = wl.kv_workload("v2lite")
    offs = [0, 0]
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, offs, w.dtype)
    ref = oracle.kv_project(w.c, C64, w.d_h, w.H, offs)
    got, _ = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, w.dtype, fill=NAN_FILL[w.dtype])
    assert np.all(np.isfinite(got))
    rel = assert_parity(got, ref, w.d_h, w.dtype, w.dtype, "v2lite, all rows")
    print(f"config 2: max relative error {rel:.2e} over {got.size} elements")


def test_full_size_config4_sampled_rows_and_whole_output():
    """Config 4 (V3 shape, T = 8192, bf16): the oracle's loops on 256 random rows plus one row in
    every 32-row block of every token tile plus the borders (about 500 rows, all 32768 columns),
    and every element against a float64 library GEMM; the output starts as NaN.  The same kernel
    with float32 outputs (results staged through LDS in 32 x 32 blocks) is held to the plain
    tolerance on its first 512 rows, every element."""
    w = wl.kv_workload("v3")
    offs = [0, 0]
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, offs, w.dtype)
    rows = _sample_rows(w.T, 256, seed=5)
    assert len(rows) >= 256 + w.T // 32 - 40
    ref = oracle.kv_project(w.c[rows], C64, w.d_h, w.H, offs)
    got, _ = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, w.dtype, fill=NAN_FILL[w.dtype])
    rel = assert_parity(got[rows], ref, w.d_h, w.dtype, w.dtype, "v3 sampled rows")
    worst = _whole_output_check(got, w.c, C64, w.d_h, w.H, offs, w.dtype, w.dtype, "v3 whole output")
    print(f"config 4: {len(rows)} oracle rows, max relative error {rel:.2e}; whole output {worst:.2e}")
    got32, _ = gh.kv_project(w.c_stored[:512], C_stored, w.d_c, w.d_h, w.H, offs, w.dtype, out_dtype=wl.F32,
                             fill=NAN_FILL[wl.F32])
    ref32 = oracle.kv_project(w.c[:64], C64, w.d_h, w.H, offs)
    assert np.all(np.isfinite(got32))
    assert_parity(got32[:64], ref32, w.d_h, w.dtype, wl.F32, "v3 fp32 out")
    _whole_output_check(got32, w.c[:512], C64, w.d_h, w.H, offs, w.dtype, wl.F32, "v3 fp32 out, every element of 512 rows")


@pytest.mark.parametrize("out_dtype", [None, wl.F32])
def test_general_streaming_kernel_cut_tiles_over_several_rounds(out_dtype):
    """Tile policy 3 (the general streaming kernel) on 32 x 12 tiles of 256 x 256, more than one per
    workgroup, where each group's last tile is cut short by the group's end (1408 = 5.5 x 256 columns):
    after such a tile fewer result stores are in flight than after a full one, which the next tile's
    first load wait has to allow for.  Every element against a float64 library product, NaN-filled
    output; 16-bit and float32 results (both staged through LDS)."""
    w = wl.custom_kv_workload("cut_tiles", T=8192, d_c=512, d_h=128, H=[11, 11], std=0.02, rms_norm=True, dtype=wl.BF16, seed=21)
    offs = [64, 384]
    p = bda.bda_kv_project_plan(w.T, w.d_c, w.d_h, w.H, offs, w.dtype, out_dtype=out_dtype, tile_policy=3)
    assert p["kernel"] == bda.KERNEL_STREAM and p["rounds"] >= 2, p
    C_stored, C64 = _prepare_stored(w.W, w.d_c, w.H, w.d_h, offs, w.dtype)
    od = w.dtype if out_dtype is None else out_dtype
    got, _ = gh.kv_project(w.c_stored, C_stored, w.d_c, w.d_h, w.H, offs, w.dtype, out_dtype=out_dtype, fill=NAN_FILL[od], policy=3)
    _whole_output_check(got, w.c, C64, w.d_h, w.H, offs, w.dtype, od, "cut tiles, general streaming kernel")
    rows = _sample_rows(w.T, 24, seed=6)[:48]
    assert_parity(got[rows], oracle.kv_project(w.c[rows], C64, w.d_h, w.H, offs), w.d_h, w.dtype, od, "cut tiles, oracle rows")


def test_full_size_lowrank_sampled_rows_and_whole_output():
    """Config 5 (BD linear layer, T = 8192, fp16).  Three checks (Section "BD for Linear Layer"):
      1. end to end against the oracle, whose h = x U' is never rounded: the h block at the plain
         tolerance, the h C block with the derived allowance for the library's one rounding of h;
      2. the second product alone at the PLAIN tolerance: the oracle is fed the h the GPU stored
         (read back from the output), so nothing but the product h C is compared;
      3. every element of the output against float64 library GEMMs on the same stored inputs
         (same two-stage form as 2), the output starting as NaN."""
    lw = wl.lowrank_workload()
    Up, C, off, _ = oracle.prepare_lowrank(lw.U, lw.V, mode=oracle.FIRST)
    Up_s, Up64 = wl.to_storage(Up, lw.dtype)
    C_s, C64 = wl.to_storage(C, lw.dtype)
    rows = _sample_rows(lw.T, 256, seed=6, block=256)
    assert len(rows) >= 256
    x_d, U_d, C_d = gh.to_device(lw.x_stored, lw.dtype), gh.to_device(Up_s, lw.dtype), gh.to_device(C_s, lw.dtype)
    out_d = gh.new_out(lw.T, lw.d_out, lw.dtype, fill=NAN_FILL[lw.dtype])
    bda.bda_lowrank_linear(x_d, lw.d_in, lw.T, lw.d_in, lw.r, lw.d_out, off, U_d, C_d, out_d,
                           lw.d_out, lw.dtype, gh.stream())
    torch.cuda.synchronize()
    got = gh.to_host64(out_d, lw.dtype)
    assert np.all(np.isfinite(got))
    r = lw.r
    # 1. end to end
    ref = oracle.lowrank_linear(lw.x[rows], Up64, C64, off)
    extra = lowrank_h_rounding_allowance(ref, C64, r, off, lw.dtype)
    worst_e2e, _ = parity_error(got[rows], ref, lw.d_out, lw.dtype, lw.dtype, extra)
    assert worst_e2e <= 1.0, worst_e2e
    assert_parity(got[rows][:, :r], ref[:, :r], r, lw.dtype, lw.dtype, "lowrank full h block")
    # 2. second product from the GPU's own stored h, plain tolerance
    h_gpu = got[rows][:, :r]
    ref2 = oracle.dense_project(h_gpu, C64)
    rel2 = assert_parity(got[rows][:, r:], ref2, lw.d_out - r, lw.dtype, lw.dtype, "lowrank h C from the stored h")
    # 3. whole output
    worst = 0.0
    for r0 in range(0, lw.T, 1024):
        h_ref = np.matmul(lw.x[r0:r0 + 1024], Up64)
        worst = max(worst, assert_parity(got[r0:r0 + 1024, :r], h_ref, r, lw.dtype, lw.dtype, f"lowrank h rows {r0}.."))
        hc_ref = np.matmul(got[r0:r0 + 1024, :r], C64)
        worst = max(worst, assert_parity(got[r0:r0 + 1024, r:], hc_ref, lw.d_out - r, lw.dtype, lw.dtype, f"lowrank h C rows {r0}.."))
    print(f"config 5: {len(rows)} oracle rows; end-to-end worst ratio to its allowance {worst_e2e:.3f}; "
          f"h C from the stored h {rel2:.2e}; whole output {worst:.2e}")


# ------------------------------------------------------------------------------------ rows past T
@pytest.mark.parametrize("T,d_c,d_h,H,offs,dtype,policy,kernel", [
    (5, 512, 128, [2, 1], [8, 384], wl.F16, 0, "decode32"),
    (40, 512, 128, [2, 1], [8, 384], wl.BF16, 0, "decode32x2"),
    (100, 512, 128, [2, 1], [8, 384], wl.F16, 0, "decode32x4"),
    (20, 512, 128, [2, 1], [8, 384], wl.F16, 5, "decode128"),
    (100, 512, 128, [2, 1], [8, 384], wl.BF16, 5, "decode64"),
    (200, 512, 128, [3, 2], [72, 384], wl.F16, 0, "decode32 token tiles"),
    (300, 512, 128, [4, 2], [64, 192], wl.F16, 1, "mfma128"),
    (300, 512, 128, [4, 2], [64, 192], wl.BF16, 2, "lean256"),
    (300, 512, 128, [4, 2], [64, 192], wl.F16, 3, "stream256"),
    (300, 512, 128, [4, 2], [64, 192], wl.BF16, 4, "lean128"),
    (300, 512, 128, [4, 2], [64, 192], wl.F16, 7, "lean64"),
    (77, 52, 20, [2, 3], [3, 32], wl.F16, 0, "general"),
    (64, 64, 16, [2], [0], wl.F32, 0, "general fp32"),
])
def test_rows_past_T_are_not_written(T, d_c, d_h, H, offs, dtype, policy, kernel):
    """Every kernel family with 40 poisoned rows after the last token and padded row pitches: the
    result is right and neither the rows past T nor the columns past N are touched."""
    w = wl.custom_kv_workload("guard", T=T, d_c=d_c, d_h=d_h, H=H, std=0.05, rms_norm=True, dtype=dtype, seed=90 + T)
    C_stored, C64 = _prepare_stored(w.W, d_c, H, d_h, offs, dtype)
    ref = oracle.kv_project(w.c, C64, d_h, H, offs)
    N = w.N
    poison = -7.0 if dtype != wl.BF16 else -7
    got, raw = gh.kv_project(w.c_stored, C_stored, d_c, d_h, H, offs, dtype, ld_out=N + 8, fill=poison,
                             policy=policy, extra_rows=40)
    assert_parity(got, ref, d_h, dtype, dtype, kernel)
    tail = raw[T:].cpu().numpy()
    assert tail.shape[0] == 40 and np.all(tail == poison), f"{kernel}: rows past T were written"
    assert np.all(raw[:T, N:].cpu().numpy() == poison), f"{kernel}: columns past N were written"


# ------------------------------------------------------------------------------------ end to end
def test_library_prepare_then_project_scores():
    """bda_prepare (library, host) -> bda_kv_project (GPU) -> per-head scores Q'K'^T.  The GPU scores
    must equal those formed from the oracle's K' on the same stored C (the GPU path adds nothing
    beyond its own rounding), and both stay close to the dense model's Q K^T -- the deviation there
    is the storage rounding of C, which the paper measures as the fp16 reconstruction error."""
    rng = np.random.default_rng(30)
    T, d_c, H, d_h, d_q = 96, 512, 2, 128, 192
    w = wl.custom_kv_workload("e2e", T=T, d_c=d_c, d_h=d_h, H=[H], std=0.02, rms_norm=True, dtype=wl.F16, seed=30)
    Wq = rng.standard_normal((d_q, H * d_h)) * 0.02
    xq = rng.standard_normal((T, d_q))
    C, Bq, off, _ = bda.bda_prepare(w.W, d_c, H, d_h, Wq, bda.SIDE_Q, bda.BASIS_RESIDUAL_MIN, 0, bda.BDA_F16)
    _, _, off_o, _ = oracle.prepare(w.W, d_c, H, d_h, Wq, oracle.SIDE_Q, oracle.RESIDUAL_MIN, 0, oracle.F16)
    assert off == off_o
    C_stored, C64 = wl.to_storage(C, wl.F16)
    Kp, _ = gh.kv_project(w.c_stored, C_stored, d_c, d_h, [H], [off], wl.F16, out_dtype=wl.F32)
    Kp_or = oracle.kv_project(w.c, C64, d_h, [H], [off])
    Qp = xq @ Bq
    Q, K = xq @ Wq, w.c @ w.W
    for h in range(H):
        s = slice(h * d_h, (h + 1) * d_h)
        got = Qp[:, s] @ Kp[:, s].T
        ref = Qp[:, s] @ Kp_or[:, s].T
        bound = np.abs(Qp[:, s]) @ np.abs(Kp_or[:, s]).T
        assert np.max(np.abs(got - ref) / bound) <= 1e-5
        dense = Q[:, s] @ K[:, s].T
        nmse = np.sum((ref - dense) ** 2) / np.sum(dense ** 2)
        assert nmse < 1e-2, nmse     # fp16 storage of C only; exact in float64 (oracle pins)


def _gpu_dense(x64, W64, dtype, out_dtype):
    """out = x W on the GPU (bda_dense_project) from float64 arrays rounded to `dtype`."""
    xs, _ = wl.to_storage(x64, dtype)
    Ws, _ = wl.to_storage(W64, dtype)
    T, K = x64.shape
    N = W64.shape[1]
    x_d, W_d = gh.to_device(xs, dtype), gh.to_device(Ws, dtype)
    out_d = gh.new_out(T, N, out_dtype)
    bda.bda_dense_project(x_d, K, T, K, W_d, N, N, out_d, N, dtype, out_dtype, stream=gh.stream())
    torch.cuda.synchronize()
    return gh.to_host64(out_d, out_dtype)


def _softmax_attention(Q, K, V, n, d_h):
    out = np.empty_like(V)
    for h in range(n):
        s = slice(h * d_h, (h + 1) * d_h)
        a = Q[:, s] @ K[:, s].T / np.sqrt(d_h)
        a = np.exp(a - a.max(axis=1, keepdims=True))
        out[:, s] = (a / a.sum(axis=1, keepdims=True)) @ V[:, s]
    return out


def test_full_bda_layer_matches_mha():
    """All six steps of Algorithm "BD Attention Inference" for one MHA layer: Q' = X B_qk (GPU dense
    GEMM), K' and V' (GPU BD projection, both groups in one launch), softmax attention per head (host,
    float64, from the GPU's Q', K', V'), Y = O' B_vo (GPU dense GEMM).  Checked against the same
    steps in float64 on the same stored weights, and against plain MHA (Algorithm "MHA Inference")
    on the original weights, from which it may differ only by the storage rounding of the BD weights."""
    rng = np.random.default_rng(41)
    T, d, n, d_h = 200, 256, 4, 64
    X = rng.standard_normal((T, d))
    Wq, Wk, Wv = (rng.standard_normal((d, n * d_h)) / np.sqrt(d) for _ in range(3))
    Wo = rng.standard_normal((n * d_h, d)) / np.sqrt(n * d_h)
    dt = wl.F16
    Cqk, Bqk, off_k, _ = bda.bda_prepare(Wk, d, n, d_h, Wq, bda.SIDE_Q, bda.BASIS_RESIDUAL_MIN, 0, bda.BDA_F16)
    Cvo, Bvo, off_v, _ = bda.bda_prepare(Wv, d, n, d_h, Wo, bda.SIDE_O, bda.BASIS_RESIDUAL_MIN, 0, bda.BDA_F16)
    Xs, X64 = wl.to_storage(X, dt)
    Cs, C64 = wl.to_storage(np.hstack([Cqk, Cvo]), dt)
    _, Bqk64 = wl.to_storage(Bqk, dt)
    _, Bvo64 = wl.to_storage(Bvo, dt)
    # GPU
    Qp = _gpu_dense(X64, Bqk64, dt, wl.F32)
    KV, _ = gh.kv_project(Xs, Cs, d, d_h, [n, n], [off_k, off_v], dt, out_dtype=wl.F32)
    Kp, Vp = KV[:, :n * d_h], KV[:, n * d_h:]
    Op = _softmax_attention(Qp, Kp, Vp, n, d_h)
    Y = _gpu_dense(Op, Bvo64, dt, wl.F32)
    # the same steps in float64 on the same stored weights
    Qp_r = oracle.dense_project(X64, Bqk64)
    KV_r = oracle.kv_project(X64, C64, d_h, [n, n], [off_k, off_v])
    Op_r = _softmax_attention(Qp_r, KV_r[:, :n * d_h], KV_r[:, n * d_h:], n, d_h)
    assert_parity(Qp, Qp_r, d_h, dt, wl.F32, "Q'")
    assert_parity(KV, KV_r, d_h, dt, wl.F32, "K', V'")
    assert_parity(Op, Op_r, d_h, dt, wl.F32, "O'")
    # step 6 on the GPU against float64 on the very same stored O' (O' is rounded to the storage type
    # on its way into the GEMM; Y cancels heavily, so two roundings of slightly different O' would
    # not be comparable at the element level)
    _, Op16 = wl.to_storage(Op, dt)
    assert_parity(Y, oracle.dense_project(Op16, Bvo64), d, dt, wl.F32, "Y")
    # plain MHA on the original weights: the whole GPU pipeline differs from it only by storage rounding
    Y_mha = _softmax_attention(X64 @ Wq, X64 @ Wk, X64 @ Wv, n, d_h) @ Wo
    for name, y in (("GPU", Y), ("float64 BDA", oracle.dense_project(wl.to_storage(Op_r, dt)[1], Bvo64))):
        nmse = np.sum((y - Y_mha) ** 2) / np.sum(Y_mha ** 2)
        assert nmse < 1e-3, (name, nmse)


# --------------------------------------------------------------------------------- GPU preparation
def _prepare_device(W_in, w_dtype, d_c, H, d_h, off, c_dtype):
    if w_dtype == wl.F64:
        W_d = torch.from_numpy(np.ascontiguousarray(W_in, dtype=np.float64)).cuda()
    else:
        W_d = gh.to_device(wl.to_storage(W_in, w_dtype)[0], w_dtype)
    N = H * d_h
    tdt = {wl.F64: torch.float64, wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.int16}[c_dtype]
    C_d = torch.full((d_c - d_h, N), -7, dtype=tdt, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    bda.bda_prepare_device(W_d, N, w_dtype, d_c, H, d_h, off, C_d, N, c_dtype, flag, gh.stream())
    torch.cuda.synchronize()
    if c_dtype == wl.F64:
        C = C_d.cpu().numpy()
    else:
        C = gh.to_host64(C_d, c_dtype)
    return C, int(flag.item()), C_d


@pytest.mark.parametrize("d_c,H,d_h,off", [(512, 4, 128, 0), (512, 3, 128, 384), (512, 2, 128, 208),
                                           (256, 5, 64, 64), (96, 3, 32, 16), (64, 2, 16, 0)])
def test_prepare_device_matches_oracle(d_c, H, d_h, off):
    """GPU preparation (Gauss-Jordan inverse in float64) against the oracle's solve, same window.
    The two eliminate in different orders, so they agree to a multiple of cond * 2^-53, not bit for
    bit; the tolerance below is 1e-9 of the largest coefficient."""
    w = wl.custom_kv_workload("prep", T=1, d_c=d_c, d_h=d_h, H=[H], std=0.02, rms_norm=False, dtype=wl.F32, seed=50 + d_h)
    C_ref, _, off_ref, _ = oracle.prepare(w.W, d_c, H, d_h, mode=oracle.EXPLICIT, explicit_offset=off)
    assert off_ref == off
    C, flag, _ = _prepare_device(w.W, wl.F64, d_c, H, d_h, off, wl.F64)
    assert flag == 0
    assert np.max(np.abs(C - C_ref)) <= 1e-9 * np.max(np.abs(C_ref))
    # the transformed weight has the identity in its window rows (the paper's defining property)
    for h in range(H):
        A = w.W[off:off + d_h, h * d_h:(h + 1) * d_h]
        rest = np.concatenate([np.arange(0, off), np.arange(off + d_h, d_c)])
        assert np.allclose(C[:, h * d_h:(h + 1) * d_h] @ A, w.W[rest, h * d_h:(h + 1) * d_h], rtol=0, atol=1e-10)


@pytest.mark.parametrize("w_dtype", [wl.F16, wl.BF16, wl.F32])
@pytest.mark.parametrize("c_dtype", [wl.F16, wl.BF16, wl.F32])
def test_prepare_device_storage_types(w_dtype, c_dtype):
    """Inputs in a storage type are taken at their stored value; outputs are the float64 result rounded
    once: equal to rounding the float64 output of the same call, element for element."""
    d_c, H, d_h, off = 256, 3, 64, 0
    w = wl.custom_kv_workload("prep", T=1, d_c=d_c, d_h=d_h, H=[H], std=0.02, rms_norm=False, dtype=wl.F32, seed=61)
    _, W64 = wl.to_storage(w.W, w_dtype)
    C64, flag, _ = _prepare_device(w.W, w_dtype, d_c, H, d_h, off, wl.F64)
    assert flag == 0
    C_ref, _, _, _ = oracle.prepare(W64, d_c, H, d_h, mode=oracle.EXPLICIT, explicit_offset=off)
    assert np.max(np.abs(C64 - C_ref)) <= 1e-9 * np.max(np.abs(C_ref))
    Cs, flag, _ = _prepare_device(w.W, w_dtype, d_c, H, d_h, off, c_dtype)
    assert flag == 0
    _, want = wl.to_storage(C64, c_dtype)
    assert np.array_equal(Cs, want)


@pytest.mark.parametrize("d_h", [32, 64, 128])
def test_prepare_device_flags_singular_head_and_feeds_projection(d_h):
    d_c, H = 4 * d_h, 3
    w = wl.custom_kv_workload("prep", T=70, d_c=d_c, d_h=d_h, H=[H], std=0.125, rms_norm=False, dtype=wl.F16, seed=62)
    Wb = w.W.copy()
    Wb[5, d_h:2 * d_h] = Wb[9, d_h:2 * d_h]          # head 1: two equal rows inside the first window
    _, flag, C_d = _prepare_device(Wb, wl.F64, d_c, H, d_h, 0, wl.F64)
    assert flag == 2
    # heads that are fine are still written; the singular one keeps the caller's fill
    assert np.all(C_d.cpu().numpy()[:, d_h:2 * d_h] == -7)
    # regular input: prepare on the GPU in the storage type, project, compare with the oracle on that C
    Cs, flag, C_d = _prepare_device(w.W, wl.F64, d_c, H, d_h, 0, wl.F16)
    assert flag == 0
    c_d = gh.to_device(w.c_stored, wl.F16)
    out_d = gh.new_out(w.T, H * d_h, wl.F16)
    bda.bda_kv_project(c_d, d_c, w.T, d_c, d_h, [H], [0], C_d, H * d_h, out_d, H * d_h, wl.F16, wl.F16, gh.stream())
    torch.cuda.synchronize()
    ref = oracle.kv_project(w.c, Cs, d_h, [H], [0])
    assert_parity(gh.to_host64(out_d, wl.F16), ref, d_h, wl.F16, wl.F16, "prepare_device -> kv_project")
