"""Packed layout of C for launches with a few tokens: bda_pack_weights against the documented layout
(bit for bit), bda_kv_project_packed against the fp64 oracle and, bit for bit, against bda_kv_project
on the canonical C (same kernels, same order of operations: only the addresses of C differ)."""
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


def _stored_C(w, offs):
    Cs, col = [], 0
    for g, Hg in enumerate(w.H):
        C, _, _, _ = oracle.prepare(w.W[:, col:col + Hg * w.d_h], w.d_c, Hg, w.d_h, mode=oracle.EXPLICIT, explicit_offset=offs[g])
        Cs.append(C)
        col += Hg * w.d_h
    return wl.to_storage(np.hstack(Cs), w.dtype)


def _pack(C_d, ldC, w):
    nbytes = bda.bda_packed_weights_bytes(w.d_c, w.d_h, w.H, w.dtype)
    K, N = w.d_c - w.d_h, sum(w.H) * w.d_h
    assert nbytes == K * N * 2
    packed = torch.full((nbytes // 2 + 64,), 0x7B7B, dtype=torch.int16, device="cuda")      # 64 guard elements behind
    bda.bda_pack_weights(C_d, ldC, w.d_c, w.d_h, w.H, w.dtype, packed, gh.stream())
    torch.cuda.synchronize()
    assert bool((packed[nbytes // 2:] == 0x7B7B).all())
    return packed


def _case(w, offs, out_dtype=None, ldc=None, ldC=None, ld_out=None, wide=None):
    K, N, T = w.d_c - w.d_h, sum(w.H) * w.d_h, w.c_stored.shape[0]
    od = w.dtype if out_dtype is None else out_dtype
    C_stored, C64 = _stored_C(w, offs)
    ldc, ldC, ld_out = ldc or w.d_c, ldC or N, ld_out or N
    c_d, C_d = gh.to_device(w.c_stored, w.dtype, ldc), gh.to_device(C_stored, w.dtype, ldC)
    packed = _pack(C_d, ldC, w)
    # the layout: element (k, j) of slice s is element ((s K + k) 32 + j)
    bits = np.ascontiguousarray(C_stored).view(np.uint16)
    want = bits.reshape(K, N // 32, 32).transpose(1, 0, 2).reshape(-1)
    assert np.array_equal(packed[:K * N].cpu().numpy().view(np.uint16), want)
    if wide is not None:
        p = bda.bda_kv_project_plan(T, w.d_c, w.d_h, w.H, offs, w.dtype, out_dtype=out_dtype)
        assert p["kernel"] == bda.KERNEL_DECODE and (p["tile_columns"] == 128) == wide, p
    out_p = gh.new_out(T + 2, ld_out, od, fill=-7.0)
    bda.bda_kv_project_packed(c_d, ldc, T, w.d_c, w.d_h, w.H, offs, packed, out_p, ld_out, w.dtype, od, gh.stream())
    out_c = gh.new_out(T + 2, ld_out, od, fill=-7.0)
    bda.bda_kv_project(c_d, ldc, T, w.d_c, w.d_h, w.H, offs, C_d, ldC, out_c, ld_out, w.dtype, od, gh.stream())
    torch.cuda.synchronize()
    assert torch.equal(out_p, out_c), f"{w.name}: packed and canonical results differ"
    assert bool((out_p[T:] == -7.0).all())
    ref = oracle.kv_project(w.c, C64, w.d_h, w.H, offs)
    assert_parity(gh.to_host64(out_p[:T], od, N), ref, w.d_h, w.dtype, od, f"{w.name} packed offs={offs}")


@pytest.mark.parametrize("T", [1, 8, 32, 33, 64])
def test_packed_decode_config(T):
    # BASELINE configuration 3 (V2-Lite decode, N = 4096): the 32-column kernel
    _case(wl.kv_workload("decode", T=T), [0, 0], wide=False)


@pytest.mark.parametrize("T", [1, 31, 64])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, wl.F32)])
def test_packed_wide_slices(T, dtype, out_dtype):
    # 160 slices of 128 columns: the wide-slice kernel (4 packed sub-slices per workgroup), two groups
    # with windows off the 64 grid (seeds whose coefficients keep the results inside fp16's range)
    w = wl.custom_kv_workload("pk_wide", T=T, d_c=512, d_h=128, H=[100, 60], std=0.02, rms_norm=True, dtype=dtype, seed=50 + T)
    _case(w, [72, 384], out_dtype=out_dtype, wide=True)


@pytest.mark.parametrize("T", [1, 7, 40, 64])
@pytest.mark.parametrize("dtype,out_dtype", [(wl.F16, None), (wl.BF16, None), (wl.F16, wl.F32)])
def test_packed_groups_ragged_tiles_and_pitches(T, dtype, out_dtype):
    # strided token rows, C and output; K = 296 (a multiple of 8 only: the last rows of the last
    # 16-row request lie past the slice), K = 1088 (above the wide kernel's limit), a head width of 32
    w = wl.custom_kv_workload("pk_a", T=T, d_c=512, d_h=128, H=[3, 2], std=0.02, rms_norm=True, dtype=dtype, seed=70 + T)
    _case(w, [64, 384], out_dtype=out_dtype, ldc=520, ldC=648, ld_out=656)
    w = wl.custom_kv_workload("pk_b", T=T, d_c=360, d_h=64, H=[5, 1], std=0.05, rms_norm=True, dtype=dtype, seed=71 + T)
    _case(w, [8, 296], out_dtype=out_dtype)
    w = wl.custom_kv_workload("pk_c", T=T, d_c=1152, d_h=64, H=[5], std=0.02, rms_norm=True, dtype=dtype, seed=72 + T)
    _case(w, [512], out_dtype=out_dtype)
    w = wl.custom_kv_workload("pk_d", T=T, d_c=96, d_h=32, H=[1, 3], std=0.1, rms_norm=True, dtype=dtype, seed=73 + T)
    _case(w, [56, 0], out_dtype=out_dtype)


@pytest.mark.parametrize("T", [1, 64])
def test_packed_v3_width(T):
    # the V3-shaped weights of BASELINE configuration 4 (N = 32768, bf16) with a few tokens: 256 wide slices
    w = wl.kv_workload("v3")
    w = wl.KVWorkload(name="v3_decode", seed=w.seed, dtype=w.dtype, T=T, d_c=w.d_c, d_h=w.d_h, H=w.H,
                      c_stored=w.c_stored[:T], c=w.c[:T], W=w.W)
    _case(w, [0, 0], wide=True)


def test_packed_wide_kernel_ragged_last_tile_and_odd_K():
    # 159 full slices of 128 columns and one of 96 in the first group, 32 in the second; K = 296: rows
    # past K in the wide kernel's last request must read as zeros, not as the next sub-slice's rows
    w = wl.custom_kv_workload("pk_e", T=5, d_c=328, d_h=32, H=[639, 1], std=0.05, rms_norm=True, dtype=wl.BF16, seed=80)
    _case(w, [16, 296], wide=True)


def test_packed_rejects_what_the_few_token_kernels_do_not_take():
    w = wl.custom_kv_workload("pk_f", T=65, d_c=96, d_h=32, H=[2], std=0.1, rms_norm=True, dtype=wl.F16, seed=81)
    C_stored, _ = _stored_C(w, [0])
    c_d, C_d = gh.to_device(w.c_stored, w.dtype), gh.to_device(C_stored, w.dtype)
    packed = _pack(C_d, 64, w)
    out = gh.new_out(65, 64, wl.F16, fill=-7.0)
    with pytest.raises(bda.BdaError, match="64 tokens"):
        bda.bda_kv_project_packed(c_d, 96, 65, 96, 32, [2], [0], packed, out, 64, wl.F16, wl.F16, gh.stream())
    with pytest.raises(bda.BdaError, match="canonical"):       # token pitch not a multiple of 8: no few-token kernel
        bda.bda_kv_project_packed(c_d, 100, 4, 96, 32, [2], [0], packed, out, 64, wl.F16, wl.F16, gh.stream())
    torch.cuda.synchronize()
    assert bool((out == -7.0).all())
