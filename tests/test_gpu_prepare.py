"""GPU preparation (bda_prepare_device_ex) against the oracle's prepare: every window mode, with and
without companion weights, stored-form residuals, the search's choice, head widths up to 256.

The GPU inverts the basis block by Gauss-Jordan elimination, the oracle solves by LU: the float64
results agree to a multiple of cond * 2^-53, not bit for bit.  Stored (rounded) outputs are therefore
compared with the rounding of the GPU's own float64 result (exact), and that float64 result with the
oracle's (1e-9 of the largest coefficient).  Residuals are compared to 1e-6 relative; window choices
must be equal (the inputs keep the candidates' residuals apart)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import bda_workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402
import oracle  # noqa: E402
import paper_2510_01718_amd as bda  # noqa: E402

pytestmark = pytest.mark.gpu

_TDT = {wl.F64: torch.float64, wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.int16}
FILL = -7


def _weights(d_c, H, d_h, d_side, seed, weak_first=True):
    """Gaussian projection and companions; in head 0 two rows of the first window are made nearly equal,
    so that the first window reconstructs visibly worse than the others once C is rounded."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((d_c, H * d_h)) * 0.05
    if weak_first:
        W[1, :d_h] = W[0, :d_h] + 2e-4 * rng.standard_normal(d_h)
    Wq = rng.standard_normal((d_side, H * d_h)) * 0.05
    Wo = rng.standard_normal((H * d_h, d_side)) * 0.05
    return W, Wq, Wo


def _host(t, dtype):
    if dtype == wl.F64:
        return t.cpu().numpy().astype(np.float64)
    return gh.to_host64(t, dtype)


def _run(W, d_c, H, d_h, c_dtype, side=None, side_kind=oracle.SIDE_NONE, mode=oracle.FIRST, explicit_offset=0,
         want_resid=True, workspace_bytes=None):
    N = H * d_h
    W_d = torch.from_numpy(np.ascontiguousarray(W)).cuda()
    C_d = torch.full((d_c - d_h, N), FILL, dtype=_TDT[c_dtype], device="cuda")
    side_d = side_out_d = None
    ld_side = d_side = 0
    if side is not None:
        side_d = torch.from_numpy(np.ascontiguousarray(side)).cuda()
        side_out_d = torch.full(side.shape, FILL, dtype=_TDT[c_dtype], device="cuda")
        ld_side = side.shape[1]
        d_side = side.shape[0] if side_kind == oracle.SIDE_Q else side.shape[1]
    off_d = torch.full((1,), -99, dtype=torch.int32, device="cuda")
    resid_d = torch.zeros(3, dtype=torch.float64, device="cuda") if want_resid else None
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    need = bda.bda_prepare_device_workspace_bytes(d_c, H, d_h, mode, want_resid)
    nbytes = need if workspace_bytes is None else workspace_bytes
    ws = torch.full((max(nbytes, 16),), 0x5A, dtype=torch.uint8, device="cuda") if nbytes else None   # (stale contents must not matter)
    bda.bda_prepare_device_ex(W_d, N, wl.F64, d_c, H, d_h, C_d, N, c_dtype, side=side_d, ld_side=ld_side, d_side=d_side,
                              side_kind=side_kind, side_out=side_out_d, ld_side_out=ld_side, mode=mode,
                              explicit_offset=explicit_offset, basis_offset_out=off_d, resid_out=resid_d,
                              singular_head=flag, workspace=ws, workspace_bytes=nbytes, stream=gh.stream())
    torch.cuda.synchronize()
    return dict(C=_host(C_d, c_dtype), side=None if side is None else _host(side_out_d, c_dtype), off=int(off_d.item()),
                resid=None if resid_d is None else resid_d.cpu().numpy(), flag=int(flag.item()), need=need)


def _check_against_oracle(W, d_c, H, d_h, store, side, side_kind, mode, explicit_offset=0, **kw):
    C_ref, side_ref, off_ref, resid_ref = oracle.prepare(W, d_c, H, d_h, side=side, side_kind=side_kind, mode=mode,
                                                         explicit_offset=explicit_offset, store_dtype=store)
    exact = _run(W, d_c, H, d_h, wl.F64, side, side_kind, oracle.EXPLICIT, off_ref, **kw)      # float64 outputs, the oracle's window
    assert exact["flag"] == 0 and exact["off"] == off_ref
    assert np.max(np.abs(exact["C"] - C_ref)) <= 1e-9 * np.max(np.abs(C_ref))
    if side is not None:
        assert np.max(np.abs(exact["side"] - side_ref)) <= 1e-12 * np.max(np.abs(side_ref))
    got = _run(W, d_c, H, d_h, store, side, side_kind, mode, explicit_offset, **kw)             # stored outputs, the mode under test
    what = f"mode {mode} side {side_kind} store {store}: oracle window {off_ref}, residuals {resid_ref}, GPU {got['off']} {got['resid']}"
    assert got["flag"] == 0, what
    assert got["off"] == off_ref, what
    assert np.array_equal(got["C"], wl.to_storage(exact["C"], store)[1]), what
    if side is not None:
        assert np.array_equal(got["side"], wl.to_storage(exact["side"], store)[1]), what
    last = d_c - d_h
    want = [resid_ref.get(0, np.nan), resid_ref.get(last, np.nan), resid_ref[off_ref]]
    for g, r in zip(got["resid"], want):
        assert (np.isnan(g) and np.isnan(r)) or abs(g - r) <= 1e-6 * abs(r), what
    return got, resid_ref


@pytest.mark.parametrize("store", [wl.F16, wl.BF16])
@pytest.mark.parametrize("side_kind", [oracle.SIDE_NONE, oracle.SIDE_Q, oracle.SIDE_O])
@pytest.mark.parametrize("mode,explicit_offset", [(oracle.FIRST, 0), (oracle.LAST, 0), (oracle.RESIDUAL_MIN, 0),
                                                  (oracle.OFFSET_SEARCH, 0), (oracle.EXPLICIT, 40)])
def test_prepare_device_ex_modes_and_companions(store, side_kind, mode, explicit_offset):
    """Algorithm "BD Attention Preparation (QK)" / Appendix "BD for VO in MHA" / "Residual-Min with Offset
    Search" on the GPU: outputs, residuals of the stored form and the chosen window against the oracle."""
    d_c, H, d_h, d_side = 128, 3, 32, 40
    W, Wq, Wo = _weights(d_c, H, d_h, d_side, seed=300 + 10 * mode + side_kind)
    side = None if side_kind == oracle.SIDE_NONE else Wq if side_kind == oracle.SIDE_Q else Wo
    got, resid_ref = _check_against_oracle(W, d_c, H, d_h, store, side, side_kind, mode, explicit_offset)
    if mode == oracle.RESIDUAL_MIN:
        assert got["off"] == d_c - d_h and resid_ref[0] > 1.5 * resid_ref[d_c - d_h]     # the weak first window lost
    if mode == oracle.OFFSET_SEARCH:
        assert len(resid_ref) == 7 and got["off"] != 0


def test_prepare_device_ex_search_keeps_first_on_ties_and_reports_nan_for_windows_not_tried():
    """Float64 storage: every window reconstructs to rounding noise; explicit window: first / last not evaluated."""
    d_c, H, d_h = 96, 2, 32
    W, _, _ = _weights(d_c, H, d_h, 8, seed=77, weak_first=False)
    got = _run(W, d_c, H, d_h, wl.F16, mode=oracle.EXPLICIT, explicit_offset=16)
    assert got["off"] == 16 and np.isnan(got["resid"][0]) and np.isnan(got["resid"][1]) and got["resid"][2] > 0
    # no residuals asked for and one window: no workspace at all
    plain = _run(W, d_c, H, d_h, wl.F16, mode=oracle.LAST, want_resid=False)
    assert plain["need"] == 0 and plain["off"] == d_c - d_h
    C_ref, _, _, _ = oracle.prepare(W, d_c, H, d_h, mode=oracle.LAST)
    assert np.max(np.abs(plain["C"] - wl.to_storage(C_ref, wl.F16)[1])) <= 2.0 ** -10 * np.max(np.abs(C_ref))


@pytest.mark.parametrize("d_c,H,d_h,blocks", [(512, 3, 256, 1), (512, 3, 256, 2), (448, 2, 192, None), (320, 5, 160, None)])
def test_prepare_device_ex_wide_heads(d_c, H, d_h, blocks):
    """Head widths above 128: the basis block is inverted in the workspace, `blocks` heads per launch
    (None: the size bda_prepare_device_workspace_bytes suggests)."""
    W, Wq, _ = _weights(d_c, H, d_h, 24, seed=500 + d_h)
    ws = None
    if blocks is not None:
        ws = 1024 + 256 * ((2 * H * (1024 // H if 1024 // H < 64 else 64) * 8 + 255) // 256) + blocks * d_h * d_h * 8
    _check_against_oracle(W, d_c, H, d_h, wl.BF16, Wq, oracle.SIDE_Q, oracle.RESIDUAL_MIN, workspace_bytes=ws)


def test_prepare_device_ex_singular_windows():
    """A head of rank below d_h makes every window singular: the search reports -1.  One singular
    candidate among good ones is passed over; an explicit singular window is flagged and its C not written."""
    d_c, H, d_h = 96, 3, 32
    W, _, _ = _weights(d_c, H, d_h, 8, seed=91, weak_first=False)
    Wbad = W.copy()
    Wbad[:, d_h + 5] = Wbad[:, d_h + 9]                # head 1: two equal columns in every window
    got = _run(Wbad, d_c, H, d_h, wl.F16, mode=oracle.OFFSET_SEARCH)
    assert got["off"] == -1 and np.isinf(got["resid"][0]) and np.isinf(got["resid"][2])
    W1 = W.copy()
    W1[3, 2 * d_h:3 * d_h] = W1[7, 2 * d_h:3 * d_h]    # head 2: two equal rows inside the first window only
    got = _run(W1, d_c, H, d_h, wl.F16, mode=oracle.RESIDUAL_MIN)
    assert got["off"] == d_c - d_h and np.isinf(got["resid"][0]) and got["flag"] == 0
    C_ref, _, _, _ = oracle.prepare(W1, d_c, H, d_h, mode=oracle.LAST)
    assert np.max(np.abs(got["C"] - wl.to_storage(C_ref, wl.F16)[1])) <= 2.0 ** -10 * np.max(np.abs(C_ref))
    got = _run(W1, d_c, H, d_h, wl.F16, mode=oracle.FIRST)
    assert got["flag"] == 3 and np.all(got["C"][:, 2 * d_h:] == FILL) and not np.any(got["C"][:, :2 * d_h] == FILL)


def test_prepare_device_ex_calls_overlapping_on_several_streams():
    """Searches for different projections issued on four streams at once, each with a workspace and outputs of
    its own (the calls share nothing else): every one gives what it gives alone on one stream, bit for bit."""
    d_c, H, d_h, d_side = 192, 4, 64, 96
    jobs = []
    for j in range(8):
        W, Wq, Wo = _weights(d_c, H, d_h, d_side, seed=700 + j, weak_first=(j % 2 == 0))
        kind = oracle.SIDE_Q if j % 2 == 0 else oracle.SIDE_O
        jobs.append((W, Wq if kind == oracle.SIDE_Q else Wo, kind))
    alone = [_run(W, d_c, H, d_h, wl.F16, side, kind, oracle.OFFSET_SEARCH) for W, side, kind in jobs]
    N = H * d_h
    need = bda.bda_prepare_device_workspace_bytes(d_c, H, d_h, oracle.OFFSET_SEARCH, True)
    streams = [torch.cuda.Stream() for _ in range(4)]
    bufs = []
    for W, side, kind in jobs:
        bufs.append(dict(W=torch.from_numpy(np.ascontiguousarray(W)).cuda(), side=torch.from_numpy(np.ascontiguousarray(side)).cuda(),
                         C=torch.full((d_c - d_h, N), FILL, dtype=torch.float16, device="cuda"),
                         side_out=torch.full(side.shape, FILL, dtype=torch.float16, device="cuda"),
                         off=torch.full((1,), -99, dtype=torch.int32, device="cuda"), resid=torch.zeros(3, dtype=torch.float64, device="cuda"),
                         flag=torch.zeros(1, dtype=torch.int32, device="cuda"), ws=torch.full((need,), 0x5A, dtype=torch.uint8, device="cuda")))
    torch.cuda.synchronize()
    for rep in range(3):                                   # three waves of eight calls, two per stream, nothing waits in between
        for j, ((W, side, kind), b) in enumerate(zip(jobs, bufs)):
            bda.bda_prepare_device_ex(b["W"], N, wl.F64, d_c, H, d_h, b["C"], N, wl.F16, side=b["side"], ld_side=side.shape[1], d_side=d_side,
                                      side_kind=kind, side_out=b["side_out"], ld_side_out=side.shape[1], mode=oracle.OFFSET_SEARCH,
                                      basis_offset_out=b["off"], resid_out=b["resid"], singular_head=b["flag"], workspace=b["ws"],
                                      workspace_bytes=need, stream=int(streams[j % 4].cuda_stream))
    torch.cuda.synchronize()
    for j, (b, ref) in enumerate(zip(bufs, alone)):
        assert int(b["flag"].item()) == 0 and int(b["off"].item()) == ref["off"], j
        assert np.array_equal(_host(b["C"], wl.F16), ref["C"]) and np.array_equal(_host(b["side_out"], wl.F16), ref["side"]), j
        assert np.array_equal(b["resid"].cpu().numpy(), ref["resid"]), j
