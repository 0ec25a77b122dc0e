"""The device entry points under HIP graph capture: nothing in them allocates, synchronises or records a
memset, so a captured sequence - GPU preparation with a window search (the entry point that allocates
nothing), repacking of C, the projection with many and with a few tokens, the gradients - replays to the
same bits as the eager calls.  The graph is replayed several times with eager work and synchronisations
of the program in between, and every replay is compared (earlier replays must not leave anything behind
that a later one depends on)."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import bda_workloads as wl  # noqa: E402
import paper_2510_01718_amd as bda  # noqa: E402

pytestmark = pytest.mark.gpu


def test_captured_sequence_replays_to_the_eager_results():
    lib = bda.load()
    d_c, d_h, H, T, Td = 512, 128, [6, 4], 700, 8
    N = sum(H) * d_h
    rng = np.random.default_rng(77)
    W = torch.from_numpy(rng.standard_normal((d_c, N)) * 0.05).cuda()
    c = torch.from_numpy(rng.standard_normal((T, d_c))).cuda().to(torch.float16)
    d_out = torch.from_numpy(rng.standard_normal((T, N)) * 0.1).cuda().to(torch.float16)
    vp = ctypes.c_void_p

    def buffers():
        return dict(C=torch.full((d_c - d_h, N), float("nan"), dtype=torch.float16, device="cuda"),
                    off=torch.full((2,), -9, dtype=torch.int32, device="cuda"),
                    flag=torch.zeros(1, dtype=torch.int32, device="cuda"),
                    packed=torch.full(((d_c - d_h) * N,), float("nan"), dtype=torch.float16, device="cuda"),
                    out=torch.full((T, N), float("nan"), dtype=torch.float16, device="cuda"),
                    out_few=torch.full((Td, N), float("nan"), dtype=torch.float16, device="cuda"),
                    gc=torch.full((T, d_c), float("nan"), dtype=torch.float16, device="cuda"),
                    gC=torch.full((d_c - d_h, N), float("nan"), dtype=torch.float16, device="cuda"))

    def prepare(b, stream):
        s = vp(stream)
        col = 0
        for g, Hg in enumerate(H):                 # one window search per group, on the device, into C's column block
            Wg = W[:, col:col + Hg * d_h]
            rc = lib.bda_prepare_device_static(vp(Wg.data_ptr()), N, wl.F64, d_c, Hg, d_h, None, 0, 0, bda.SIDE_NONE,
                                               bda.BASIS_RESIDUAL_MIN, 0, vp(b["C"].data_ptr() + col * 2), N, None, 0, wl.F16,
                                               vp(b["off"].data_ptr() + 4 * g), None, vp(b["flag"].data_ptr()), s)
            assert rc == 0, lib.bda_last_error()
            col += Hg * d_h

    def sequence(b, stream, offs):
        # (the window starts a search writes stay on the device; the host passes the ones it learnt from an
        # earlier run of the same search to the calls that follow)
        prepare(b, stream)
        bda.bda_pack_weights(b["C"], N, d_c, d_h, H, wl.F16, b["packed"], stream)
        bda.bda_kv_project(c, d_c, T, d_c, d_h, H, offs, b["C"], N, b["out"], N, wl.F16, wl.F16, stream)
        bda.bda_kv_project_packed(c, d_c, Td, d_c, d_h, H, offs, b["packed"], b["out_few"], N, wl.F16, wl.F16, stream)
        bda.bda_kv_project_backward(c, d_c, d_out, N, b["C"], N, T, d_c, d_h, H, offs, b["gc"], d_c, b["gC"], N, wl.F16, wl.F16, stream)

    first = buffers()
    prepare(first, int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    offs = first["off"].tolist()
    assert all(o in (0, d_c - d_h) for o in offs) and int(first["flag"].item()) == 0
    eager = buffers()
    sequence(eager, int(torch.cuda.current_stream().cuda_stream), offs)
    torch.cuda.synchronize()
    assert eager["off"].tolist() == offs
    for name, t in eager.items():                  # every buffer started as NaN (or -9): all of it was written
        unwritten = (t == -9) if t.dtype == torch.int32 else torch.isnan(t)
        assert not bool(unwritten.any()), name

    cap = buffers()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence(cap, int(torch.cuda.current_stream().cuda_stream), offs)
    torch.cuda.synchronize()
    for replay in range(4):
        for name, t in cap.items():                # eager work of the program between the replays
            t.fill_(float("nan") if t.dtype != torch.int32 else 0 if name == "flag" else -9)   # (the flag is only ever raised: the caller clears it)
        scratch = torch.randn(1 << 20, device="cuda").sum()    # a library reduction and a synchronisation in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(cap[name], eager[name]), f"replay {replay}: {name} differs from the eager call"
        del scratch
