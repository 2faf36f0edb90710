"""The whole path recorded into a HIP graph (through torch.cuda.graphs) and replayed: nothing in the library
allocates, synchronises or uses host state between launches, and counters are cleared by fill kernels rather
than memset nodes, so every replay must reproduce the eager results exactly -- including after other work has
run between replays, and with a fault injected in some replays only through device-resident arguments."""
import numpy as np
import pytest

import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import _dev, _gen, _session  # noqa: E402


@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 768, 256, 0), ("f32", 256, 256, 128, 1),
                                                 ("bf16", 300, 520, 200, 1)])
def test_graph_replay_matches_eager(dtype, M, N, K, transB):
    A, B = _gen(dtype, M, N, K, transB, 81, "n_1e-6_1")
    A2, B2 = _gen(dtype, M, N, K, transB, 82, "n_1_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    faults = [(M // 2, N // 3, 29)]
    inj = vg.make_inject(mode=1, faults=faults)
    keys = ("Be", "S", "expected", "T", "rowsum", "E", "flags", "rowsum2", "loc", "delta", "colsum", "E_col",
            "colflags")

    def whole_path():
        vg.encode(dB, defer_S=True)                # S1..S3 left as partials, folded inside the fused call
        vg.gemm_fused(dA, dB, deferred_S=True)
        t_deferred = vg.T.clone()
        vg.encode(dB)
        vg.gemm_fused(dA, dB)                      # fault-free fused call
        t_plain = vg.T.clone()
        c_clean = vg.C.clone()
        vg.run_weighted(dA, dB, inj=inj, correct=1)  # weighted route with the planted fault, corrected
        vg.encode_a(dA)
        vg.threshold_cols(dB)
        vg.gemm_rc(dA, dB, inj)                    # row + column check with the fault
        return c_clean, t_deferred, t_plain

    # eager reference
    c_ref, t_ref, t_plain_ref = whole_path()
    torch.cuda.synchronize()
    assert torch.equal(t_ref, t_plain_ref)  # the deferred fold gives the same thresholds bit for bit
    ref = {k: getattr(vg, k).clone() for k in keys}
    ref["C"] = vg.C.clone()
    ref["nflag"], ref["ncolflag"], ref["ncorrected"] = (int(vg.nflag.item()), int(vg.ncolflag.item()),
                                                         int(vg.ncorrected.item()))
    assert ref["nflag"] == 1 and ref["ncolflag"] == 1 and ref["ncorrected"] == 1

    # capture on a side stream, as torch requires
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        whole_path()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(s)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        c_graph, t_graph, t_plain_graph = whole_path()

    for replay in range(4):
        # other work between replays: different inputs through the same session (same workspace, same outputs)
        vg.run_fused(_dev(A2, dtype), _dev(B2, dtype))
        for k in keys:
            getattr(vg, k).fill_(0 if getattr(vg, k).dtype in (torch.int32,) else 7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(getattr(vg, k), ref[k]), (replay, k)
        assert torch.equal(vg.C, ref["C"]) and torch.equal(c_graph, c_ref) and torch.equal(t_graph, t_ref) and torch.equal(t_plain_graph, t_ref)
        assert int(vg.nflag.item()) == ref["nflag"] and int(vg.ncolflag.item()) == ref["ncolflag"]
        assert int(vg.ncorrected.item()) == ref["ncorrected"]
