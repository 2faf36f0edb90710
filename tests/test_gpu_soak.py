"""Bounded determinism soak of the single-launch verified GEMMs.

The workgroups of a tile-row hand their partial row sums and statistics to the last arriver through
device-scope stores, a wait for their completion and an arrival ticket, without a release / acquire fence (a
fence there writes back the whole L2).  A stale partial would show as an output that differs from the first
pass over the same input; nothing else in the suite would notice a rare one.  A few thousand back-to-back
launches on rotating inputs, every output compared bit for bit with the first pass of the same input, stopping
at the first mismatch."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import _dev, _gen, _session  # noqa: E402

_BITS = {torch.float32: torch.int32, torch.float64: torch.int64, torch.bfloat16: torch.int16,
         torch.float16: torch.int16, torch.int32: torch.int32}


def _differs(a, b):
    return (a.view(_BITS[a.dtype]) != b.view(_BITS[b.dtype])).sum()


@pytest.mark.parametrize("dtype,M,N,K,transB,launches", [
    ("bf16", 2048, 2048, 512, 0, 2000), ("f16", 1024, 2048, 512, 1, 2000),
    ("bf16", 4096, 5120, 256, 1, 600),   # 320 tiles: more than one round per compute unit, arrivals spread over rounds
    ("f32", 512, 512, 256, 0, 1500), ("f64", 512, 512, 256, 1, 1500),          # 64 x 64 tiles
    ("f32", 2048, 1024, 128, 1, 1000), ("f64", 1024, 2048, 128, 0, 1000),      # 128 x 128 tiles
])
def test_back_to_back_fused_launches_repeat_bit_for_bit(dtype, M, N, K, transB, launches):
    rot = 4
    sessions, inputs, first = [], [], []
    for k in range(rot):
        A, B = _gen(dtype, M, N, K, transB, 500 + k, "n_1_1" if k % 2 else "n_1e-6_1")
        dA, dB = _dev(A, dtype), _dev(B, dtype)
        vg = _session(M, N, K, dtype, transB)
        vg.run_fused(dA, dB)
        torch.cuda.synchronize()
        first.append({n: getattr(vg, n).clone() for n in ("C", "rowsum", "E", "T", "expected", "astat", "flags", "nflag")})
        sessions.append(vg)
        inputs.append((dA, dB))
    # one session (one workspace, one set of output buffers) takes all launches: the partials and counters of a
    # launch are what the previous launch, on another input, left behind
    vg = sessions[0]
    bad = torch.zeros((), dtype=torch.int64, device="cuda")
    for it in range(launches):
        k = it % rot
        dA, dB = inputs[k]
        vg.encode(dB, defer_S=(it % 2 == 0))
        vg.gemm_fused(dA, dB, deferred_S=(it % 2 == 0))
        for n, ref in first[k].items():
            bad += _differs(getattr(vg, n), ref)
        if it % 100 == 99:
            nbad = int(bad.item())
            assert nbad == 0, f"launch {it - 99}..{it}: {nbad} output words differ from the first pass ({dtype})"
    assert int(bad.item()) == 0
    print(f"{dtype} {M}x{N}x{K}: {launches} launches, every output identical to the first pass", flush=True)
