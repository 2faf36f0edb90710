"""Parity of the block-wise verification path (paper section 5.2 "Integration with Block-wise ABFT") with the
CPU oracle, through the C ABI: statistics, thresholds and checksums per block of W columns (W is the width
the GEMM kernels sum before they write a partial: 256, or 64 for FP32 / FP64)."""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import (_acc_np, _dev, _gen, _session, _tol, check_C)  # noqa: E402


def _emax_blk(dtype, K, W):
    from paper_2602_08043_amd import binding as vb
    return vb.vabft_default_emax(dtype, K, W)


def check_blocks(r, ob, dtype, rows_ok=True):
    tol = _tol(dtype)
    tiny = 1e-300
    assert np.all(np.abs(r["Be_blk"] - ob["Be_blk"]) <= tol * ob["scale_Be_blk"] + tiny), "Be_blk"
    W = ob["W"]
    mean_scale = ob["scale_Be_blk"].sum(axis=1) / W          # sum_k mean|B| of the block
    dS = np.abs(r["S_blk"] - ob["S_blk"])
    assert np.all(dS[:, 0] <= tol * mean_scale * 4 + tiny), "S1 per block"
    assert np.all(dS[:, 1] <= 1e-4 * ob["S_blk"][:, 1] + tiny), "S2 per block"
    assert np.all(dS[:, 2] <= 1e-4 * ob["S_blk"][:, 2] + tol * mean_scale ** 2 + tiny), "S3 per block"
    assert np.array_equal(r["astat"][:, 0].astype(np.float64), ob["astat"][:, 0])
    assert np.array_equal(r["astat"][:, 1].astype(np.float64), ob["astat"][:, 1])
    assert np.all(np.abs(r["expected_blk"] - ob["expected_blk"]) <= tol * ob["scale_expected_blk"] + tiny), "expected_blk"
    assert np.all(np.abs(r["T_blk"] - ob["T_blk"]) <= 1e-4 * ob["T_blk"] + tiny), "T_blk"
    if rows_ok:
        assert np.all(np.abs(r["rowsum_blk"] - ob["rowsum_blk"]) <= tol * ob["scale_rowsum_blk"] + tiny), "rowsum_blk"
        assert np.all(np.abs(r["E_blk"] - ob["E_blk"]) <= 2 * tol * ob["scale_rowsum_blk"] + tiny), "E_blk"
        assert np.all(np.abs(r["E"] - ob["E"]) <= 2 * tol * ob["scale_rowsum_blk"].sum(axis=0) + tiny), "E aggregate"


BLOCK_SHAPES = [("bf16", 512, 768, 256, 0), ("bf16", 512, 512, 128, 1), ("bf16", 300, 520, 200, 0),
                ("bf16", 257, 130, 77, 1), ("f16", 512, 256, 192, 1), ("f16", 100, 99, 50, 0),
                ("f32", 256, 256, 256, 0), ("f32", 200, 260, 70, 1), ("f64", 256, 384, 128, 0), ("f64", 131, 67, 33, 1),
                ("bf16", 1, 1, 1, 0), ("f64", 3, 2, 1, 1)]


@pytest.mark.parametrize("dtype,M,N,K,transB", BLOCK_SHAPES)
def test_blockwise_fault_free_parity(dtype, M, N, K, transB):
    from paper_2602_08043_amd import binding as vb
    W = vb.vabft_block_width(dtype)
    assert W == (64 if dtype in ("f32", "f64") else 256)
    for seed, dist in ((91, "n_1e-6_1"), (92, "n_1_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        print(f"blocks {dtype} {M}x{N}x{K} transB={transB} {dist} W={W}", flush=True)
        e_blk = _emax_blk(dtype, K, min(N, W))
        vg = _session(M, N, K, dtype, transB)
        assert vg.nblocks == (N + W - 1) // W
        vg.run_blocks(_dev(A, dtype), _dev(B, dtype))
        r = vg.results()
        ob = orc.verify_blocks(A, B, dtype, transB, W, e_blk)
        check_blocks(r, ob, dtype)
        check_C(r, ob, A, B, dtype, transB)
        assert r["nflag"] == 0 and r["nblockflag"] == 0 and not r["blockflags"].any() and not r["flags"].any()
        assert np.all(np.abs(r["E_blk"]) <= r["T_blk"])
        if dtype != "f64":
            assert not ob["blockflags"].any()


@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 768, 128, 0), ("bf16", 300, 520, 96, 1),
                                                 ("f32", 256, 384, 128, 0), ("f64", 200, 260, 70, 1)])
def test_blockwise_flags_exactly_the_block_of_the_fault(dtype, M, N, K, transB):
    from paper_2602_08043_amd import binding as vb
    W = vb.vabft_block_width(dtype)
    g = wl.rng(95, transB)
    A = wl.to_storage(g.integers(-1, 2, size=(M, K)).astype(np.float64), dtype)
    Bl = g.integers(-1, 2, size=(K, N)).astype(np.float64)
    B = wl.to_storage(np.ascontiguousarray(Bl.T) if transB else Bl, dtype)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    ob = orc.verify_blocks(A, B, dtype, transB, W, _emax_blk(dtype, K, min(N, W)))
    top = 51 if dtype == "f64" else 22
    cand = [(0, 0), (M - 1, N - 1), (min(255, M - 2), min(256, N - 2)), (M // 2, W - 1), (7, W), (M // 3, N // 2 + 5)]
    faults = [(i, j, top) for (i, j) in cand if abs(ob["C"][i, j]) >= 1]
    assert len(faults) >= 3
    vg = _session(M, N, K, dtype, transB)
    vg.encode_blocks(dB)
    vg.threshold_blocks(dA)
    vg.gemm_blocks(dA, dB, vg.make_inject(mode=1, faults=faults))
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == len(faults)
    rs = orc.replay_faults_blocks(ob["rowsum_blk"], recs, W)
    assert np.array_equal(r["rowsum_blk"].astype(np.float64), rs)
    E = ob["expected_blk"] - rs
    assert np.array_equal(r["E_blk"].astype(np.float64), E)
    want = orc.fault_flags(E, ob["T_blk"])
    assert np.array_equal(r["blockflags"], want)
    assert sorted(zip(*np.nonzero(want))) == sorted((j // W, i) for (i, j, _b) in faults)
    assert r["nblockflag"] == len(faults)
    rows = sorted(set(f[0] for f in faults))
    assert np.nonzero(r["flags"])[0].tolist() == rows and r["nflag"] == len(rows)
    assert np.array_equal(r["E"].astype(np.float64), E.sum(axis=0))
    # the fault-free call afterwards is clean
    vg.gemm_blocks(dA, dB)
    r = vg.results()
    assert r["nflag"] == 0 and r["nblockflag"] == 0 and not r["E_blk"].any()


def test_blockwise_thresholds_are_tighter_than_the_full_row_threshold_c2():
    """BF16 4096^3 (the benchmark workload): block quantities on sampled rows; a fault between the block
    threshold and the full-row threshold is caught block-wise only."""
    from paper_2602_08043_amd import binding as vb
    cfg = wl.make_config("c2_bf16_4096", seed=7)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    W = vb.vabft_block_width(dt)
    dA, dB = _dev(cfg["A"], dt), _dev(cfg["B"], dt)
    vg = _session(M, N, K, dt, tb)
    vg.run_blocks(dA, dB)
    r = vg.results()
    ob = orc.verify_blocks(cfg["A"], cfg["B"], dt, tb, W, _emax_blk(dt, K, W), full_gemm=False)
    check_blocks(r, ob, dt, rows_ok=False)
    rows = np.sort(wl.rng(7, 7).choice(M, size=16, replace=False))
    A = orc.decode(cfg["A"], dt)[rows]
    C = A @ orc.logical_B(cfg["B"], dt, tb)
    rs = C.reshape(len(rows), N // W, W).sum(axis=2).T
    assert np.all(np.abs(r["rowsum_blk"][:, rows] - rs) <= _tol(dt) * ob["scale_rowsum_blk"][:, rows])
    assert r["nflag"] == 0 and r["nblockflag"] == 0
    # full-row thresholds for comparison
    vg.run_fused(dA, dB)
    T_row = vg.results()["T"]
    ratio = float(np.median(T_row / r["T_blk"].mean(axis=0)))
    print(f"median full-row threshold / mean block threshold = {ratio:.1f}", flush=True)
    assert ratio > 3.0
