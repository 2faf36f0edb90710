"""Parity of the column-checksum path (paper section 2.2: c1, A^c, C^{c1}, C^{c1'}) with the CPU oracle,
through the C ABI.  Tolerances as in tests/test_gpu_parity.py, with the scales of the column quantities."""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import (_acc_np, _dev, _emax, _gen, _session, _tol, check_C, check_light, check_rows)  # noqa: E402


def check_columns(r, oc, dtype, M, N, K):
    tol = _tol(dtype)
    tiny = 1e-300
    assert np.all(np.abs(r["eA"] - oc["eA"]) <= tol * oc["scale_eA"] + tiny), "eA"
    assert np.array_equal(r["acolstat"][:, 0].astype(np.float64), oc["acolstat"][:, 0]), "A column max"
    assert np.array_equal(r["acolstat"][:, 1].astype(np.float64), oc["acolstat"][:, 1]), "A column min"
    assert np.all(np.abs(r["acolstat"][:, 2] - oc["acolstat"][:, 2]) <= tol * oc["scale_eA"] / M + tiny), "A column mean"
    assert np.array_equal(r["bcolstat"][:, 0].astype(np.float64), oc["bcolstat"][:, 0]), "B column max"
    assert np.array_equal(r["bcolstat"][:, 1].astype(np.float64), oc["bcolstat"][:, 1]), "B column min"
    mean_abs = oc["scale_eA"] / M
    mu = oc["acolstat"][:, 2]
    span = oc["acolstat"][:, 0] - oc["acolstat"][:, 1]
    dS = np.abs(r["SA"] - oc["SA"])
    assert dS[0] <= tol * mean_abs.sum() + tiny, "S1 of A"
    assert dS[1] <= tol * (span * mean_abs).sum() + 1e-12 * oc["SA"][1] + tiny, "S2 of A"
    assert dS[2] <= tol * (2 * np.abs(mu) * mean_abs + mean_abs ** 2 * tol).sum() + tiny, "S3 of A"
    assert np.all(np.abs(r["expected_col"] - oc["expected_col"]) <= tol * oc["scale_expected_col"] + tiny), "expected_col"
    assert np.all(np.abs(r["T_col"] - oc["T_col"]) <= max(tol, 2e-7 if dtype != "f64" else 0) * oc["T_col"] + tiny), "T_col"
    assert np.all(np.abs(r["colsum"] - oc["colsum"]) <= tol * oc["scale_colsum"] + tiny), "colsum"
    assert np.all(np.abs(r["E_col"] - oc["E_col"]) <= 2 * tol * oc["scale_colsum"] + tiny), "E_col"


COL_SHAPES = [("bf16", 512, 768, 256, 0), ("bf16", 512, 512, 128, 1), ("bf16", 300, 520, 200, 0),
              ("bf16", 257, 130, 77, 1), ("f16", 512, 256, 192, 0), ("f16", 100, 99, 50, 1),
              ("f32", 256, 256, 256, 0), ("f32", 200, 260, 70, 1), ("f64", 256, 384, 128, 0), ("f64", 131, 67, 33, 1),
              ("bf16", 1, 1, 1, 0), ("f64", 3, 2, 1, 1)]


@pytest.mark.parametrize("dtype,M,N,K,transB", COL_SHAPES)
def test_column_check_fault_free_parity(dtype, M, N, K, transB):
    for seed, dist in ((61, "n_1e-6_1"), (62, "n_1_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        print(f"columns {dtype} {M}x{N}x{K} transB={transB} {dist}", flush=True)
        vg = _session(M, N, K, dtype, transB)
        e_row, e_col = _emax(dtype, K, N), _emax(dtype, K, max(N, M))
        vg.run_rc(_dev(A, dtype), _dev(B, dtype))
        r = vg.results()
        o = orc.verify(A, B, dtype, transB, e_max=e_row)
        oc = orc.verify_columns(A, B, dtype, transB, e_max=e_col)
        check_light(r, o, dtype, M, N, K)
        check_rows(r, o, dtype)
        check_C(r, o, A, B, dtype, transB)
        check_columns(r, oc, dtype, M, N, K)
        assert r["nflag"] == 0 and not r["flags"].any()
        assert r["ncolflag"] == 0 and not r["colflags"].any()
        if dtype != "f64":  # the oracle's own FP64 rounding noise is of the order of an FP64-level threshold
            assert not oc["colflags"].any()
        assert np.all(np.abs(r["E_col"]) <= r["T_col"])


@pytest.mark.parametrize("dtype,M,N,K,transB", [("f32", 256, 384, 128, 0), ("bf16", 512, 512, 128, 0),
                                                 ("bf16", 300, 520, 96, 1), ("f64", 200, 260, 70, 1)])
def test_row_and_column_flags_intersect_at_the_fault(dtype, M, N, K, transB):
    """Small-integer matrices (exact arithmetic): every planted fault raises exactly its row flag and its
    column flag, with E_row = E_col = -delta."""
    g = wl.rng(71, transB)
    A = wl.to_storage(g.integers(-1, 2, size=(M, K)).astype(np.float64), dtype)
    Bl = g.integers(-1, 2, size=(K, N)).astype(np.float64)
    B = wl.to_storage(np.ascontiguousarray(Bl.T) if transB else Bl, dtype)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    oc = orc.verify_columns(A, B, dtype, transB, e_max=_emax(dtype, K, max(N, M)))
    top = 51 if dtype == "f64" else 22
    # distinct rows and distinct columns, including the corners of the matrix and of the 256-tiles
    cand = [(0, 0), (M - 1, N - 1), (min(255, M - 2), min(256, N - 2)), (M // 2, 1), (7, N // 2 + 3), (M // 3, N // 3)]
    faults = [(i, j, top) for (i, j) in cand if abs(o["C"][i, j]) >= 1]
    assert len(faults) >= 3
    vg = _session(M, N, K, dtype, transB)
    vg.encode(dB)
    vg.threshold(dA)
    vg.encode_a(dA)
    vg.threshold_cols(dB)
    vg.gemm_rc(dA, dB, vg.make_inject(mode=1, faults=faults))
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == len(faults)
    rows = sorted(f[0] for f in faults)
    cols = sorted(f[1] for f in faults)
    assert np.nonzero(r["flags"])[0].tolist() == rows and r["nflag"] == len(rows)
    assert np.nonzero(r["colflags"])[0].tolist() == cols and r["ncolflag"] == len(cols)
    cs = orc.replay_faults_columns(oc["colsum"], recs)
    assert np.array_equal(r["colsum"].astype(np.float64), cs)
    assert np.array_equal(r["E_col"].astype(np.float64), oc["expected_col"] - cs)
    assert np.array_equal(r["colflags"], orc.fault_flags(oc["expected_col"] - cs, oc["T_col"]))
    for (i, j, _b, before, after) in recs:
        assert r["E"][i] == -(after - before) == r["E_col"][j]
    # and the same call without faults is clean again
    vg.gemm_rc(dA, dB)
    r = vg.results()
    assert r["nflag"] == 0 and r["ncolflag"] == 0 and not r["E_col"].any()


def test_column_check_full_size_c2():
    cfg = wl.make_config("c2_bf16_4096", seed=5)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    dA, dB = _dev(cfg["A"], dt), _dev(cfg["B"], dt)
    vg = _session(M, N, K, dt, tb)
    vg.run_rc(dA, dB, inj=None)
    r = vg.results()
    oc = orc.verify_columns(cfg["A"], cfg["B"], dt, tb, e_max=_emax(dt, K, max(N, M)), full_gemm=False)
    tol = _tol(dt)
    assert np.all(np.abs(r["eA"] - oc["eA"]) <= tol * oc["scale_eA"])
    assert np.all(np.abs(r["expected_col"] - oc["expected_col"]) <= tol * oc["scale_expected_col"])
    assert np.all(np.abs(r["T_col"] - oc["T_col"]) <= 2e-7 * oc["T_col"] + tol * oc["T_col"])
    # sampled columns of the product
    cols = np.unique(np.concatenate([wl.rng(5, 9).choice(N, size=24, replace=False), [0, 255, 256, N - 1]]))
    A = orc.decode(cfg["A"], dt)
    Bc = orc.logical_B(cfg["B"], dt, tb)[:, cols]
    colsum = (A @ Bc).sum(axis=0)
    assert np.all(np.abs(r["colsum"][cols] - colsum) <= tol * oc["scale_colsum"][cols])
    assert r["ncolflag"] == 0 and r["nflag"] == 0
    assert np.all(np.abs(r["E_col"]) <= r["T_col"])
    # one planted fault: its row and its column
    i, j = 1234, 3210
    vg.gemm_rc(dA, dB, vg.make_inject(mode=1, faults=[(i, j, 28)]))
    r2 = vg.results()
    assert np.nonzero(r2["flags"])[0].tolist() == [i] and np.nonzero(r2["colflags"])[0].tolist() == [j]


def test_column_argument_errors():
    from paper_2602_08043_amd import binding as vb
    vg = _session(64, 64, 64, "f32", 0)
    A, B = _gen("f32", 64, 64, 64, 0, 1)
    dA, dB = _dev(A, "f32"), _dev(B, "f32")
    p, st = vg.problem, vg._stream()
    assert vb.vabft_encode_a(p, dA.data_ptr(), None, vg.acolstat.data_ptr(), vg.SA.data_ptr(), vg.ws.data_ptr(),
                             vg.ws_bytes, st, check=False) == vb.VABFT_EINVAL
    assert vb.vabft_encode_a(p, dA.data_ptr(), vg.eA.data_ptr(), vg.acolstat.data_ptr(), vg.SA.data_ptr(), None, 0, st,
                             check=False) == vb.VABFT_EWORKSPACE
    assert vb.vabft_threshold_cols(p, dB.data_ptr(), vg.eA.data_ptr(), vg.SA.data_ptr(), 0.0, 2.5,
                                   vg.bcolstat.data_ptr(), vg.expected_col.data_ptr(), vg.T_col.data_ptr(),
                                   vg.ws.data_ptr(), vg.ws_bytes, st, check=False) == vb.VABFT_EINVAL
    assert vb.vabft_gemm_verified_rc(p, dA.data_ptr(), dB.data_ptr(), vg.C.data_ptr(), vg.expected.data_ptr(),
                                     vg.T.data_ptr(), vg.expected_col.data_ptr(), vg.T_col.data_ptr(), None,
                                     vg.rowsum.data_ptr(), vg.E.data_ptr(), vg.flags.data_ptr(), vg.nflag.data_ptr(),
                                     None, vg.E_col.data_ptr(), vg.colflags.data_ptr(), vg.ncolflag.data_ptr(), None,
                                     None, vg.ws.data_ptr(), vg.ws_bytes, st, check=False) == vb.VABFT_EINVAL
