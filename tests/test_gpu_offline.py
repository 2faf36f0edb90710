"""Parity of the offline (post-quantisation) check, paper section 3.6 "Offline vs. Online ABFT", with the
CPU oracle.  The row sum of a stored 16-bit product depends on how each element was rounded; an element
whose exact value lies closer to a rounding boundary than the accumulation error can legitimately land on
either side, so the row-sum tolerance adds one unit in the last place for every such element."""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import (U_OUT, _acc_np, _dev, _gen, _session, _tol, check_C, check_light)  # noqa: E402


def _emax_off(dtype, K, N):
    from paper_2602_08043_amd import binding as vb
    return vb.vabft_default_emax_offline(dtype, K, N)


def _offline_rowsum_tolerance(o, A_st, B_st, dtype, transB):
    """tol * scale + one output ulp per element that sits within the accumulation error of a rounding
    boundary of the output type."""
    tol = _tol(dtype)
    base = tol * o["scale_rowsum"] + 1e-300
    if dtype in ("f32", "f64"):
        return base
    C = o["C"]
    q = orc.quantize(C, dtype)
    with np.errstate(divide="ignore"):
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(q), 1e-300))) - (7 if dtype == "bf16" else 10))
    absprod = np.abs(orc.decode(A_st, dtype)) @ np.abs(orc.logical_B(B_st, dtype, transB))
    to_boundary = ulp / 2 - np.abs(C - q)
    ambiguous = to_boundary <= tol * absprod + U_OUT["f32"] * np.abs(C) * 2
    return base + (ambiguous * ulp).sum(axis=1)


OFFLINE_SHAPES = [("bf16", 512, 512, 256, 0), ("bf16", 300, 520, 200, 1), ("bf16", 257, 130, 77, 0),
                  ("f16", 512, 256, 192, 1), ("f16", 100, 99, 50, 0),
                  ("f32", 256, 256, 256, 0), ("f32", 131, 67, 33, 1), ("f64", 200, 260, 70, 0), ("bf16", 1, 1, 1, 0)]


@pytest.mark.parametrize("dtype,M,N,K,transB", OFFLINE_SHAPES)
def test_offline_check_parity(dtype, M, N, K, transB):
    for seed, dist in ((31, "u_0_1"), (32, "n_1e-6_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        print(f"offline {dtype} {M}x{N}x{K} transB={transB} {dist}", flush=True)
        e_off = _emax_off(dtype, K, N)
        vg = _session(M, N, K, dtype, transB)
        vg.run_offline(_dev(A, dtype), _dev(B, dtype))
        r = vg.results()
        o = orc.verify(A, B, dtype, transB, e_max=e_off)
        if dtype in ("bf16", "f16"):  # 2 u_output on both sides; wide outputs keep the device-calibrated law
            assert e_off == orc.default_emax_offline(dtype, K, N)
        check_light(r, o, dtype, M, N, K)          # Be, statistics, expected, T (with the offline e_max)
        check_C(r, o, A, B, dtype, transB)
        rs_off = orc.row_sums_offline(o["C"], dtype)
        tol_rows = _offline_rowsum_tolerance(o, A, B, dtype, transB)
        assert np.all(np.abs(r["rowsum"] - rs_off) <= tol_rows), "offline rowsum"
        E_off = orc.verification_difference(o["expected"], rs_off)
        assert np.all(np.abs(r["E"] - E_off) <= tol_rows + _tol(dtype) * o["scale_expected"]), "offline E"
        assert not orc.fault_flags(E_off, o["T"]).any()
        assert r["nflag"] == 0 and not r["flags"].any()
        # property that holds at any size: the reported row sum is the sum of the stored elements
        stored = orc.decode(r["C"], dtype)
        assert np.all(np.abs(r["rowsum"] - stored.sum(axis=1)) <= 4 * U_OUT["f64" if dtype == "f64" else "f32"] *
                      np.abs(stored).sum(axis=1) + 1e-300)


def test_offline_exact_arithmetic_and_granularity():
    """Small-integer matrices: the stored product is exact, so the offline difference is exactly zero.  A
    planted error between the two thresholds is caught by the fused (accumulator-level) check and passes the
    offline one: the granularity gap of section 3.6."""
    dtype, M, N, K, transB = "bf16", 512, 512, 128, 0
    g = wl.rng(41, 0)
    A = wl.to_storage(g.integers(-1, 2, size=(M, K)).astype(np.float64), dtype)
    B = wl.to_storage(g.integers(-1, 2, size=(K, N)).astype(np.float64), dtype)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    vg.run_offline(dA, dB)
    r = vg.results()
    o_off = orc.verify(A, B, dtype, transB, e_max=_emax_off(dtype, K, N))
    assert np.array_equal(r["rowsum"].astype(np.float64), orc.row_sums_offline(o_off["C"], dtype))
    assert not r["E"].any() and r["nflag"] == 0
    # a flip of the top mantissa bit of an element equal to +-1: |delta| = 0.5
    from paper_2602_08043_amd import binding as vb
    o_on = orc.verify(A, B, dtype, transB, e_max=vb.vabft_default_emax(dtype, K, N))
    i = 77
    j = int(np.argmax(np.abs(o_on["C"][i]) == 1))  # |C| = 1: the flip moves it by 0.5
    delta = abs(orc.bitflip(o_on["C"][i, j], 22, np.float32) - o_on["C"][i, j])
    assert 10 * o_on["T"][i] < delta < 0.1 * o_off["T"][i], (o_on["T"][i], delta, o_off["T"][i])
    inj = vg.make_inject(mode=1, faults=[(i, j, 22)])
    vg.run_fused(dA, dB, inj=inj)
    assert vg.results()["flags"][i] == 1                      # fused check, FP32-level e_max
    vg.run_offline(dA, dB, inj=inj)
    r_off = vg.results()
    assert r_off["nflag"] == 0                                 # same error, offline e_max: passes
    assert abs(abs(float(r_off["E"][i])) - delta) <= 1e-6 * delta
    # a large error (exponent MSB: +-1 becomes +-inf) is caught by both
    inj = vg.make_inject(mode=1, faults=[(i, j, 30)])
    vg.run_offline(dA, dB, inj=inj)
    r_big = vg.results()
    assert r_big["flags"][i] == 1 and r_big["nflag"] == 1 and r_big["flags"].sum() == 1


def test_offline_check_of_a_product_computed_elsewhere():
    """The check takes any stored product: here torch.matmul's BF16 result, then the same with one element
    overwritten."""
    dtype, M, N, K = "bf16", 1024, 768, 512
    A, B = _gen(dtype, M, N, K, 0, 51, "n_1_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    C = torch.matmul(dA, dB)
    e_off = _emax_off(dtype, K, N)
    vg = _session(M, N, K, dtype, 0)
    vg.encode(dB)
    vg.threshold(dA, e_off)
    vg.check_offline(C)
    r = vg.results()
    o = orc.verify(A, B, dtype, 0, e_max=e_off)
    assert r["nflag"] == 0
    stored = C.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(r["rowsum"] - stored.sum(axis=1)) <= 4 * U_OUT["f32"] * np.abs(stored).sum(axis=1))
    assert np.all(np.abs(r["E"]) <= o["T"])
    C[5, 700] = C[5, 700] + 4.0 * float(o["T"][5])
    vg.check_offline(C)
    r = vg.results()
    assert r["flags"][5] == 1 and r["nflag"] == 1


def test_offline_argument_errors():
    from paper_2602_08043_amd import binding as vb
    vg = _session(64, 64, 64, "f32", 0)
    assert vb.vabft_check_offline(vg.problem, None, vg.expected.data_ptr(), vg.T.data_ptr(), vg.rowsum.data_ptr(),
                                  vg.E.data_ptr(), vg.flags.data_ptr(), vg.nflag.data_ptr(), None,
                                  check=False) == vb.VABFT_EINVAL
    assert vb.vabft_check_offline(vg.problem, vg.C.data_ptr(), vg.expected.data_ptr(), vg.T.data_ptr(),
                                  vg.rowsum.data_ptr(), vg.E.data_ptr(), vg.flags.data_ptr(), None, None,
                                  check=False) == vb.VABFT_EINVAL
    assert vb.vabft_default_emax_offline("bf16", 10, 10) == 2.0 ** -7
    assert vb.vabft_default_emax_offline("f16", 10, 10) == 2.0 ** -10
    assert vb.vabft_default_emax_offline("f64", 300, 200) == vb.vabft_default_emax("f64", 300, 200)
