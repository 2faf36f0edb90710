"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Tolerances (written from the arithmetic):
  FP32 accumulation: 1e-5 x (sum of absolute values of the terms of the quantity)
  FP64 accumulation: 1e-12 x the same scale
  max / min: exact.  Flags: exact.  Injection records: exact (set of (row, col, bit),
  after == bitflip(before)).
"""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

U_OUT = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24, "f64": 2.0 ** -53}
# largest magnitude that still rounds to a finite value of the output type
# smallest positive (subnormal) value of the output type: absolute rounding error near zero
OUT_TINY = {"bf16": 2.0 ** -133, "f16": 2.0 ** -24, "f32": 2.0 ** -149, "f64": 5e-324}
OUT_MAX = {"bf16": 3.38e38, "f16": 65504.0, "f32": 3.4e38, "f64": 1.79e308}


def _emax(dtype, K, N):
    """The library's default e_max (a parameter of Algorithm 1; the oracle is given the same value)."""
    from paper_2602_08043_amd import binding as vb
    return vb.vabft_default_emax(dtype, K, N)


def _tol(dtype):
    return 1e-12 if dtype == "f64" else 1e-5


def _session(M, N, K, dtype, transB, **kw):
    from paper_2602_08043_amd.session import VerifiedGemm
    return VerifiedGemm(M, N, K, dtype, transB, **kw)


def _dev(x, dtype):
    from paper_2602_08043_amd.session import to_device
    return to_device(x, dtype)


def _gen(dtype, M, N, K, transB, seed, dist="n_1e-6_1"):
    g = wl.rng(seed, 9)
    A = wl.to_storage(wl.paper_distribution(g, dist, (M, K)), dtype)
    Bl = wl.paper_distribution(g, dist, (K, N))
    B = wl.to_storage(np.ascontiguousarray(Bl.T) if transB else Bl, dtype)
    return A, B


def check_light(r, o, dtype, M, N, K):
    """Everything the oracle computes in O(MK + KN)."""
    tol = _tol(dtype)
    tiny = 1e-300
    assert np.all(np.abs(r["Be"] - o["Be"]) <= tol * o["scale_Be"] + tiny), "Be"
    assert np.array_equal(r["bstat"][:, 0].astype(np.float64), o["bstat"][:, 0]), "B row max"
    assert np.array_equal(r["bstat"][:, 1].astype(np.float64), o["bstat"][:, 1]), "B row min"
    assert np.all(np.abs(r["bstat"][:, 2] - o["bstat"][:, 2]) <= tol * o["scale_Be"] / N + tiny), "B row mean"
    assert np.array_equal(r["astat"][:, 0].astype(np.float64), o["astat"][:, 0]), "A row max"
    assert np.array_equal(r["astat"][:, 1].astype(np.float64), o["astat"][:, 1]), "A row min"
    # S1 = sum|mu|, S2 = sum var, S3 = sum mu^2: errors come from the rounded row sums of B
    mean_abs = o["scale_Be"] / N
    mu = o["bstat"][:, 2]
    span = o["bstat"][:, 0] - o["bstat"][:, 1]
    dS = np.abs(r["S"] - o["S"])
    assert dS[0] <= tol * mean_abs.sum() + tiny, "S1"
    assert dS[1] <= tol * (span * mean_abs).sum() + 1e-12 * o["S"][1] + tiny, "S2"
    assert dS[2] <= tol * (2 * np.abs(mu) * mean_abs + mean_abs ** 2 * tol).sum() + tiny, "S3"
    assert np.all(np.abs(r["expected"] - o["expected"]) <= tol * o["scale_expected"] + tiny), "expected"
    assert np.all(np.abs(r["T"] - o["T"]) <= max(tol, 2e-7 if dtype != "f64" else 0) * o["T"] + tiny), "T"


def check_rows(r, o, dtype, rows=None):
    """Quantities that need the product: C, row sums, E (on the rows the oracle holds)."""
    tol = _tol(dtype)
    sel = slice(None) if rows is None else rows
    scale = o["scale_rowsum"][sel]
    assert np.all(np.abs(r["rowsum"][sel] - o["rowsum"]) <= tol * scale + 1e-300), "rowsum"
    assert np.all(np.abs(r["E"][sel] - o["E"]) <= 2 * tol * scale + 1e-300), "E"
    if not o["flags"].any():  # (o["flags"], like o["E"], covers the selected rows only)
        # A bound that still means something at full size, where the K-scaled tolerance above is orders of
        # magnitude wider than the threshold: on fault-free rows both differences are rounding noise, and the
        # threshold of the row (the paper's own bound on that noise) bounds how far apart they can be.
        assert np.all(np.abs(r["E"][sel] - o["E"]) <= o["T"][sel]), "E against the row's threshold"


def check_C(r, o, A_st, B_st, dtype, transB, rows=None):
    from oracle.vabft_oracle import decode, logical_B
    sel = slice(None) if rows is None else rows
    C = orc.decode(r["C"], dtype)[sel]
    absprod = np.abs(decode(A_st, dtype)[sel]) @ np.abs(logical_B(B_st, dtype, transB))
    bound = U_OUT[dtype] * np.abs(o["C"]) + _tol(dtype) * absprod + 1e-300
    assert np.all(np.abs(C - o["C"]) <= bound), "C"


SMALL = [
    # dtype, M, N, K, transB
    ("bf16", 512, 512, 256, 0), ("bf16", 512, 512, 256, 1),
    ("bf16", 300, 520, 200, 0), ("bf16", 300, 520, 200, 1),
    ("bf16", 257, 130, 77, 0), ("bf16", 257, 130, 77, 1),
    ("f16", 512, 256, 192, 0), ("f16", 300, 520, 200, 1), ("f16", 100, 99, 50, 0),
    ("f32", 256, 256, 256, 0), ("f32", 256, 256, 256, 1), ("f32", 200, 260, 70, 0), ("f32", 131, 67, 33, 1),
    ("f64", 256, 384, 128, 0), ("f64", 256, 128, 64, 1), ("f64", 200, 260, 70, 0), ("f64", 131, 67, 33, 1),
    ("bf16", 1, 1, 1, 0), ("f32", 1, 1, 1, 0), ("f64", 3, 2, 1, 1), ("f16", 2, 300, 5, 1),
]


@pytest.mark.parametrize("dtype,M,N,K,transB", SMALL)
def test_fault_free_parity_small(dtype, M, N, K, transB):
    for seed, dist in ((1, "n_1e-6_1"), (2, "n_1_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        print(f"case {dtype} {M}x{N}x{K} transB={transB} seed={seed} {dist}", flush=True)
        vg = _session(M, N, K, dtype, transB)
        vg.run(_dev(A, dtype), _dev(B, dtype))
        r = vg.results()
        o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
        check_light(r, o, dtype, M, N, K)
        check_rows(r, o, dtype)
        check_C(r, o, A, B, dtype, transB)
        assert not o["flags"].any()
        assert not r["flags"].any() and r["nflag"] == 0
        assert np.all(np.abs(r["E"]) <= r["T"])


@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 512, 512, 0), ("f16", 512, 256, 384, 1),
                                                 ("f32", 256, 128, 512, 0), ("f64", 256, 128, 64, 1),
                                                 ("f64", 384, 384, 384, 0)])
def test_no_false_positive_on_positive_matrices(dtype, M, N, K, transB):
    """|N(1,1)| inputs (the calibration protocol's matrices, section 3.6): no cancellation, so the
    relative verification difference is at its largest; the default e_max must still clear it."""
    for seed in range(6):
        A, B = _gen(dtype, M, N, K, transB, 40 + seed, "abs_n_1_1")
        vg = _session(M, N, K, dtype, transB)
        vg.run_fused(_dev(A, dtype), _dev(B, dtype))
        r = vg.results()
        assert r["nflag"] == 0 and not r["flags"].any(), (seed, float((np.abs(r["E"]) / r["T"]).max()))
        o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
        check_light(r, o, dtype, M, N, K)
        check_rows(r, o, dtype)


@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 768, 256, 0), ("f16", 300, 520, 200, 1),
                                                 ("f32", 256, 256, 256, 0), ("f64", 200, 260, 70, 1)])
def test_plain_gemm_matches_verified(dtype, M, N, K, transB):
    """verify=0 is the same product (bit-identical C) with no check outputs touched."""
    A, B = _gen(dtype, M, N, K, transB, 5)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    vg.run(dA, dB)
    C1 = vg.results()["C"].copy()
    vg.C.zero_()
    vg.rowsum.fill_(123.0)
    vg.gemm(dA, dB, verify=0)
    r = vg.results()
    assert np.array_equal(r["C"], C1)
    assert np.all(r["rowsum"] == 123.0)


FUSED = [
    # whole-tile 16-bit problems: statistics and compare/flag inside the GEMM kernel
    ("bf16", 512, 512, 256, 0), ("bf16", 512, 768, 384, 1), ("f16", 256, 1024, 512, 0), ("f16", 768, 512, 128, 1),
    ("bf16", 256, 512, 1152, 0),
    # everything else: the two passes back to back behind the same entry point
    ("bf16", 512, 256, 256, 0), ("bf16", 512, 512, 192, 0), ("bf16", 300, 520, 200, 1), ("f16", 100, 99, 50, 0),
    ("f32", 256, 256, 256, 0), ("f64", 200, 260, 70, 1),
    # a single k-tile (the whole-tile GEMM's loop runs one body, whose loads of a next tile re-read the only one)
    ("bf16", 256, 256, 64, 0), ("f16", 256, 512, 64, 1),
    # whole-tile FP32 / FP64 problems: the same in-kernel path on the 128 x 128 tile kernels, with a k-tile count
    # that is not a multiple of the tile-columns, and with more tile-columns than k-tiles (some fold nothing)
    ("f32", 384, 512, 272, 1), ("f32", 128, 512, 32, 0), ("f32", 128, 128, 16, 0), ("f64", 256, 384, 128, 0),
    ("f64", 256, 128, 64, 1), ("f64", 128, 640, 48, 1),
]


@pytest.mark.parametrize("dtype,M,N,K,transB", FUSED)
def test_fused_entry_point_parity(dtype, M, N, K, transB):
    """vabft_gemm_verified_fused against the oracle, twice in a row on the same workspace
    (arrival counters must come back to zero), then against the three-call route."""
    for seed, dist in ((11, "n_1e-6_1"), (12, "n_1_1"), (13, "u_-1_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        print(f"fused case {dtype} {M}x{N}x{K} transB={transB} seed={seed} {dist}", flush=True)
        dA, dB = _dev(A, dtype), _dev(B, dtype)
        vg = _session(M, N, K, dtype, transB)
        o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
        for rep in range(2):
            vg.rowsum.fill_(7.0)
            vg.T.fill_(-1.0)
            vg.run_fused(dA, dB)
            r = vg.results()
            check_light(r, o, dtype, M, N, K)
            check_rows(r, o, dtype)
            check_C(r, o, A, B, dtype, transB)
            assert np.array_equal(r["astat"][:, 0].astype(np.float64), o["astat"][:, 0])
            assert np.array_equal(r["astat"][:, 1].astype(np.float64), o["astat"][:, 1])
            assert np.all(np.abs(r["astat"][:, 2] - o["astat"][:, 2]) <= _tol(dtype) * np.abs(orc.decode(A, dtype)).mean(axis=1) + 1e-300)
            assert not r["flags"].any() and r["nflag"] == 0
        # same C bit for bit, same flags, as the three-call route
        C_fused = r["C"].copy()
        vg.run(dA, dB)
        r3 = vg.results()
        assert np.array_equal(r3["C"], C_fused)
        assert np.array_equal(r3["rowsum"], r["rowsum"])
        assert np.allclose(r3["T"], r["T"], rtol=2e-6 if dtype != "f64" else 1e-12, atol=0)
    # one exponent flip through the fused call
    i, j = M // 2, N // 3
    bit = 61 if dtype == "f64" else 29
    inj = vg.make_inject(mode=1, faults=[(i, j, bit)])
    vg.run_fused(dA, dB, inj=inj)
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == 1 and recs[0][:3] == (i, j, bit)
    assert r["flags"][i] == 1 and r["nflag"] == 1 and r["flags"].sum() == 1
    # and the counters are clean again afterwards
    vg.run_fused(dA, dB)
    assert vg.results()["nflag"] == 0


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32", "f64"])
@pytest.mark.parametrize("transB", [0, 1])
def test_exact_arithmetic_gives_zero_difference(dtype, transB):
    """Entries in {-1, 0, 1}: every product and partial sum is an exactly representable
    integer, so C e == A (B e) bit for bit and E is exactly zero (section 2.2 identity)."""
    M, N, K = 384, 520, 320
    g = wl.rng(17, transB)
    A = wl.to_storage(g.integers(-1, 2, size=(M, K)).astype(np.float64), dtype)
    Bl = g.integers(-1, 2, size=(K, N)).astype(np.float64)
    B = wl.to_storage(np.ascontiguousarray(Bl.T) if transB else Bl, dtype)
    vg = _session(M, N, K, dtype, transB)
    vg.run(_dev(A, dtype), _dev(B, dtype))
    r = vg.results()
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    assert np.array_equal(r["Be"].astype(np.float64), o["Be"])
    assert np.array_equal(r["expected"].astype(np.float64), o["expected"])
    assert np.array_equal(r["rowsum"].astype(np.float64), o["rowsum"])
    assert not r["E"].any()
    assert np.array_equal(orc.decode(r["C"], dtype), o["C"])
    assert r["nflag"] == 0


def _acc_np(dtype):
    return np.float64 if dtype == "f64" else np.float32


@pytest.mark.parametrize("dtype,M,N,K,transB", [("f32", 256, 256, 256, 0), ("bf16", 300, 520, 200, 1),
                                                 ("bf16", 512, 512, 128, 0), ("f16", 257, 130, 77, 0),
                                                 ("f64", 200, 260, 70, 0)])
def test_explicit_bit_flips(dtype, M, N, K, transB):
    """Config-1 style runs: one seeded single-bit flip per run in the accumulator."""
    A, B = _gen(dtype, M, N, K, transB, 0, "n_1e-6_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    vg.run(dA, dB)
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    acc = _acc_np(dtype)
    nbits = 64 if dtype == "f64" else 32
    hi_bits = list(range(52, 63)) if dtype == "f64" else list(range(20, 31))
    g = wl.rng(99, 3)
    for run in range(8):
        i, j = int(g.integers(0, M)), int(g.integers(0, N))
        bit = int(g.choice(hi_bits))
        print(f"flip run {run}: ({i},{j}) bit {bit}", flush=True)
        inj = vg.make_inject(mode=1, faults=[(i, j, bit)])
        vg.gemm(dA, dB, 1, inj)
        r = vg.results()
        n, recs = vg.inject_records()
        assert n == 1 and recs[0][:3] == (i, j, bit)
        before, after = recs[0][3], recs[0][4]
        assert after == orc.bitflip(before, bit, acc) or (np.isnan(after) and np.isnan(orc.bitflip(before, bit, acc)))
        assert abs(before - o["C"][i, j]) <= _tol(dtype) * (np.abs(orc.decode(A, dtype)[i]) @ np.abs(orc.logical_B(B, dtype, transB)[:, j])) + 1e-300
        # the corrupted value is what C receives
        Cij = orc.decode(r["C"], dtype)[i, j]
        if np.isfinite(after) and abs(after) < OUT_MAX[dtype]:
            assert abs(Cij - after) <= U_OUT[dtype] * abs(after) * 1.01 + OUT_TINY[dtype]
        else:
            assert not np.isfinite(Cij)
        rs = orc.replay_faults(o["rowsum"], recs)
        with np.errstate(invalid="ignore"):
            want = orc.fault_flags(orc.verification_difference(o["expected"], rs), o["T"])
        delta = abs(after - before)
        if not (delta < 10 * o["T"][i]):  # also true for inf / nan
            assert np.array_equal(r["flags"], want), (i, j, bit, before, after, o["T"][i])
            assert r["flags"][i] == 1 and r["nflag"] == 1
        others = np.delete(r["flags"], i)
        assert not others.any()
    # an out-of-range entry and an empty list are ignored
    inj = vg.make_inject(mode=1, faults=[(M + 5, 0, 3), (0, N, 3), (0, 0, nbits)])
    vg.gemm(dA, dB, 1, inj)
    assert vg.inject_records()[0] == 0 and vg.results()["nflag"] == 0


@pytest.mark.parametrize("dtype,M,N,K,transB,rate", [("f16", 512, 512, 128, 0, 2e-4), ("bf16", 300, 520, 200, 1, 1e-3),
                                                      ("f32", 200, 260, 70, 0, 1e-3), ("f64", 131, 67, 33, 1, 5e-3)])
def test_bernoulli_injector_matches_oracle_generator(dtype, M, N, K, transB, rate):
    A, B = _gen(dtype, M, N, K, transB, 4, "u_-1_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    vg.run(dA, dB)
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    acc = _acc_np(dtype)
    lo, hi = (40, 63) if dtype == "f64" else (16, 31)
    seed = 0xC0FFEE
    inj = vg.make_inject(mode=2, seed=seed, rate=rate, bit_lo=lo, bit_hi=hi)
    vg.gemm(dA, dB, 1, inj)
    r = vg.results()
    n, recs = vg.inject_records()
    want_set = orc.bernoulli_faults(seed, rate, lo, hi, M, N)
    assert n == len(want_set) > 0
    assert [rec[:3] for rec in recs] == sorted(want_set)
    for (_i, _j, bit, before, after) in recs:
        f = orc.bitflip(before, bit, acc)
        assert after == f or (np.isnan(after) and np.isnan(f))
    rs = orc.replay_faults(o["rowsum"], recs)
    with np.errstate(invalid="ignore"):
        want = orc.fault_flags(orc.verification_difference(o["expected"], rs), o["T"])
        # rows whose every fault is >= 10 T (or non-finite) must agree; rows without faults must be clean
        per_row = {}
        for (i, _j, _b, before, after) in recs:
            d = abs(after - before)
            per_row.setdefault(i, []).append(d)
    for i in range(M):
        if i not in per_row:
            assert r["flags"][i] == 0
        elif len(per_row[i]) == 1 and not (per_row[i][0] < 10 * o["T"][i]):
            assert r["flags"][i] == want[i] == 1
    assert r["nflag"] == int(r["flags"].sum())


def test_detection_rule_with_exact_arithmetic():
    """With small-integer inputs E is exactly the injected delta, so a flip is flagged
    iff |after - before| > T_i (the only pin available for detection by bit position)."""
    dtype, M, N, K = "bf16", 256, 256, 128
    g = wl.rng(31)
    A = wl.to_storage(g.integers(-2, 3, size=(M, K)).astype(np.float64), dtype)
    B = wl.to_storage(g.integers(-2, 3, size=(K, N)).astype(np.float64), dtype)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, 0)
    vg.run(dA, dB)
    T = vg.results()["T"].astype(np.float64)
    faults = [(int(g.integers(0, M)), int(g.integers(0, N)), bit) for bit in range(8, 31)]
    for f in faults:
        inj = vg.make_inject(mode=1, faults=[f])
        vg.gemm(dA, dB, 1, inj)
        r = vg.results()
        _n, recs = vg.inject_records()
        before, after = recs[0][3], recs[0][4]
        delta = abs(after - before)
        if np.isfinite(delta):
            # E = -(applied delta) up to the FP32 rounding of the corrupted row sum
            assert abs(float(r["E"][f[0]]) + (after - before)) <= 1e-5 * (abs(before) + abs(after) + 1.0)
        if not np.isfinite(delta) or abs(delta - T[f[0]]) > 1e-3 * T[f[0]]:
            assert r["flags"][f[0]] == int(not (delta <= T[f[0]]))


def test_argument_errors():
    from paper_2602_08043_amd import binding as vb
    vg = _session(64, 64, 64, "f32", 0)
    A = torch.zeros((64, 64), device="cuda")
    p = vb.make_problem(64, 64, 64, "f32")
    assert vb.vabft_encode(p, 0, vg.Be.data_ptr(), vg.bstat.data_ptr(), vg.S.data_ptr(), None, 0, None, check=False) == vb.VABFT_EINVAL
    bad = vb.make_problem(64, 64, 64, "f32", lda=10)
    assert vb.vabft_threshold(bad, A.data_ptr(), vg.Be.data_ptr(), vg.S.data_ptr(), 1e-6, 2.5, vg.astat.data_ptr(),
                              vg.expected.data_ptr(), vg.T.data_ptr(), None, check=False) == vb.VABFT_EINVAL
    assert vb.vabft_threshold(p, A.data_ptr(), vg.Be.data_ptr(), vg.S.data_ptr(), -1.0, 2.5, vg.astat.data_ptr(),
                              vg.expected.data_ptr(), vg.T.data_ptr(), None, check=False) == vb.VABFT_EINVAL
    # workspace too small
    rc = vb.vabft_gemm_verified(p, A.data_ptr(), A.data_ptr(), vg.C.data_ptr(), vg.expected.data_ptr(), vg.T.data_ptr(),
                                1, None, vg.rowsum.data_ptr(), vg.E.data_ptr(), vg.flags.data_ptr(), vg.nflag.data_ptr(),
                                None, None, vg.ws.data_ptr(), 8, None, check=False)
    assert rc == vb.VABFT_EWORKSPACE
    inj = vg.make_inject(mode=2, seed=1, rate=2.0, bit_lo=0, bit_hi=31)
    with pytest.raises(vb.VabftError):
        vg.gemm(A, A, 1, inj)
    with pytest.raises(vb.VabftError):
        vg.gemm(A, A, 0, vg.make_inject(mode=2, seed=1, rate=0.5, bit_lo=0, bit_hi=31))


# --------------------------------------------------------------------------
# full benchmark sizes, in the launch configuration bench.py times
# --------------------------------------------------------------------------
FULL = [("c2_bf16_4096", 0), ("c3_bf16_ffn", 0), ("c4_f16_8192", 0), ("c5_f64_2048", 0), ("c5_f64_2048", 1)]


@pytest.mark.parametrize("name,variant", FULL)
def test_full_size_sampled(name, variant):
    cfg = wl.make_config(name, seed=3, variant=variant)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    print(f"full {name} variant {variant}: {M}x{N}x{K} {dt} transB={tb}", flush=True)
    dA, dB = _dev(cfg["A"], dt), _dev(cfg["B"], dt)
    vg = _session(M, N, K, dt, tb)
    vg.run_fused(dA, dB)  # the launch configuration bench.py times
    r = vg.results()
    rows = np.sort(wl.rng(3, 77).choice(M, size=64, replace=False))
    # tile-boundary rows too
    rows = np.unique(np.concatenate([rows, [0, 255, 256, M - 1]]))
    o = orc.verify(cfg["A"], cfg["B"], dt, tb, e_max=_emax(dt, K, N), rows=rows)
    check_light(r, o, dt, M, N, K)
    check_rows(r, o, dt, rows)
    check_C(r, o, cfg["A"], cfg["B"], dt, tb, rows)
    assert not r["flags"].any() and r["nflag"] == 0
    assert not o["flags"].any()
    assert np.all(np.abs(r["E"]) <= r["T"])
    # the three-call route at full size agrees too
    vg.run(dA, dB)
    r3 = vg.results()
    check_light(r3, o, dt, M, N, K)
    check_rows(r3, o, dt, rows)
    assert np.array_equal(r3["C"], r["C"]) and r3["nflag"] == 0
    # one exponent-bit flip at full size, replayed by the oracle on a sampled row
    i = int(rows[5])
    j = N - 3
    bit = 61 if dt == "f64" else 29
    inj = vg.make_inject(mode=1, faults=[(i, j, bit)])
    vg.gemm(dA, dB, 1, inj)
    r2 = vg.results()
    n, recs = vg.inject_records()
    assert n == 1 and recs[0][:3] == (i, j, bit)
    assert r2["flags"][i] == 1 and r2["nflag"] == 1
    assert r2["flags"].sum() == 1


# --------------------------------------------------------------------------
# degenerate inputs
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 512, 256, 0), ("bf16", 300, 200, 100, 1),
                                                 ("f32", 256, 128, 64, 0), ("f64", 130, 70, 40, 1)])
def test_constant_and_zero_matrices(dtype, M, N, K, transB):
    """Zero matrices: every statistic, checksum, threshold and difference is exactly zero and nothing is flagged
    (0 <= 0).  Constant matrices a, b: variances vanish, T = e_max N |a| K |b|, and with small-integer constants
    both checksum paths are exact."""
    for a, b in ((0.0, 0.0), (0.0, 3.0), (2.0, -0.5)):
        A = wl.to_storage(np.full((M, K), a), dtype)
        B = wl.to_storage(np.full((N, K) if transB else (K, N), b), dtype)
        vg = _session(M, N, K, dtype, transB)
        for route in ("run", "run_fused"):
            getattr(vg, route)(_dev(A, dtype), _dev(B, dtype))
            r = vg.results()
            e_max = _emax(dtype, K, N)
            assert np.all(r["Be"] == N * b) and np.all(r["expected"] == K * a * N * b)
            assert np.all(r["rowsum"] == K * a * N * b) and not r["E"].any()
            assert np.allclose(r["T"], e_max * N * abs(a) * K * abs(b), rtol=1e-6, atol=0)
            assert np.all(r["S"] == [K * abs(b), 0.0, K * b * b])
            assert r["nflag"] == 0 and not r["flags"].any()
            assert np.all(orc.decode(r["C"], dtype) == K * a * b)


@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 512, 256, 0), ("f16", 300, 200, 100, 1),
                                                 ("f32", 256, 128, 64, 0), ("f64", 130, 70, 40, 0)])
def test_nan_and_inf_inputs_flag_their_rows(dtype, M, N, K, transB):
    """A NaN or an infinity in a row of A poisons that row's checksums; `flag = !(|E| <= T)` flags it (the oracle
    agrees) and leaves the other rows alone.  A NaN in B poisons every row."""
    A, B = _gen(dtype, M, N, K, transB, 77, "n_1e-6_1")
    A = A.copy()
    nan_code = {"bf16": np.uint16(0x7FC0)}.get(dtype)
    inf_code = {"bf16": np.uint16(0x7F80)}.get(dtype)
    A[5, 7] = nan_code if nan_code is not None else np.nan
    A[M - 2, K - 1] = inf_code if inf_code is not None else np.inf
    vg = _session(M, N, K, dtype, transB)
    for route in ("run", "run_fused"):
        getattr(vg, route)(_dev(A, dtype), _dev(B, dtype))
        r = vg.results()
        with np.errstate(invalid="ignore", over="ignore"):
            o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
        assert o["flags"][5] == 1 and o["flags"][M - 2] == 1 and o["flags"].sum() == 2
        assert np.array_equal(r["flags"], o["flags"]) and r["nflag"] == 2
        ok = np.ones(M, dtype=bool)
        ok[[5, M - 2]] = False
        assert np.all(np.abs(r["E"][ok]) <= r["T"][ok])
    Bn = B.copy()
    Bn[3, 4] = nan_code if nan_code is not None else np.nan
    vg.run_fused(_dev(A, dtype), _dev(Bn, dtype))
    r = vg.results()
    assert r["nflag"] == M and r["flags"].all()


DEFERRED = [
    # single-launch kernels (the GEMM folds the partials in its prologue), both layouts of B
    ("bf16", 512, 512, 256, 0), ("f16", 768, 512, 128, 1), ("bf16", 256, 512, 1152, 0), ("f32", 384, 512, 272, 1),
    ("f32", 128, 128, 16, 0), ("f64", 256, 384, 128, 0), ("f64", 128, 640, 48, 1),
    # K over 4096: more partials than folding threads
    ("bf16", 256, 512, 4352, 0),
    # the passes back to back (a small kernel folds the partials first)
    ("bf16", 300, 520, 200, 1), ("f16", 100, 99, 50, 0), ("f32", 200, 260, 70, 0), ("f64", 131, 67, 33, 1),
    # row walks in which several wavefronts share a row of B (few rows, long rows), one with two wavefronts per row,
    # and one where the encode with the fold deferred runs its smaller workgroups (K >= 4096): the split of a row
    # into segments, and with it the bits of Be, must not depend on the route
    ("f64", 1024, 2048, 128, 0), ("f64", 256, 2048, 2048, 0), ("f32", 128, 4096, 4096, 0), ("f16", 256, 8192, 256, 0),
]


@pytest.mark.parametrize("dtype,M,N,K,transB", DEFERRED)
def test_deferred_fold_of_S_gives_the_same_bits(dtype, M, N, K, transB):
    """vabft_encode(d_S = NULL) + vabft_gemm_verified_fused(d_S = NULL): S1..S3 travel as per-workgroup partials and
    are folded by the consumer in the encode's own order, so thresholds, flags and everything else must equal the
    ordinary route bit for bit (Algorithm 1: S1, S2, S3 are plain sums over k)."""
    for seed, dist in ((21, "n_1e-6_1"), (22, "u_-1_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        dA, dB = _dev(A, dtype), _dev(B, dtype)
        vg = _session(M, N, K, dtype, transB)
        vg.run_fused(dA, dB)
        r0 = {k: np.copy(v) for k, v in vg.results().items()}
        o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
        check_light(r0, o, dtype, M, N, K)
        for rep in range(2):
            vg.S.fill_(float("nan"))  # the deferred route must not read it
            vg.T.fill_(-1.0)
            vg.expected.fill_(0.0)
            vg.flags.fill_(7)
            vg.run_fused(dA, dB, defer_S=True)
            r = vg.results()
            for key in ("T", "expected", "rowsum", "E", "flags", "astat", "C", "Be", "bstat"):
                assert np.array_equal(r[key], r0[key]), (key, rep)
            assert r["nflag"] == r0["nflag"] == 0
            assert np.isnan(r["S"]).all()
    # a fault through the deferred route
    i, j = M // 3, N // 2
    bit = 61 if dtype == "f64" else 29
    inj = vg.make_inject(mode=1, faults=[(i, j, bit)])
    vg.run_fused(dA, dB, inj=inj, defer_S=True)
    r = vg.results()
    assert r["flags"][i] == 1 and r["nflag"] == 1 and r["flags"].sum() == 1


def _random_shapes():
    """Seeded shapes: a mix of whole-tile problems (the single-launch kernels) and ragged ones (the guarded kernels
    and the passes of their own), both layouts of B, every floating-point type of the paper's table."""
    g = np.random.default_rng(20260208)
    cases = []
    for dtype, tile, kstep in (("bf16", 256, 128), ("f16", 256, 128), ("f32", 128, 16), ("f64", 128, 16)):
        for whole in (True, True, False, False, False):
            if whole:
                M, N = tile * int(g.integers(1, 4)), tile * int(g.integers(1, 4))
                K = kstep * int(g.integers(1, 6))
            else:
                M, N, K = (int(g.integers(1, 420)) for _ in range(3))
            cases.append((dtype, M, N, K, int(g.integers(0, 2)), int(g.integers(0, 1 << 30))))
    return cases


@pytest.mark.parametrize("dtype,M,N,K,transB,seed", _random_shapes())
def test_random_shapes_every_main_route(dtype, M, N, K, transB, seed):
    """The three-call route, the fused call and the fused call with the deferred fold against the oracle on seeded
    random shapes, a planted exponent flip through each, and clean counters afterwards."""
    print(f"random case {dtype} {M}x{N}x{K} transB={transB} seed={seed}", flush=True)
    A, B = _gen(dtype, M, N, K, transB, seed, "n_1_1" if seed & 1 else "n_1e-6_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    assert not o["flags"].any()
    i, j = (seed >> 3) % M, (seed >> 11) % N
    bit = 62 if dtype == "f64" else 30
    routes = (lambda inj=None: vg.run(dA, dB, inj=inj), lambda inj=None: vg.run_fused(dA, dB, inj=inj),
              lambda inj=None: vg.run_fused(dA, dB, inj=inj, defer_S=True))
    for route in routes:
        vg.T.fill_(-1.0)
        vg.flags.fill_(3)
        route()
        r = vg.results()
        if route is not routes[2]:
            check_light(r, o, dtype, M, N, K)
        else:
            assert np.all(np.abs(r["T"] - o["T"]) <= max(_tol(dtype), 2e-7 if dtype != "f64" else 0) * o["T"] + 1e-300)
        check_rows(r, o, dtype)
        check_C(r, o, A, B, dtype, transB)
        assert not r["flags"].any() and r["nflag"] == 0
        assert np.all(np.abs(r["E"]) <= r["T"])
        route(vg.make_inject(mode=1, faults=[(i, j, bit)]))
        rf = vg.results()
        n, recs = vg.inject_records()
        assert n == 1 and recs[0][:3] == (i, j, bit)
        before, after = recs[0][3], recs[0][4]
        if abs(after - before) > 4 * o["T"][i]:  # a flip of a tiny value can stay under the threshold
            assert rf["flags"][i] == 1 and rf["nflag"] == 1 and rf["flags"].sum() == 1
        route()
        assert vg.results()["nflag"] == 0


@pytest.mark.parametrize("dtype,M,N,K,transB", [("bf16", 512, 512, 256, 0), ("f16", 300, 520, 200, 1),
                                                 ("f32", 256, 256, 64, 1), ("f64", 128, 256, 48, 0)])
@pytest.mark.parametrize("e_max,c_sigma", [(1e-6, 0.0), (3e-7, 1.0), (2e-5, 6.0)])
def test_caller_chosen_emax_and_csigma(dtype, M, N, K, transB, e_max, c_sigma):
    """e_max and c_sigma are parameters of Algorithm 1: with c_sigma = 0 only the deterministic term remains, and
    the thresholds scale linearly with e_max; every route takes the caller's values."""
    if dtype == "f64":
        e_max *= 1e-9
    A, B = _gen(dtype, M, N, K, transB, 61, "n_1_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    o = orc.verify(A, B, dtype, transB, e_max=e_max, c_sigma=c_sigma)
    rtol = max(_tol(dtype), 2e-7 if dtype != "f64" else 0)
    for route in ("three", "fused", "deferred"):
        vg.T.fill_(-1.0)
        if route == "three":
            vg.encode(dB)
            vg.threshold(dA, e_max, c_sigma)
            vg.gemm(dA, dB, 1)
        else:
            vg.encode(dB, defer_S=route == "deferred")
            vg.gemm_fused(dA, dB, e_max, c_sigma, deferred_S=route == "deferred")
        r = vg.results()
        assert np.all(np.abs(r["T"] - o["T"]) <= rtol * o["T"] + 1e-300), route
        assert np.array_equal(r["flags"], o["flags"]), route
        assert r["nflag"] == int(o["flags"].sum())
    if c_sigma == 0.0:
        # T = e_max N |mu_A| S1 exactly (section 3.4, deterministic term)
        mu = np.abs(o["astat"][:, 2])
        assert np.allclose(o["T"], e_max * N * mu * o["S"][0], rtol=1e-12)
