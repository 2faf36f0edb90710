"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each is chosen so that a plausible
mistake in the oracle (dropped term, wrong sign/index, transposed operand,
wrong constant) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc


# --------------------------------------------------------------------------
# storage decode / bit flips: IEEE identities
# --------------------------------------------------------------------------
def test_bf16_decode_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x4049, 0x0000, 0x3F00, 0x7F80], dtype=np.uint16)
    got = orc.decode(bits, "bf16")
    assert got.tolist() == [1.0, -2.0, 3.140625, 0.0, 0.5, math.inf]


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 (even) and 1+2^-7 (odd) -> 1.0;
    # 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even) -> 1+2^-6
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = orc.decode(wl.f32_to_bf16_bits(x), "bf16")
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


def test_bitflip_identities_fp32():
    f32 = np.float32
    assert orc.bitflip(1.0, 31, f32) == -1.0            # sign
    assert orc.bitflip(1.0, 23, f32) == 0.5             # exponent LSB 127 -> 126
    assert orc.bitflip(1.0, 30, f32) == math.inf        # exponent MSB: 0x7f800000
    assert orc.bitflip(2.0, 30, f32) == 0.0             # 0x40000000 -> 0
    assert orc.bitflip(1.0, 22, f32) == 1.5             # top mantissa bit
    assert orc.bitflip(1.0, 0, f32) == 1.0 + 2.0 ** -23
    # involution
    for bit in range(32):
        v = 0.7431
        w = orc.bitflip(orc.bitflip(v, bit, f32), bit, f32)
        assert w == float(np.float32(v))


def test_bitflip_identities_fp64():
    f64 = np.float64
    assert orc.bitflip(1.0, 63, f64) == -1.0
    assert orc.bitflip(1.0, 52, f64) == 0.5
    assert orc.bitflip(1.0, 62, f64) == math.inf
    assert orc.bitflip(1.0, 51, f64) == 1.5
    assert orc.bitflip(1.0, 0, f64) == 1.0 + 2.0 ** -52


# --------------------------------------------------------------------------
# counter-based generator: published vector
# --------------------------------------------------------------------------
def test_splitmix64_published_vector(golden_dir):
    lines = [l.strip() for l in open(os.path.join(golden_dir, "splitmix64_vector.txt")) if not l.startswith("#")]
    seed = int(lines[0].split()[1])
    want = [int(v) for v in lines[1:] if v]
    got = [orc.splitmix64_at(seed, i) for i in range(len(want))]
    assert got == want
    vec = orc._splitmix64_vec(seed, np.arange(len(want)))
    assert [int(v) for v in vec] == want


def test_bernoulli_faults_statistics_and_brute_force():
    M, N, rate = 64, 96, 0.01
    got = orc.bernoulli_faults(7, rate, 16, 30, M, N)
    # brute force through the scalar generator
    lim = orc.bernoulli_hit_limit(rate)
    want = []
    for e in range(M * N):
        z = orc.splitmix64_at(7, e)
        if (z >> 11) < lim:
            want.append((e // N, e % N, 16 + (z & 0x7FF) % 15))
    assert got == want
    # hit count is Binomial(M*N, rate): within 5 sigma
    n = M * N
    assert abs(len(got) - n * rate) < 5 * math.sqrt(n * rate)
    assert all(16 <= b <= 30 for (_, _, b) in got)


# --------------------------------------------------------------------------
# section 2.2: brute-force integer identities on tiny matrices
# --------------------------------------------------------------------------
def _brute_gemm(A, B):
    M, K = len(A), len(A[0])
    N = len(B[0])
    return [[sum(A[i][k] * B[k][j] for k in range(K)) for j in range(N)] for i in range(M)]


def test_gemm_and_checksum_identity_brute_force():
    g = wl.rng(3)
    for (M, K, N) in [(1, 1, 1), (2, 3, 4), (5, 7, 3), (8, 8, 8), (3, 1, 6)]:
        A = g.integers(-9, 10, size=(M, K))
        B = g.integers(-9, 10, size=(K, N))
        Cb = _brute_gemm(A.tolist(), B.tolist())
        C = orc.gemm(A.astype(np.float64), B.astype(np.float64))
        assert C.tolist() == [[float(v) for v in r] for r in Cb]
        # non-square shapes catch a transposed operand or a checksum over the wrong axis
        Be = orc.encode_checksum(B.astype(np.float64))
        assert Be.tolist() == [float(sum(r)) for r in B.tolist()]
        exp = orc.expected_checksum(A.astype(np.float64), Be)
        rs = orc.row_sums(C)
        assert rs.tolist() == [float(sum(r)) for r in Cb]
        # C e == A (B e) exactly in integer arithmetic
        assert exp.tolist() == rs.tolist()
        E = orc.verification_difference(exp, rs)
        assert not E.any()


def test_sign_of_verification_difference_and_flag_rule():
    exp = np.array([10.0, 10.0, 10.0, 10.0, 10.0])
    rs = np.array([9.0, 11.0, 10.5, np.nan, np.inf])
    E = orc.verification_difference(exp, rs)
    assert E[0] == 1.0 and E[1] == -1.0            # E = checksum - rowsum
    T = np.full(5, 0.75)
    f = orc.fault_flags(E, T)
    assert f.tolist() == [1, 1, 0, 1, 1]           # NaN / Inf rows are flagged
    # boundary: |E| == T is not a fault (strict '>')
    assert orc.fault_flags(np.array([0.75, -0.75]), np.array([0.75, 0.75])).tolist() == [0, 0]


def test_transB_layout():
    g = wl.rng(5)
    B = g.normal(size=(6, 9)).astype(np.float32)
    assert np.array_equal(orc.logical_B(B, "f32", 0), B.astype(np.float64))
    assert np.array_equal(orc.logical_B(np.ascontiguousarray(B.T), "f32", 1), B.astype(np.float64))


# --------------------------------------------------------------------------
# section 3.5: extrema-variance theorem
# --------------------------------------------------------------------------
def test_extrema_variance_theorem_holds_and_is_tight():
    g = wl.rng(11)
    for dist in ("n_1_1", "u_-1_1", "trunc_n_0_1", "n_1e-6_1"):
        X = wl.paper_distribution(g, dist, (64, 257))
        mx, mn, mu = orc.row_stats(X)
        bound = orc.extrema_variance(mx, mn, mu)
        true_var = X.var(axis=1)  # population variance, as in the theorem
        assert np.all(true_var <= bound * (1 + 1e-12))
    # equality: half the entries at l, half at m
    row = np.array([[-3.0] * 8 + [5.0] * 8])
    mx, mn, mu = orc.row_stats(row)
    assert orc.extrema_variance(mx, mn, mu)[0] == 16.0 == row.var()
    # constant row -> 0 ; asymmetric two-point row: p(1-p)(m-l)^2
    row = np.array([[2.5] * 10])
    assert orc.extrema_variance(*orc.row_stats(row))[0] == 0.0
    row = np.array([[0.0] * 3 + [4.0] * 1])
    assert orc.extrema_variance(*orc.row_stats(row))[0] == pytest.approx(0.25 * 0.75 * 16.0)
    # a mean rounded outside [min, max] must not give a negative variance
    assert orc.extrema_variance(np.array([1.0]), np.array([1.0]), np.array([1.0 + 1e-16]))[0] == 0.0


# --------------------------------------------------------------------------
# section 3.4 / Algorithm 1: closed forms of the threshold
# --------------------------------------------------------------------------
def test_threshold_closed_form_constant_matrices():
    # sigma_A = sigma_B = 0: only the deterministic term survives
    M, K, N = 3, 5, 7
    A = np.full((M, K), -2.0)
    B = np.full((K, N), 0.5)
    T = orc.threshold(A, B, e_max=1e-3, c_sigma=2.5)
    assert np.allclose(T, 1e-3 * N * 2.0 * K * 0.5, rtol=1e-15)


def test_threshold_closed_form_two_point_zero_mean():
    # rows of A and B half -a / +a, half -b / +b: mu = 0, sigma^2 = a^2, b^2
    # -> only the interaction term: c_sigma sqrt(N) a sqrt(K b^2)
    M, K, N = 2, 8, 6
    a, b = 3.0, 0.5
    A = np.tile(np.array([a, -a] * (K // 2)), (M, 1))
    B = np.tile(np.array([b, -b] * (N // 2)), (K, 1))
    T = orc.threshold(A, B, e_max=2.0, c_sigma=2.5)
    assert np.allclose(T, 2.0 * 2.5 * math.sqrt(N) * a * math.sqrt(K * b * b), rtol=1e-15)


def test_threshold_closed_form_mixed_terms():
    # A row two-point {0, 2} (mu=1, var=1); B rows two-point {1, 3} (mu=2, var=1)
    K, N = 4, 10
    A = np.array([[0.0, 2.0, 0.0, 2.0]])
    B = np.tile(np.array([1.0, 3.0] * (N // 2)), (K, 1))
    S1, S2, S3 = orc.b_aggregates(B)
    assert (S1, S2, S3) == (8.0, 4.0, 16.0)
    t_det, t23, t4 = orc.threshold_terms(A, B, c_sigma=2.0)
    assert t_det[0] == N * 1.0 * 8.0
    assert t23[0] == pytest.approx(2.0 * math.sqrt(N * 1.0 * 4.0 + N * N * 1.0 * 16.0))
    assert t4[0] == pytest.approx(2.0 * math.sqrt(N) * 1.0 * 2.0)
    # the three terms are weighted equally by e_max and c_sigma enters terms 2-4 only
    T1 = orc.threshold(A, B, 1.0, 2.0)[0]
    T2 = orc.threshold(A, B, 1.0, 4.0)[0]
    assert T2 - T1 == pytest.approx(t23[0] + t4[0])


def test_threshold_rectangular_uses_N_of_B_and_K_sums():
    # distinguishes N from K and rows-of-B statistics from columns-of-B statistics
    K, N = 3, 5
    A = np.array([[1.0, 1.0, 1.0]])
    B = np.arange(K * N, dtype=np.float64).reshape(K, N)  # row k: 5k..5k+4, mean 5k+2
    T = orc.threshold(A, B, 1.0, 2.5)[0]
    assert T == pytest.approx(N * 1.0 * (2 + 7 + 12) + 2.5 * math.sqrt(N * 1.0 * 3 * 4.0))


def _read_table(golden_dir, which):
    rows = []
    for line in open(os.path.join(golden_dir, "paper_tightness_tables.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t, n, act, thr, tight = line.split()
        if t == which:
            rows.append((int(n), float(act), float(thr), float(tight)))
    return rows


def test_threshold_bf16_table_closed_form(golden_dir):
    # U(0,1) with ideal statistics (mu=1/2, max=1, min=0) has a closed form:
    # T = e_max (n^2/4 + 2.5 sqrt(n^2/16 + n^3/16) + 2.5 n/4)
    for n, _act, thr, _tight in _read_table(golden_dir, "bf16"):
        closed = 8e-3 * (n * n / 4 + 2.5 * math.sqrt(n * n / 16 + n ** 3 / 16) + 0.625 * n)
        assert closed == pytest.approx(thr, rel=0.01)


@pytest.mark.parametrize("table,dist,stype,trials", [("bf16", "u_0_1", "bf16", 4), ("fp32", "u_-1_1", "f32", 6),
                                                    ("fp64", "u_-1_1", "f64", 6)])
def test_threshold_reproduces_paper_tables(golden_dir, table, dist, stype, trials):
    """Row-mean V-ABFT threshold of the oracle on fresh matrices vs the value the
    paper prints, for all five sizes of each tightness table."""
    for n, _act, thr, _tight in _read_table(golden_dir, table):
        vals = []
        for t in range(trials):
            g = wl.rng(1000 + t, n)
            A = wl.to_storage(wl.paper_distribution(g, dist, (n, n)), stype)
            B = wl.to_storage(wl.paper_distribution(g, dist, (n, n)), stype)
            if table == "bf16":
                e_max = 8e-3
            else:
                e_max = orc.default_emax(stype, n, n)
            T = orc.threshold(orc.decode(A, stype), orc.decode(B, stype), e_max)
            vals.append(T.mean())
        got = float(np.mean(vals))
        tol = 0.05 if n == 128 else 0.03
        assert got == pytest.approx(thr, rel=tol), (table, n, got, thr)


def test_default_emax_table_values():
    assert orc.default_emax("f32", 1024, 1024) == pytest.approx(5.0e-9 * 32 + 1.2e-7)
    assert orc.default_emax("bf16", 4096, 4096) == pytest.approx(4.4e-7)
    assert orc.default_emax("f16", 8192, 8192) == orc.default_emax("f32", 8192, 8192)
    assert orc.default_emax("f64", 2048, 2048) == pytest.approx(1.0e-17 * math.sqrt(2048) + 2.5e-16)
    # rectangular: the larger accumulation depth
    assert orc.default_emax("bf16", 4096, 11008) == orc.default_emax("bf16", 11008, 11008)


# --------------------------------------------------------------------------
# scaling laws that follow from the boxed formula
# --------------------------------------------------------------------------
def test_threshold_scaling_and_invariances():
    g = wl.rng(21)
    A = g.normal(0.3, 1.0, size=(9, 33))
    B = g.normal(-0.2, 2.0, size=(33, 17))
    T = orc.threshold(A, B, 1e-6)
    assert np.allclose(orc.threshold(A, B, 3e-6), 3 * T, rtol=1e-14)
    assert np.allclose(orc.threshold(-4.0 * A, B, 1e-6), 4 * T, rtol=1e-12)
    assert np.allclose(orc.threshold(A, 0.5 * B, 1e-6), 0.5 * T, rtol=1e-12)
    pn = g.permutation(17)
    assert np.allclose(orc.threshold(A, B[:, pn], 1e-6), T, rtol=1e-12)
    pk = g.permutation(33)
    assert np.allclose(orc.threshold(A[:, pk], B[pk, :], 1e-6), T, rtol=1e-12)
    # T_m depends on row m of A only
    A2 = A.copy()
    A2[0] *= 7
    T2 = orc.threshold(A2, B, 1e-6)
    assert np.allclose(T2[1:], T[1:], rtol=1e-14) and T2[0] == pytest.approx(7 * T[0])


# --------------------------------------------------------------------------
# the verification difference on a real CPU path: tightness band and zero FPR
# --------------------------------------------------------------------------
@pytest.mark.parametrize("stype,lo,hi", [("f32", 5.0, 25.0), ("f64", 5.0, 25.0)])
def test_tightness_band_cpu(stype, lo, hi):
    """mean T / mean |E| of the CPU accumulator-precision path on U(-1,1) lands in
    the band of the paper's FP32/FP64 tightness tables (7-20x printed; CPU BLAS
    accumulation orders differ, so the accepted band is 5-25x)."""
    for n in (128, 256, 512, 1024):
        ratios = []
        for t in range(3):
            g = wl.rng(50 + t, n)
            A = wl.to_storage(wl.uniform(g, (n, n)), stype)
            B = wl.to_storage(wl.uniform(g, (n, n)), stype)
            T = orc.threshold(orc.decode(A, stype), orc.decode(B, stype), orc.default_emax(stype, n, n))
            _, _, E = orc.accumulator_path(A, B, stype)
            assert np.all(np.abs(E) <= T)
            ratios.append(orc.tightness(T, E)[0])
        r = float(np.mean(ratios))
        assert lo <= r <= hi, (stype, n, r)


@pytest.mark.parametrize("stype", ["bf16", "f16", "f32", "f64"])
@pytest.mark.parametrize("dist", wl.PAPER_DISTRIBUTIONS)
def test_zero_false_positives_cpu(stype, dist):
    for t, (M, K, N) in enumerate([(96, 128, 160), (128, 1024, 256), (256, 256, 256)]):
        g = wl.rng(77 + t, wl.PAPER_DISTRIBUTIONS.index(dist))
        A = wl.to_storage(wl.paper_distribution(g, dist, (M, K)), stype)
        B = wl.to_storage(wl.paper_distribution(g, dist, (K, N)), stype)
        o = orc.verify(A, B, stype, 0)
        assert not o["flags"].any()                      # exact-path E is far below T
        _, _, E = orc.accumulator_path(A, B, stype)
        assert not orc.fault_flags(E, o["T"]).any()      # accumulator-precision path too


def test_replay_faults_flags_large_deltas_only():
    g = wl.rng(5)
    A = wl.to_storage(g.normal(size=(32, 64)), "f32")
    B = wl.to_storage(g.normal(size=(64, 48)), "f32")
    o = orc.verify(A, B, "f32")
    i, j = 7, 11
    before = float(np.float32(o["C"][i, j]))
    for bit, must_flag in [(30, True), (28, True), (2, False)]:
        after = orc.bitflip(before, bit, np.float32)
        rs = orc.replay_faults(o["rowsum"], [(i, j, bit, before, after)])
        f = orc.fault_flags(orc.verification_difference(o["expected"], rs), o["T"])
        assert f.sum() == (1 if must_flag else 0)
        if must_flag:
            assert f[i] == 1


# --------------------------------------------------------------------------
# position-weighted checksum, localisation, correction (section 2.2)
# --------------------------------------------------------------------------
def _brute_weighted(A, B):
    """Triple loops, straight from the definitions of r2, C^{r2} and C^{r2'}."""
    M, K, N = len(A), len(B), len(B[0])
    Be2 = [sum((n + 1) * B[k][n] for n in range(N)) for k in range(K)]
    C = [[sum(A[i][k] * B[k][j] for k in range(K)) for j in range(N)] for i in range(M)]
    exp2 = [sum(A[i][k] * Be2[k] for k in range(K)) for i in range(M)]
    rs2 = [sum((j + 1) * C[i][j] for j in range(N)) for i in range(M)]
    return np.array(Be2, float), np.array(C, float), np.array(exp2, float), np.array(rs2, float)


def test_weighted_checksum_matches_brute_force_and_identity():
    rng = np.random.Generator(np.random.Philox(key=[91, 1]))
    A = rng.integers(-6, 7, size=(5, 7)).astype(np.float64)
    B = rng.integers(-6, 7, size=(7, 6)).astype(np.float64)
    Be2, C, exp2, rs2 = _brute_weighted(A.tolist(), B.tolist())
    assert np.array_equal(orc.weight_vector(6), np.array([1, 2, 3, 4, 5, 6], float))
    assert np.array_equal(orc.encode_checksum_weighted(B), Be2)
    assert np.array_equal(orc.expected_checksum_weighted(A, Be2), exp2)
    assert np.array_equal(orc.row_sums_weighted(orc.gemm(A, B)), rs2)
    # C r2 == A (B r2) exactly for small integers; a weight vector starting at 0 or a
    # transposed operand breaks the first column / non-square case
    assert np.array_equal(exp2, rs2)
    # column 0 carries weight 1 (not 0): a matrix that is zero except column 0
    B0 = np.zeros((7, 6))
    B0[:, 0] = 1.0
    assert np.array_equal(orc.encode_checksum_weighted(B0), np.ones(7))
    # last column carries weight N
    BN = np.zeros((7, 6))
    BN[:, 5] = 1.0
    assert np.array_equal(orc.encode_checksum_weighted(BN), 6.0 * np.ones(7))


@pytest.mark.parametrize("j", [0, 1, 17, 30, 31])
@pytest.mark.parametrize("delta", [5.0, -3.0, 1024.0])
def test_single_error_is_localised_and_corrected_exactly(j, delta):
    rng = np.random.Generator(np.random.Philox(key=[91, 2]))
    A = rng.integers(-4, 5, size=(6, 9)).astype(np.float64)
    B = rng.integers(-4, 5, size=(9, 32)).astype(np.float64)
    C = orc.gemm(A, B)
    exp1 = orc.expected_checksum(A, orc.encode_checksum(B))
    exp2 = orc.expected_checksum_weighted(A, orc.encode_checksum_weighted(B))
    bad = C.copy()
    bad[3, j] += delta
    D1, D2 = orc.checksum_differences(exp1, orc.row_sums(bad), exp2, orc.row_sums_weighted(bad))
    # D1 = delta, D2 = w(j) delta with w(j) = j + 1 (the paper's two difference equations)
    assert D1[3] == delta and D2[3] == (j + 1) * delta
    assert np.all(np.delete(D1, 3) == 0) and np.all(np.delete(D2, 3) == 0)
    flags = orc.fault_flags(-D1, np.full(6, 0.5))
    loc = orc.localize(D1, D2, flags, 32)
    assert loc.tolist() == [-1, -1, -1, j, -1, -1]
    assert np.array_equal(orc.correct(bad, loc, D1), C)


def test_sign_conventions_of_differences():
    # D1 is post-computation minus pre-computed (= -E of the verification difference)
    exp1, rs1 = np.array([10.0]), np.array([13.0])
    exp2, rs2 = np.array([100.0]), np.array([112.0])
    D1, D2 = orc.checksum_differences(exp1, rs1, exp2, rs2)
    assert D1[0] == 3.0 and D2[0] == 12.0
    assert orc.verification_difference(exp1, rs1)[0] == -D1[0]
    assert orc.localize(D1, D2, np.array([1]), 8)[0] == 3  # 12 / 3 - 1


def test_localisation_refuses_what_is_not_a_single_error():
    N = 16
    one = np.array([1])
    # two errors of equal size in columns 2 and 5: ratio 4.5 -> between two columns
    D1, D2 = np.array([2.0]), np.array([3.0 + 6.0])
    assert orc.localize(D1, D2, one, N)[0] == orc.LOC_UNRESOLVED
    # ratio points beyond the last column / before the first
    assert orc.localize(np.array([1.0]), np.array([18.0]), one, N)[0] == orc.LOC_UNRESOLVED
    assert orc.localize(np.array([1.0]), np.array([0.0]), one, N)[0] == orc.LOC_UNRESOLVED
    # last and first column are fine
    assert orc.localize(np.array([1.0]), np.array([16.0]), one, N)[0] == 15
    assert orc.localize(np.array([-2.0]), np.array([-2.0]), one, N)[0] == 0
    # infinities / NaN from exponent-MSB flips
    assert orc.localize(np.array([np.inf]), np.array([np.inf]), one, N)[0] == orc.LOC_UNRESOLVED
    assert orc.localize(np.array([np.nan]), np.array([1.0]), one, N)[0] == orc.LOC_UNRESOLVED
    # a row that is not flagged is never touched
    assert orc.localize(np.array([5.0]), np.array([10.0]), np.array([0]), N)[0] == orc.LOC_NOT_FLAGGED
    # tolerance of the rounding: 0.25 accepted, 0.3 not
    assert orc.localize(np.array([4.0]), np.array([4.0 * 7.25]), one, N)[0] == 6
    assert orc.localize(np.array([4.0]), np.array([4.0 * 7.3]), one, N)[0] == orc.LOC_UNRESOLVED


def test_weighted_replay_matches_recomputation():
    rng = np.random.Generator(np.random.Philox(key=[91, 3]))
    C = rng.integers(-9, 10, size=(4, 12)).astype(np.float64)
    recs = [(1, 0, 23, C[1, 0], C[1, 0] + 8.0), (2, 11, 30, C[2, 11], -C[2, 11])]
    bad = C.copy()
    bad[1, 0] += 8.0
    bad[2, 11] = -C[2, 11]
    assert np.array_equal(orc.replay_faults_weighted(orc.row_sums_weighted(C), recs), orc.row_sums_weighted(bad))
    assert np.array_equal(orc.replay_faults(orc.row_sums(C), recs), orc.row_sums(bad))


def test_verify_reports_weighted_quantities():
    cfg = wl.make_config("c1_f32_256", seed=3, shape=(24, 40, 16))
    o = orc.verify(cfg["A"], cfg["B"], cfg["dtype"], cfg["transB"])
    A = orc.decode(cfg["A"], "f32")
    B = orc.logical_B(cfg["B"], "f32", cfg["transB"])
    w = np.arange(1, 41, dtype=np.float64)
    assert np.allclose(o["Be2"], (B * w).sum(axis=1), rtol=1e-13)
    assert np.allclose(o["expected2"], o["rowsum2"], rtol=0, atol=1e-9 * o["scale_rowsum2"].max())
    assert np.allclose(o["rowsum2"], ((A @ B) * w).sum(axis=1), rtol=1e-12, atol=1e-9)
    assert np.all(o["scale_rowsum2"] >= np.abs(o["rowsum2"]))


# --------------------------------------------------------------------------
# offline (post-quantisation) verification, section 3.6
# --------------------------------------------------------------------------
def test_quantize_known_values():
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.14159, 65520.0, 1e39, -0.0])
    assert orc.quantize(x, "bf16").tolist() == [1.0, 1.015625, 3.140625, 65536.0, math.inf, -0.0]
    y = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65519.9, 65520.0, 2.0 ** -25, 2.0 ** -24])
    assert orc.quantize(y, "f16").tolist() == [1.0, 1.0 + 2.0 ** -9, 65504.0, math.inf, 0.0, 2.0 ** -24]
    assert np.isnan(orc.quantize(np.array([np.nan]), "bf16")[0])
    z = np.array([1.0 + 2.0 ** -24, 1.0 + 3 * 2.0 ** -24, 0.1])
    assert orc.quantize(z, "f32").tolist() == [1.0, 1.0 + 2.0 ** -22, float(np.float32(0.1))]
    assert orc.quantize(z, "f64").tolist() == z.tolist()


def test_quantize_agrees_with_the_input_generators_rounding():
    g = np.random.Generator(np.random.Philox(key=[5, 5]))
    x = (g.standard_normal(20000) * np.exp(g.uniform(-20, 20, 20000))).astype(np.float32).astype(np.float64)
    for dt in ("bf16", "f16"):
        with np.errstate(over="ignore"):
            want = orc.decode(wl.to_storage(x, dt), dt)
        assert np.array_equal(orc.quantize(x, dt), want)


def test_offline_difference_is_online_difference_plus_rounding_of_c():
    cfg = wl.make_config("c2_bf16_4096", seed=2, shape=(48, 200, 64))
    o = orc.verify(cfg["A"], cfg["B"], "bf16", 0)
    rs_off = orc.row_sums_offline(o["C"], "bf16")
    E_off = orc.verification_difference(o["expected"], rs_off)
    resid = (o["C"] - orc.quantize(o["C"], "bf16")).sum(axis=1)
    assert np.allclose(E_off - o["E"], resid, rtol=0, atol=1e-9)
    # every element moves by at most half a unit in the last place of the output type
    assert np.all(np.abs(o["C"] - orc.quantize(o["C"], "bf16")) <= 2.0 ** -8 * np.abs(o["C"]) * (1 + 1e-6))
    # small integers survive the rounding: the offline difference is exactly zero
    g = np.random.Generator(np.random.Philox(key=[5, 6]))
    A = g.integers(-1, 2, size=(16, 24)).astype(np.float64)
    B = g.integers(-1, 2, size=(24, 40)).astype(np.float64)
    C = orc.gemm(A, B)
    assert not orc.verification_difference(orc.expected_checksum(A, orc.encode_checksum(B)),
                                           orc.row_sums_offline(C, "bf16")).any()


def test_offline_difference_follows_the_uniform_rounding_model():
    """U(0,1) BF16 inputs: each stored element carries an independent rounding error, uniform over
    one unit in the last place, so E_i ~ N(0, sum_j ulp_ij^2 / 12) and mean |E| = sqrt(2/pi) sigma."""
    n = 256
    g = np.random.Generator(np.random.Philox(key=[5, 7]))
    A = wl.to_storage(g.random((n, n)), "bf16")
    B = wl.to_storage(g.random((n, n)), "bf16")
    o = orc.verify(A, B, "bf16", 0)
    E_off = orc.verification_difference(o["expected"], orc.row_sums_offline(o["C"], "bf16"))
    ulp = 2.0 ** (np.floor(np.log2(o["C"])) - 7)
    sigma = np.sqrt((ulp ** 2).sum(axis=1) / 12.0)
    ratio = np.abs(E_off).mean() / (math.sqrt(2.0 / math.pi) * sigma.mean())
    assert 0.85 < ratio < 1.15, ratio
    # with e_max = 2 u_output (2^-7, the paper quotes 8e-3) nothing is flagged and the threshold is
    # one to two orders of magnitude above the actual difference (the paper's table: 48x - 158x)
    T = orc.threshold(orc.decode(A, "bf16"), orc.decode(B, "bf16"), orc.default_emax_offline("bf16", n, n))
    assert not orc.fault_flags(E_off, T).any()
    assert 40 < T.mean() / np.abs(E_off).mean() < 400


def test_offline_emax_is_twice_the_output_unit_roundoff():
    assert orc.default_emax_offline("bf16", 4096, 4096) == 2.0 ** -7
    assert abs(orc.default_emax_offline("bf16", 1, 1) - 8e-3) < 0.03 * 8e-3      # the table's e_max for BF16
    assert abs(orc.default_emax_offline("f16", 1, 1) - 1e-3) < 0.03 * 1e-3       # "~1e-3 for FP16"
    assert orc.default_emax_offline("f32", 512, 256) == orc.default_emax("f32", 512, 256)
    assert orc.default_emax_offline("f64", 512, 256) == orc.default_emax("f64", 512, 256)


# --------------------------------------------------------------------------
# column checksums (section 2.2)
# --------------------------------------------------------------------------
def test_column_check_is_the_row_check_of_the_transposed_product():
    """C^T = B^T A^T: every column quantity of (A, B) equals the row quantity of (B^T, A^T)."""
    g = np.random.Generator(np.random.Philox(key=[6, 1]))
    A = g.standard_normal((37, 23)) + 0.3
    B = g.standard_normal((23, 51)) * 2 - 0.1
    col = orc.verify_columns(A.astype(np.float64), B.astype(np.float64), "f64", 0, e_max=1e-15)
    row = orc.verify(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), "f64", 0, e_max=1e-15)
    assert np.allclose(col["eA"], row["Be"], rtol=1e-14)
    assert np.allclose(col["acolstat"], row["bstat"], rtol=1e-14)
    assert np.allclose(col["SA"], row["S"], rtol=1e-13)
    assert np.allclose(col["bcolstat"], row["astat"], rtol=1e-14)
    assert np.allclose(col["expected_col"], row["expected"], rtol=1e-12, atol=1e-12)
    assert np.allclose(col["T_col"], row["T"], rtol=1e-12)
    assert np.allclose(col["colsum"], row["rowsum"], rtol=1e-12, atol=1e-12)
    assert np.array_equal(col["colflags"], row["flags"])


def test_column_checksums_match_brute_force_and_catch_a_planted_error():
    g = np.random.Generator(np.random.Philox(key=[6, 2]))
    A = g.integers(-5, 6, size=(6, 4)).astype(np.float64)
    B = g.integers(-5, 6, size=(4, 7)).astype(np.float64)
    col = orc.verify_columns(A, B, "f64", 0, e_max=1e-12)
    eA = [sum(A[m][k] for m in range(6)) for k in range(4)]
    exp = [sum(eA[k] * B[k][n] for k in range(4)) for n in range(7)]
    C = [[sum(A[i][k] * B[k][j] for k in range(4)) for j in range(7)] for i in range(6)]
    cs = [sum(C[i][j] for i in range(6)) for j in range(7)]
    assert col["eA"].tolist() == eA and col["expected_col"].tolist() == exp and col["colsum"].tolist() == cs
    assert exp == cs and not col["colflags"].any()                       # c1 (A B) == (c1 A) B exactly
    assert col["acolstat"][:, 0].tolist() == [max(A[m][k] for m in range(6)) for k in range(4)]
    assert col["bcolstat"][:, 1].tolist() == [min(B[k][n] for k in range(4)) for n in range(7)]
    # an error in C[2][5] shows up in column 5 only, with E_col = -delta
    bad = orc.replay_faults_columns(col["colsum"], [(2, 5, 0, C[2][5], C[2][5] + 9.0)])
    E = col["expected_col"] - bad
    assert E.tolist() == [0, 0, 0, 0, 0, -9.0, 0]
    assert orc.fault_flags(E, col["T_col"]).tolist() == [0, 0, 0, 0, 0, 1, 0]


def test_column_threshold_counts_m_terms():
    """Constant matrices: A = a, B = b.  Every variance vanishes and T_col = e_max * M |b| * K |a|
    (M terms per checksum entry, K columns of A each with mean a)."""
    M, K, N, a, b = 12, 5, 9, 0.5, -3.0
    col = orc.verify_columns(np.full((M, K), a), np.full((K, N), b), "f64", 0, e_max=1e-3)
    assert np.allclose(col["T_col"], 1e-3 * M * abs(b) * K * abs(a), rtol=1e-14)
    assert np.allclose(col["expected_col"], M * a * K * b)


# --------------------------------------------------------------------------
# FP8 E4M3 storage (OCP): decode and the input generator's rounding
# --------------------------------------------------------------------------
def test_e4m3_decode_known_codes():
    codes = np.array([0x00, 0x01, 0x07, 0x08, 0x38, 0x3C, 0x40, 0x7E, 0xB8, 0x80, 0xFE], dtype=np.uint8)
    want = [0.0, 2.0 ** -9, 7 * 2.0 ** -9, 2.0 ** -6, 1.0, 1.5, 2.0, 448.0, -1.0, -0.0, -448.0]
    assert orc.decode(codes, "f8").tolist() == want
    assert np.isnan(orc.decode(np.array([0x7F, 0xFF], dtype=np.uint8), "f8")).all()
    # all 254 finite codes are distinct, symmetric, and increase with the code within a sign
    allv = orc.decode(np.arange(256, dtype=np.uint8), "f8")
    pos = allv[:0x7F]
    assert np.all(np.diff(pos) > 0) and np.array_equal(allv[0x80:0xFF], -pos)


def test_e4m3_rounding_of_the_generators():
    # every representable value survives; midpoints go to the even code; beyond the range saturates
    codes = np.arange(0x7F, dtype=np.uint8)
    vals = orc.decode(codes, "f8")
    assert np.array_equal(wl.to_storage(vals, "f8"), codes)
    assert np.array_equal(wl.to_storage(-vals[1:], "f8"), codes[1:] | 0x80)
    mid = (vals[:-1] + vals[1:]) / 2
    got = wl.to_storage(mid, "f8")
    assert np.all(got % 2 == 0) and np.all((got == codes[:-1]) | (got == codes[1:]))
    assert wl.to_storage(np.array([1e6, -1e6, 449.0]), "f8").tolist() == [0x7E, 0xFE, 0x7E]
    assert orc.output_dtype("f8") == "f16" and orc.output_dtype("bf16") == "bf16"
    assert orc.default_emax_offline("f8", 64, 64) == 2.0 ** -10   # "FP8 ... e_max ~ 2 u_FP16 ~ 1e-3"
    assert orc.acc_dtype("f8") == np.float32


def test_e5m2_decode_is_the_top_byte_of_binary16():
    # OCP E5M2 has binary16's sign / exponent layout with the mantissa cut to two bits: code c is the
    # half-precision number with bit pattern c << 8 (numpy's float16 decodes that independently)
    codes = np.arange(256, dtype=np.uint8)
    half = (codes.astype(np.uint16) << np.uint16(8)).view(np.float16).astype(np.float64)
    got = orc.decode(codes, "f8e5m2")
    assert np.array_equal(got, half, equal_nan=True)
    assert np.array_equal(np.signbit(got), np.signbit(half))
    assert got[0x3C] == 1.0 and got[0x7B] == 57344.0 and got[0x01] == 2.0 ** -16 and np.isinf(got[0x7C])
    assert np.isnan(got[[0x7D, 0x7E, 0x7F, 0xFD]]).all()


def test_e5m2_rounding_of_the_generators():
    codes = np.arange(0x7C, dtype=np.uint8)          # finite non-negative values
    vals = orc.decode(codes, "f8e5m2")
    assert np.all(np.diff(vals) > 0)
    assert np.array_equal(wl.to_storage(vals, "f8e5m2"), codes)
    assert np.array_equal(wl.to_storage(-vals[1:], "f8e5m2"), codes[1:] | 0x80)
    mid = (vals[:-1] + vals[1:]) / 2
    got = wl.to_storage(mid, "f8e5m2")
    assert np.all(got % 2 == 0) and np.all((got == codes[:-1]) | (got == codes[1:]))
    assert wl.to_storage(np.array([1e9, -1e9, 60000.0]), "f8e5m2").tolist() == [0x7B, 0xFB, 0x7B]
    # values of binary16 that need no more than two mantissa bits survive a trip through numpy's float16
    x = np.array([0.75, -1.25, 3.5, 1.0e-3, 448.0, -6.1e-5])
    h = x.astype(np.float16)
    st = wl.to_storage(h.astype(np.float64), "f8e5m2")
    back = orc.decode(st, "f8e5m2")
    assert np.all(np.abs(back - h.astype(np.float64)) <= 0.125 * np.abs(h.astype(np.float64)))
    assert orc.output_dtype("f8e5m2") == "f16" and orc.acc_dtype("f8e5m2") == np.float32
    assert orc.default_emax_offline("f8e5m2", 64, 64) == 2.0 ** -10


# --------------------------------------------------------------------------
# block-wise verification (section 5.2)
# --------------------------------------------------------------------------
def test_blockwise_reduces_to_the_plain_check_and_adds_up():
    g = np.random.Generator(np.random.Philox(key=[7, 1]))
    A = g.standard_normal((9, 14)) + 0.2
    B = g.standard_normal((14, 23)) - 0.1
    full = orc.verify(A, B, "f64", 0, e_max=1e-15)
    # one block as wide as the matrix is Algorithm 1 itself
    one = orc.verify_blocks(A, B, "f64", 0, 64, 1e-15)
    assert one["nblocks"] == 1
    assert np.allclose(one["T_blk"][0], full["T"], rtol=1e-14) and np.allclose(one["Be_blk"][0], full["Be"])
    assert np.allclose(one["S_blk"][0], full["S"])
    # blocks of 8 columns (the last one ragged: 23 = 8 + 8 + 7)
    blk = orc.verify_blocks(A, B, "f64", 0, 8, 1e-15)
    assert blk["nblocks"] == 3
    assert np.allclose(blk["Be_blk"].sum(axis=0), full["Be"], rtol=1e-13)
    assert np.allclose(blk["expected_blk"].sum(axis=0), full["expected"], rtol=1e-12, atol=1e-12)
    assert np.allclose(blk["rowsum_blk"].sum(axis=0), full["rowsum"], rtol=1e-12, atol=1e-12)
    assert np.allclose(blk["E"], full["E"], rtol=0, atol=1e-12)
    # each block's threshold is Algorithm 1 on the block alone (brute force on the last, ragged block)
    Bt = B[:, 16:23]
    assert np.allclose(blk["T_blk"][2], orc.threshold(A, Bt, 1e-15), rtol=1e-14)
    assert np.allclose(blk["S_blk"][2], orc.b_aggregates(Bt))


def test_blockwise_localises_a_planted_error_to_its_block():
    g = np.random.Generator(np.random.Philox(key=[7, 2]))
    A = g.integers(-3, 4, size=(6, 10)).astype(np.float64)
    B = g.integers(-3, 4, size=(10, 20)).astype(np.float64)
    blk = orc.verify_blocks(A, B, "f64", 0, 8, 1e-12)
    assert not blk["E_blk"].any() and not blk["blockflags"].any()     # exact arithmetic
    rs = orc.replay_faults_blocks(blk["rowsum_blk"], [(4, 17, 0, blk["C"][4, 17], blk["C"][4, 17] + 5.0)], 8)
    E = blk["expected_blk"] - rs
    want = np.zeros((3, 6))
    want[2, 4] = -5.0                                                   # column 17 lies in block 2
    assert np.array_equal(E, want)
    assert orc.fault_flags(E, blk["T_blk"]).sum() == 1 and orc.fault_flags(E, blk["T_blk"])[2, 4] == 1


# ---------------------------------------------------------------------------------------------------------
# the magnitude scales that the GPU parity tolerances are multiplied with (a too-large scale would loosen
# every parity assertion silently): brute force on small integer matrices, every term written out
# ---------------------------------------------------------------------------------------------------------
def _int_matrices(seed, M, K, N):
    g = wl.rng(seed, 31)
    A = g.integers(-4, 5, size=(M, K)).astype(np.float64)
    B = g.integers(-3, 4, size=(K, N)).astype(np.float64)
    return A, B


def test_row_check_tolerance_scales_match_brute_force():
    M, K, N = 5, 7, 6
    A, B = _int_matrices(11, M, K, N)
    o = orc.verify(A, B, "f64", 0, e_max=1e-9)
    Be = [sum(B[k][n] for n in range(N)) for k in range(K)]
    Be2 = [sum((n + 1) * B[k][n] for n in range(N)) for k in range(K)]
    for k in range(K):
        assert o["scale_Be"][k] == sum(abs(B[k][n]) for n in range(N))
        assert o["scale_Be2"][k] == sum((n + 1) * abs(B[k][n]) for n in range(N))
    for i in range(M):
        assert o["scale_expected"][i] == sum(abs(A[i][k]) * abs(Be[k]) for k in range(K))
        assert o["scale_expected2"][i] == sum(abs(A[i][k]) * abs(Be2[k]) for k in range(K))
        # every product term of every element of the row: sum_j sum_k |a_ik| |b_kj|
        assert o["scale_rowsum"][i] == sum(abs(A[i][k]) * abs(B[k][j]) for k in range(K) for j in range(N))
        assert o["scale_rowsum2"][i] == sum((j + 1) * abs(A[i][k]) * abs(B[k][j]) for k in range(K) for j in range(N))
    # a scale bounds the quantity it belongs to, and is attained by a sign-free row (so it is not larger than needed)
    assert np.all(np.abs(o["Be"]) <= o["scale_Be"]) and np.all(np.abs(o["expected"]) <= o["scale_expected"])
    assert np.all(np.abs(o["rowsum"]) <= o["scale_rowsum"])
    op = orc.verify(np.abs(A), np.abs(B), "f64", 0, e_max=1e-9)
    assert np.array_equal(op["scale_Be"], op["Be"]) and np.array_equal(op["scale_expected"], op["expected"])
    assert np.array_equal(op["scale_rowsum"], op["rowsum"])
    # the transposed storage of B gives the same scales
    ot = orc.verify(A, np.ascontiguousarray(B.T), "f64", 1, e_max=1e-9)
    for key in ("scale_Be", "scale_expected", "scale_rowsum"):
        assert np.array_equal(o[key], ot[key]), key


def test_k_blocked_blockwise_partitions_the_blockwise_check():
    """Splitting K as well: the K-block shares of a column block add up to the column block's quantities, one
    K-block as deep as K is the column-block check itself, and every (K-block, column-block) threshold is
    Algorithm 1 on that piece alone (brute force)."""
    g = np.random.default_rng(77)
    M, K, N, W, KB = 9, 20, 23, 8, 6        # K-blocks of 6, 6, 6, 2; column blocks of 8, 8, 7
    A = g.integers(-3, 4, size=(M, K)).astype(np.float64)
    B = g.integers(-3, 4, size=(K, N)).astype(np.float64)
    blk = orc.verify_blocks(A, B, "f64", 0, W, 1e-12)
    kb = orc.verify_blocks_k(A, B, "f64", 0, W, KB, 1e-12)
    assert kb["nkblocks"] == 4 and kb["nblocks"] == 3
    assert np.array_equal(kb["rowsum_blk"].sum(axis=0), blk["rowsum_blk"])          # integers: exact
    assert np.array_equal(kb["expected_blk"].sum(axis=0), blk["expected_blk"])
    assert np.array_equal(np.concatenate(kb["Be_blk"], axis=1), blk["Be_blk"])
    assert not kb["E_blk"].any() and not kb["flags"].any()
    one = orc.verify_blocks_k(A, B, "f64", 0, W, 64, 1e-12)
    assert one["nkblocks"] == 1
    for key in ("expected_blk", "T_blk", "rowsum_blk", "S_blk"):   # K-block 0 carries e_max itself
        assert np.array_equal(one[key][0], blk[key]), key
    # brute force of one interior piece and of the ragged corner piece
    for (b, t) in ((1, 1), (3, 2)):
        ks, ns = range(b * KB, min(K, (b + 1) * KB)), range(t * W, min(N, (t + 1) * W))
        for i in (0, 4, M - 1):
            a = [A[i, k] for k in ks]
            mu_a = sum(a) / len(a)
            var_a = max(0.0, (max(a) - mu_a) * (mu_a - min(a)))
            s1 = s2 = s3 = 0.0
            exp = rs = 0.0
            for k in ks:
                row = [B[k, n] for n in ns]
                mu = sum(row) / len(row)
                s1 += abs(mu)
                s2 += max(0.0, (max(row) - mu) * (mu - min(row)))
                s3 += mu * mu
                exp += A[i, k] * sum(row)
                rs += sum(A[i, k] * x for x in row)
            n = len(ns)
            T = 1e-12 * (b + 1) * (n * abs(mu_a) * s1 + 2.5 * math.sqrt(n * mu_a ** 2 * s2 + n ** 2 * var_a * s3)
                         + 2.5 * math.sqrt(n) * math.sqrt(var_a) * math.sqrt(s2))
            assert kb["T_blk"][b, t, i] == pytest.approx(T, rel=1e-13)
            assert kb["expected_blk"][b, t, i] == exp and kb["rowsum_blk"][b, t, i] == rs
            assert kb["astat"][b, i].tolist() == [max(a), min(a), mu_a]
    # a fault on the finished accumulator lands in the last K-block's share of its column block
    rs = orc.replay_faults_blocks_k(kb["rowsum_blk"], [(4, 17, 0, kb["C"][4, 17], kb["C"][4, 17] + 5.0)], W)
    E = kb["expected_blk"] - rs
    want = np.zeros_like(E)
    want[3, 2, 4] = -5.0
    assert np.array_equal(E, want)
    # tolerance scales: the pieces' scales add up to the column block's
    assert np.array_equal(kb["scale_rowsum_blk"].sum(axis=0), blk["scale_rowsum_blk"])


def test_column_and_block_tolerance_scales_match_brute_force():
    M, K, N, W = 6, 5, 8, 3
    A, B = _int_matrices(12, M, K, N)
    oc = orc.verify_columns(A, B, "f64", 0, e_max=1e-9)
    eA = [sum(A[m][k] for m in range(M)) for k in range(K)]
    for k in range(K):
        assert oc["scale_eA"][k] == sum(abs(A[m][k]) for m in range(M))
    for j in range(N):
        assert oc["scale_expected_col"][j] == sum(abs(eA[k]) * abs(B[k][j]) for k in range(K))
        assert oc["scale_colsum"][j] == sum(abs(A[m][k]) * abs(B[k][j]) for m in range(M) for k in range(K))
    assert np.all(np.abs(oc["colsum"]) <= oc["scale_colsum"])
    ob = orc.verify_blocks(A, B, "f64", 0, W, e_max=1e-9)
    for t in range(ob["nblocks"]):
        cols = range(t * W, min(N, (t + 1) * W))
        Be_t = [sum(B[k][n] for n in cols) for k in range(K)]
        for k in range(K):
            assert ob["scale_Be_blk"][t][k] == sum(abs(B[k][n]) for n in cols)
        for i in range(M):
            assert ob["scale_expected_blk"][t][i] == sum(abs(A[i][k]) * abs(Be_t[k]) for k in range(K))
            assert ob["scale_rowsum_blk"][t][i] == sum(abs(A[i][k]) * abs(B[k][j]) for k in range(K) for j in cols)
    # the block scales of a row add up to the row scale of the plain check
    o = orc.verify(A, B, "f64", 0, e_max=1e-9)
    assert np.array_equal(ob["scale_rowsum_blk"].sum(axis=0), o["scale_rowsum"])
