"""Leading dimensions larger than the row length, and the largest benchmark workload under the
Bernoulli injector (benchmark configuration 4: FP16 8192^3, rate 1e-6 per element)."""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import (_acc_np, _dev, _emax, _gen, _session, check_C, check_light, check_rows)  # noqa: E402

_TDT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32, "f64": torch.float64}


def _padded(x_dev, ld, fill):
    """Device matrix with row pitch `ld` elements holding x in its first columns, `fill` elsewhere."""
    rows, cols = x_dev.shape
    buf = torch.full((rows, ld), fill, dtype=x_dev.dtype, device=x_dev.device)
    buf[:, :cols] = x_dev
    return buf


@pytest.mark.parametrize("dtype,M,N,K,transB,pads", [
    # pads = extra elements per row of (A, B, C); multiples of 8 keep 16-bit rows 16-byte aligned
    ("bf16", 512, 512, 256, 0, (8, 16, 24)), ("bf16", 512, 512, 256, 1, (64, 8, 8)),
    ("bf16", 512, 512, 256, 0, (3, 5, 1)), ("f16", 300, 520, 200, 1, (8, 8, 8)), ("f16", 256, 256, 128, 0, (1, 2, 3)),
    ("f32", 256, 256, 64, 0, (4, 8, 12)), ("f32", 200, 260, 70, 1, (1, 3, 2)),
    ("f64", 256, 128, 64, 0, (2, 4, 6)), ("f64", 131, 67, 33, 1, (1, 1, 1)),
])
def test_padded_leading_dimensions(dtype, M, N, K, transB, pads):
    from paper_2602_08043_amd import binding as vb
    A, B = _gen(dtype, M, N, K, transB, 21, "n_1e-6_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    pa, pb, pc = pads
    lda, ldb, ldc = K + pa, (K if transB else N) + pb, N + pc
    print(f"padded {dtype} {M}x{N}x{K} transB={transB} lda={lda} ldb={ldb} ldc={ldc}", flush=True)
    # padding holds a large value: reading it would wreck every sum and extremum
    Ap, Bp = _padded(dA, lda, 1000.0), _padded(dB, ldb, -1000.0)
    vg = _session(M, N, K, dtype, transB)
    vg.problem = vb.make_problem(M, N, K, dtype, transB, lda, ldb, ldc)
    vg.C = torch.full((M, ldc), 7.0, dtype=_TDT[dtype], device="cuda")
    for route in ("run", "run_fused", "run_weighted"):
        vg.C.fill_(7.0)
        getattr(vg, route)(Ap, Bp)
        r = vg.results()
        Cfull = vg.C.float().cpu().numpy() if dtype != "f64" else vg.C.cpu().numpy()
        assert np.all(Cfull[:, N:] == 7.0), "padding of C was written"
        r["C"] = r["C"][:, :N]
        o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
        check_light(r, o, dtype, M, N, K)
        check_rows(r, o, dtype)
        check_C(r, o, A, B, dtype, transB)
        assert r["nflag"] == 0 and not r["flags"].any()
    # the contiguous problem gives the same numbers bit for bit when the same kernels run
    # (aligned padding keeps the whole-tile kernels; odd padding switches to the guarded ones)
    vg2 = _session(M, N, K, dtype, transB)
    vg2.run(dA, dB)
    r2 = vg2.results()
    elem = 8 if dtype == "f64" else 4 if dtype == "f32" else 2
    if all((p * elem) % 16 == 0 for p in pads):
        vg.C.fill_(7.0)
        vg.run(Ap, Bp)
        r = vg.results()
        assert np.array_equal(r["C"][:, :N], r2["C"]) and np.array_equal(r["rowsum"], r2["rowsum"])
        assert np.array_equal(r["Be"], r2["Be"]) and np.array_equal(r["expected"], r2["expected"])


def test_full_size_bernoulli_c4():
    """FP16 8192^3, U(-1,1), Bernoulli 1e-6 per element on accumulator bits 16..31: the injected set
    equals the oracle's generator, every record is a true bit flip, and flags match the replay."""
    cfg = wl.make_config("c4_f16_8192", seed=0)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    dA, dB = _dev(cfg["A"], dt), _dev(cfg["B"], dt)
    vg = _session(M, N, K, dt, tb)
    seed, rate, lo, hi = 20260208, 1e-6, 16, 31
    inj = vg.make_inject(mode=2, seed=seed, rate=rate, bit_lo=lo, bit_hi=hi)
    vg.run_fused(dA, dB, inj=inj)
    r = vg.results()
    n, recs = vg.inject_records()
    want_set = orc.bernoulli_faults(seed, rate, lo, hi, M, N)
    print(f"c4 bernoulli: {n} flips", flush=True)
    assert 30 <= len(want_set) <= 120  # about 67 expected
    assert n == len(want_set) and [rec[:3] for rec in recs] == sorted(want_set)
    acc = _acc_np(dt)
    for (_i, _j, bit, before, after) in recs:
        f = orc.bitflip(before, bit, acc)
        assert after == f or (np.isnan(after) and np.isnan(f))
    rows = np.array(sorted(set(rec[0] for rec in recs)))
    clean = np.setdiff1d(np.arange(M), rows)
    assert not r["flags"][clean].any()
    o = orc.verify(cfg["A"], cfg["B"], dt, tb, e_max=_emax(dt, K, N), rows=rows)
    index = {int(i): p for p, i in enumerate(rows)}
    for (i, j, _b, before, _after) in recs:
        ref = o["C"][index[i], j]
        assert abs(before - ref) <= 1e-5 * (np.abs(orc.decode(cfg["A"], dt)[i]) @ np.abs(orc.logical_B(cfg["B"], dt, tb)[:, j]))
    rs = orc.replay_faults(o["rowsum"], recs, index)
    with np.errstate(invalid="ignore"):
        want = orc.fault_flags(orc.verification_difference(o["expected"][rows], rs), o["T"][rows])
    per_row = {}
    for (i, _j, _b, before, after) in recs:
        per_row.setdefault(i, []).append(abs(after - before))
    decided = 0
    for i, ds in per_row.items():
        if len(ds) == 1 and (not (ds[0] < 10 * o["T"][i]) or ds[0] < 0.1 * o["T"][i]):
            assert r["flags"][i] == want[index[i]], (i, ds, o["T"][i])
            decided += 1
    assert decided >= len(per_row) // 2
    assert r["nflag"] == int(r["flags"].sum())


def test_full_size_c3_every_route():
    """BF16 FFN shape 4096 x 11008 x 4096 with B stored N x K (43 tile-columns, an odd count): the
    weighted, row+column and block-wise routes at full size on sampled rows and columns."""
    from test_gpu_weighted import check_weighted
    from paper_2602_08043_amd import binding as vb
    cfg = wl.make_config("c3_bf16_ffn", seed=1)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    dA, dB = _dev(cfg["A"], dt), _dev(cfg["B"], dt)
    vg = _session(M, N, K, dt, tb)
    rows = np.unique(np.concatenate([wl.rng(1, 5).choice(M, size=20, replace=False), [0, 255, 256, M - 1]]))
    o = orc.verify(cfg["A"], cfg["B"], dt, tb, e_max=_emax(dt, K, N), rows=rows)
    tol = 1e-5
    # weighted route
    vg.run_weighted(dA, dB, correct=1)
    r = vg.results()
    check_light(r, o, dt, M, N, K)
    check_rows(r, o, dt, rows)
    check_weighted(r, o, dt, rows)
    assert r["nflag"] == 0 and r["ncorrected"] == 0 and np.all(r["loc"] == orc.LOC_NOT_FLAGGED)
    # row + column route: sampled columns against the product of A with those columns
    vg.run_rc(dA, dB)
    r = vg.results()
    oc = orc.verify_columns(cfg["A"], cfg["B"], dt, tb, e_max=_emax(dt, K, max(N, M)), full_gemm=False)
    assert np.all(np.abs(r["eA"] - oc["eA"]) <= tol * oc["scale_eA"])
    assert np.all(np.abs(r["expected_col"] - oc["expected_col"]) <= tol * oc["scale_expected_col"])
    assert np.all(np.abs(r["T_col"] - oc["T_col"]) <= 2e-5 * oc["T_col"])
    cols = np.unique(np.concatenate([wl.rng(1, 6).choice(N, size=20, replace=False), [0, 255, 256, N - 1]]))
    A64 = orc.decode(cfg["A"], dt)
    B64 = orc.logical_B(cfg["B"], dt, tb)
    colsum = (A64 @ B64[:, cols]).sum(axis=0)
    assert np.all(np.abs(r["colsum"][cols] - colsum) <= tol * oc["scale_colsum"][cols])
    assert r["nflag"] == 0 and r["ncolflag"] == 0
    assert np.all(np.abs(r["E_col"]) <= r["T_col"])
    # block-wise route
    W = vb.vabft_block_width(dt)
    vg.run_blocks(dA, dB)
    r = vg.results()
    ob = orc.verify_blocks(cfg["A"], cfg["B"], dt, tb, W, vb.vabft_default_emax(dt, K, W), full_gemm=False)
    assert np.all(np.abs(r["Be_blk"] - ob["Be_blk"]) <= tol * ob["scale_Be_blk"] + 1e-30)
    assert np.all(np.abs(r["expected_blk"] - ob["expected_blk"]) <= tol * ob["scale_expected_blk"] + 1e-30)
    assert np.all(np.abs(r["T_blk"] - ob["T_blk"]) <= 1e-4 * ob["T_blk"])
    rs = o["C"].reshape(len(rows), N // W, W).sum(axis=2).T
    assert np.all(np.abs(r["rowsum_blk"][:, rows] - rs) <= tol * ob["scale_rowsum_blk"][:, rows])
    assert r["nflag"] == 0 and r["nblockflag"] == 0
    # one fault: its row, its column, its block
    i, j = int(rows[9]), 10999
    inj = vg.make_inject(mode=1, faults=[(i, j, 29)])
    vg.gemm_blocks(dA, dB, inj)
    r = vg.results()
    assert list(zip(*np.nonzero(r["blockflags"]))) == [(j // W, i)] and r["nblockflag"] == 1 and r["nflag"] == 1
    vg.run_rc(dA, dB, inj=inj)
    r = vg.results()
    assert np.nonzero(r["flags"])[0].tolist() == [i] and np.nonzero(r["colflags"])[0].tolist() == [j]


@pytest.mark.parametrize("dtype,M,N,K,transB", [
    # more than 65535 rows / columns / tile indices in one direction; whole tiles and ragged
    ("bf16", 196608, 256, 128, 0), ("bf16", 256, 196608, 128, 1), ("f16", 100003, 130, 72, 0),
    ("f32", 131072, 128, 16, 0), ("f32", 70001, 40, 33, 1), ("f64", 128, 66000, 16, 0),
    ("bf16", 256, 256, 16384, 0), ("f64", 130, 70, 20001, 1),
])
def test_long_dimensions(dtype, M, N, K, transB):
    """One dimension far beyond the benchmark shapes (index arithmetic, grids, the S1..S3 partials of a long K)."""
    print(f"long {dtype} {M}x{N}x{K} transB={transB}", flush=True)
    A, B = _gen(dtype, M, N, K, transB, 33, "n_1e-6_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB)
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    for route, kw in (("run", {}), ("run_fused", {"defer_S": True})):
        vg.flags.fill_(5)
        getattr(vg, route)(dA, dB, **kw)
        r = vg.results()
        if route == "run":
            check_light(r, o, dtype, M, N, K)
        check_rows(r, o, dtype)
        check_C(r, o, A, B, dtype, transB)
        assert r["nflag"] == 0 and not r["flags"].any()
    i, j = M - 1, N - 1
    bit = 62 if dtype == "f64" else 30
    vg.run_fused(dA, dB, inj=vg.make_inject(mode=1, faults=[(i, j, bit)]))
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == 1 and recs[0][:3] == (i, j, bit)
    assert r["flags"][i] == 1 and r["nflag"] == 1 and r["flags"].sum() == 1


@pytest.mark.parametrize("dtype,Ms,Ml,N,K,transB", [("bf16", 256, 15616, 256, 128, 0), ("f16", 256, 15616, 256, 128, 1),
                                                    ("f32", 128, 7808, 128, 64, 0), ("f64", 128, 7808, 128, 64, 1)])
def test_encode_of_B_serves_any_row_count(dtype, Ms, Ml, N, K, transB):
    """B is encoded once through a problem with few rows (fold of S1..S3 deferred); a fused GEMM with many rows
    on the same workspace must find the partials: their place depends on B's shape only, not on M (61 tile-rows
    put the arrival counters of the large problem past one 256-byte step, 2 tile-rows do not)."""
    A, B = _gen(dtype, Ml, N, K, transB, 77)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    big = _session(Ml, N, K, dtype, transB)
    small = _session(Ms, N, K, dtype, transB)
    small.ws, small.ws_bytes = big.ws, big.ws_bytes  # one workspace, sized for the larger problem
    small.Be, small.bstat = big.Be, big.bstat
    print(f"encode through M={Ms}, fused GEMM with M={Ml}: {dtype} N={N} K={K} transB={transB}", flush=True)
    big.S.fill_(float("nan"))  # the deferred route must not read it
    small.encode(dB, defer_S=True)
    big.gemm_fused(dA, dB, deferred_S=True)
    r = big.results()
    ref = _session(Ml, N, K, dtype, transB)
    ref.run_fused(dA, dB)
    r2 = ref.results()
    assert r["nflag"] == 0 and r2["nflag"] == 0
    for key in ("T", "expected", "rowsum", "E"):
        assert np.array_equal(r[key], r2[key]), key
    # ... and an encode of the columns of A takes that place: documented to invalidate the deferred fold
    o = orc.verify(A, B, dtype, transB, e_max=_emax(dtype, K, N))
    assert np.all(np.abs(r["T"] - o["T"]) <= 1e-5 * o["T"] + 1e-300)
