"""FP8 (OCP E4M3 and E5M2) inputs with FP32 accumulation and FP16 output (paper section 3.6: "FP8 inputs -> FP32
accumulation -> FP16 output"): parity of the whole path with the CPU oracle.  Whole 256 x 256 x 256 tiles with B
stored N x K run on the FP8 matrix instruction; any other shape or layout takes the guarded route."""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import (OUT_TINY, U_OUT, _dev, _emax, _session, _tol, check_light, check_rows)  # noqa: E402
from test_gpu_weighted import check_weighted  # noqa: E402
from test_gpu_columns import check_columns  # noqa: E402
from test_gpu_blocks import check_blocks  # noqa: E402


FORMATS = ["f8", "f8e5m2"]   # E4M3, E5M2 (section 3.6 names both)


def _gen8(M, N, K, transB, seed, dist="n_1e-6_1", f8="f8"):
    g = wl.rng(seed, 19)
    A = wl.to_storage(wl.paper_distribution(g, dist, (M, K)), f8)
    Bl = wl.paper_distribution(g, dist, (K, N))
    B = wl.to_storage(np.ascontiguousarray(Bl.T) if transB else Bl, f8)
    return A, B


def check_C8(r, o, A_st, B_st, transB, f8="f8"):
    C = r["C"].astype(np.float64)                       # FP16 product
    absprod = np.abs(orc.decode(A_st, f8)) @ np.abs(orc.logical_B(B_st, f8, transB))
    bound = U_OUT["f16"] * np.abs(o["C"]) + _tol(f8) * absprod + OUT_TINY["f16"]
    assert np.all(np.abs(C - o["C"]) <= bound), "C"


@pytest.mark.parametrize("f8", FORMATS)
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (512, 768, 512), (256, 512, 1024)])
def test_fp8_fault_free_parity(M, N, K, f8):
    for seed, dist in ((1, "n_1e-6_1"), (2, "n_1_1"), (3, "u_-1_1")):
        A, B = _gen8(M, N, K, 1, seed, dist, f8)
        print(f"{f8} {M}x{N}x{K} {dist}", flush=True)
        vg = _session(M, N, K, f8, 1)
        dA, dB = _dev(A, f8), _dev(B, f8)
        o = orc.verify(A, B, f8, 1, e_max=_emax(f8, K, N))
        for route in ("run", "run_fused", "run_weighted", "run_rc"):
            getattr(vg, route)(dA, dB)
            r = vg.results()
            check_light(r, o, f8, M, N, K)
            check_rows(r, o, f8)
            check_C8(r, o, A, B, 1, f8)
            assert r["nflag"] == 0 and not r["flags"].any() and not o["flags"].any()
            if route == "run_weighted":
                check_weighted(r, o, f8)
            if route == "run_rc":
                oc = orc.verify_columns(A, B, f8, 1, e_max=_emax(f8, K, max(N, M)))
                check_columns(r, oc, f8, M, N, K)
                assert r["ncolflag"] == 0
        # plain GEMM gives the same C
        C1 = vg.results()["C"].copy()
        vg.gemm(dA, dB, 0)
        assert np.array_equal(vg.results()["C"], C1)


@pytest.mark.parametrize("f8", FORMATS)
def test_fp8_exact_arithmetic_flips_and_localisation(f8):
    M, N, K = 512, 512, 256
    g = wl.rng(5, 5)
    A = wl.to_storage(g.integers(-2, 3, size=(M, K)).astype(np.float64), f8)
    B = wl.to_storage(g.integers(-2, 3, size=(N, K)).astype(np.float64), f8)
    dA, dB = _dev(A, f8), _dev(B, f8)
    vg = _session(M, N, K, f8, 1)
    vg.run_weighted(dA, dB)
    r = vg.results()
    o = orc.verify(A, B, f8, 1, e_max=_emax(f8, K, N))
    assert np.array_equal(r["Be"].astype(np.float64), o["Be"])
    assert np.array_equal(r["expected"].astype(np.float64), o["expected"])
    assert np.array_equal(r["rowsum"].astype(np.float64), o["rowsum"])
    assert np.array_equal(r["rowsum2"].astype(np.float64), o["rowsum2"])
    assert np.array_equal(r["C"].astype(np.float64), o["C"])      # |C| <= 4 * 256: exact in FP16
    assert not r["E"].any() and r["nflag"] == 0
    # planted flips of the top mantissa bit: detected, located, corrected exactly
    cand = [(0, 0), (M - 1, N - 1), (255, 256), (300, 17)]
    faults = [(i, j, 22) for (i, j) in cand if abs(o["C"][i, j]) >= 1]
    assert len(faults) >= 2
    vg.run_weighted(dA, dB, inj=vg.make_inject(mode=1, faults=faults), correct=1)
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == len(faults) and [x[:3] for x in recs] == sorted(faults)
    for (i, j, b, before, after) in recs:
        assert before == o["C"][i, j] and after == orc.bitflip(before, b, np.float32)
        assert r["flags"][i] == 1 and r["loc"][i] == j and r["E"][i] == -(after - before)
    assert r["nflag"] == len(faults) and r["ncorrected"] == len(faults)
    assert np.array_equal(r["C"].astype(np.float64), o["C"])


@pytest.mark.parametrize("f8", FORMATS)
@pytest.mark.parametrize("M,N,K,transB", [(300, 200, 77, 1), (100, 130, 50, 0), (64, 48, 16, 1), (512, 512, 512, 0),
                                          (257, 515, 300, 0), (256, 256, 128, 1)])
def test_fp8_any_shape_and_layout(M, N, K, transB, f8):
    """Ragged FP8 problems, a K x N B, and a K that is not a multiple of 256: every pass, the GEMM on the guarded
    route (operands widened to FP16 on load), the fused call, weighted sums and column check, against the oracle;
    then the offline check of an FP16 product computed elsewhere."""
    from paper_2602_08043_amd import binding as vb
    A, B = _gen8(M, N, K, transB, 7, f8=f8)
    print(f"{f8} any shape {M}x{N}x{K} transB={transB}", flush=True)
    vg = _session(M, N, K, f8, transB)
    dA, dB = _dev(A, f8), _dev(B, f8)
    o = orc.verify(A, B, f8, transB, e_max=_emax(f8, K, N))
    for route in ("run", "run_fused", "run_weighted", "run_rc"):
        getattr(vg, route)(dA, dB)
        r = vg.results()
        check_light(r, o, f8, M, N, K)
        check_rows(r, o, f8)
        check_C8(r, o, A, B, transB, f8)
        assert r["nflag"] == 0 and not r["flags"].any() and not o["flags"].any()
        if route == "run_weighted":
            check_weighted(r, o, f8)
        if route == "run_rc":
            oc = orc.verify_columns(A, B, f8, transB, e_max=_emax(f8, K, max(N, M)))
            check_columns(r, oc, f8, M, N, K)
            assert r["ncolflag"] == 0
    # a planted flip of the exponent's top bit is flagged in its row, and only there
    i, j = M - 1, N // 3
    vg.run(dA, dB, inj=vg.make_inject(mode=1, faults=[(i, j, 30)]))
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == 1 and recs[0][:3] == (i, j, 30)
    assert r["flags"][i] == 1 and r["nflag"] == 1 and r["flags"].sum() == 1
    # offline check of an FP16 product computed elsewhere, with e_max = 2 u_FP16
    e_off = vb.vabft_default_emax_offline(f8, K, N)
    assert e_off == 2.0 ** -10
    vg.encode(dB)
    vg.threshold(dA, e_off)
    Bl = orc.logical_B(B, f8, transB)
    # the stored product: rounded the way the oracle's offline check reads it (through the FP32 accumulator);
    # rounding the FP64 product straight to FP16 differs in rare double-rounding cases
    C16 = torch.from_numpy(orc.quantize(orc.decode(A, f8) @ Bl, "f16").astype(np.float16)).cuda()
    vg.check_offline(C16)
    r = vg.results()
    assert r["nflag"] == 0
    rs_off = orc.row_sums_offline(orc.decode(A, f8) @ Bl, "f16")
    assert np.all(np.abs(r["rowsum"] - rs_off) <= 4 * U_OUT["f32"] * np.abs(C16.float().cpu().numpy()).sum(axis=1) + 1e-30)


@pytest.mark.parametrize("name", ["c6_f8_4096", "c8_f8e5m2_4096"])
def test_fp8_full_size_sampled(name):
    cfg = wl.make_config(name, seed=0)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    dA, dB = _dev(cfg["A"], dt), _dev(cfg["B"], dt)
    vg = _session(M, N, K, dt, tb)
    vg.run_fused(dA, dB)
    r = vg.results()
    rows = np.unique(np.concatenate([wl.rng(3, 78).choice(M, size=48, replace=False), [0, 255, 256, M - 1]]))
    o = orc.verify(cfg["A"], cfg["B"], dt, tb, e_max=_emax(dt, K, N), rows=rows)
    check_light(r, o, dt, M, N, K)
    check_rows(r, o, dt, rows)
    C = r["C"].astype(np.float64)[rows]
    absprod = np.abs(orc.decode(cfg["A"], dt)[rows]) @ np.abs(orc.logical_B(cfg["B"], dt, tb))
    assert np.all(np.abs(C - o["C"]) <= U_OUT["f16"] * np.abs(o["C"]) + _tol(dt) * absprod + OUT_TINY["f16"])
    assert r["nflag"] == 0 and np.all(np.abs(r["E"]) <= r["T"])
    i = int(rows[7])
    vg.gemm(dA, dB, 1, vg.make_inject(mode=1, faults=[(i, N - 5, 28)]))
    r2 = vg.results()
    assert np.nonzero(r2["flags"])[0].tolist() == [i] and r2["nflag"] == 1


@pytest.mark.parametrize("M,N,K", [(256, 512, 256), (512, 1024, 2048), (768, 512, 3072), (256, 512, 3584),
                                   (256, 768, 768)])
@pytest.mark.parametrize("f8", FORMATS)
def test_fp8_fused_call_single_launch(M, N, K, f8):
    """vabft_gemm_verified_fused on FP8 problems the single-launch kernel takes (statistics of A folded from the
    operand fragments: units of 256 k dealt to the tile-columns, up to eight per workgroup) and one it hands to
    the two-pass route (3584 / 256 = 14 units on two tile-columns), with and without the deferred fold of S1..S3,
    against the oracle and against the three-call route."""
    for seed, dist in ((41, "n_1e-6_1"), (42, "u_-1_1")):
        A, B = _gen8(M, N, K, 1, seed, dist, f8)
        print(f"{f8} fused {M}x{N}x{K} {dist}", flush=True)
        vg = _session(M, N, K, f8, 1)
        dA, dB = _dev(A, f8), _dev(B, f8)
        o = orc.verify(A, B, f8, 1, e_max=_emax(f8, K, N))
        vg.run(dA, dB)
        r3 = {k: np.copy(v) for k, v in vg.results().items()}
        for defer in (False, True, False):
            vg.T.fill_(-1.0)
            vg.astat.fill_(9.0)
            vg.flags.fill_(3)
            vg.run_fused(dA, dB, defer_S=defer)
            r = vg.results()
            if not defer:
                check_light(r, o, f8, M, N, K)
            check_rows(r, o, f8)
            check_C8(r, o, A, B, 1, f8)
            assert np.array_equal(r["astat"][:, 0].astype(np.float64), o["astat"][:, 0])
            assert np.array_equal(r["astat"][:, 1].astype(np.float64), o["astat"][:, 1])
            assert np.allclose(r["T"], r3["T"], rtol=2e-6, atol=0)
            assert np.array_equal(r["C"], r3["C"]) and np.array_equal(r["rowsum"], r3["rowsum"])
            assert r["nflag"] == 0 and not r["flags"].any()
    i, j = M - 1, N // 2
    vg.run_fused(dA, dB, inj=vg.make_inject(mode=1, faults=[(i, j, 30)]), defer_S=True)
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == 1 and recs[0][:3] == (i, j, 30)
    assert r["flags"][i] == 1 and r["nflag"] == 1 and r["flags"].sum() == 1
    vg.run_fused(dA, dB)
    assert vg.results()["nflag"] == 0


@pytest.mark.parametrize("f8", FORMATS)
@pytest.mark.parametrize("M,N,K,transB", [(512, 768, 256, 1), (300, 520, 200, 0)])
def test_fp8_blockwise(M, N, K, transB, f8):
    """Block-wise verification (blocks of 256 columns) of FP8 problems: the whole-tile kernel's partials-only mode
    and the guarded route, against the oracle; a planted fault flags exactly its (block, row) pair."""
    from paper_2602_08043_amd import binding as vb
    W = vb.vabft_block_width(f8)
    assert W == 256
    A, B = _gen8(M, N, K, transB, 23, "n_1_1", f8)
    print(f"{f8} blocks {M}x{N}x{K} transB={transB}", flush=True)
    e_blk = vb.vabft_default_emax(f8, K, min(N, W))
    vg = _session(M, N, K, f8, transB)
    dA, dB = _dev(A, f8), _dev(B, f8)
    vg.run_blocks(dA, dB)
    r = vg.results()
    ob = orc.verify_blocks(A, B, f8, transB, W, e_blk)
    check_blocks(r, ob, f8)
    check_C8(r, ob, A, B, transB, f8)
    assert r["nflag"] == 0 and r["nblockflag"] == 0 and not r["blockflags"].any() and not ob["blockflags"].any()
    i, j = M // 2, N - 3
    vg.run_blocks(dA, dB, inj=vg.make_inject(mode=1, faults=[(i, j, 30)]))
    r = vg.results()
    assert r["nblockflag"] == 1 and r["blockflags"][j // W, i] == 1 and r["blockflags"].sum() == 1
    assert r["flags"][i] == 1 and r["nflag"] == 1
