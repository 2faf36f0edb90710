"""Parity of the block-wise verification with K split as well (paper section 5.2: statistics "for each block of A
and B", tile (M, K, N) = (128, 1024, 256)) with the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from oracle import vabft_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import _dev, _gen, _tol, check_C  # noqa: E402


def _session(M, N, K, dtype, transB, kblock):
    from paper_2602_08043_amd.session import KBlockedGemm
    return KBlockedGemm(M, N, K, dtype, transB, kblock)


def _emax(dtype, KB, W):
    from paper_2602_08043_amd import binding as vb
    return vb.vabft_default_emax(dtype, KB, W)


def check_pieces(r, ob, dtype, M, N, K, kblock, gemm=True):
    tol, tiny = _tol(dtype), 1e-300
    nkb, nb, W = ob["nkblocks"], ob["nblocks"], ob["W"]
    for b in range(nkb):
        k0, len_b = b * kblock, min(kblock, K - b * kblock)
        be = r["Be_blk_k"][nb * k0: nb * k0 + nb * len_b].reshape(nb, len_b)
        assert np.all(np.abs(be - ob["Be_blk"][b]) <= tol * ob["scale_Be_blk"][b] + tiny), ("Be", b)
        mean_scale = ob["scale_Be_blk"][b].sum(axis=1) / W
        dS = np.abs(r["S_blk_k"][b] - ob["S_blk"][b])
        assert np.all(dS[:, 0] <= tol * mean_scale * 4 + tiny), ("S1", b)
        assert np.all(dS[:, 1] <= 1e-4 * ob["S_blk"][b][:, 1] + tiny), ("S2", b)
        assert np.all(dS[:, 2] <= 1e-4 * ob["S_blk"][b][:, 2] + tol * mean_scale ** 2 + tiny), ("S3", b)
        assert np.array_equal(r["astat_k"][b][:, 0].astype(np.float64), ob["astat"][b][:, 0])
        assert np.array_equal(r["astat_k"][b][:, 1].astype(np.float64), ob["astat"][b][:, 1])
    assert np.all(np.abs(r["expected_blk_k"] - ob["expected_blk"]) <= tol * ob["scale_expected_blk"] + tiny), "expected"
    assert np.all(np.abs(r["T_blk_k"] - ob["T_blk"]) <= 1e-4 * ob["T_blk"] + tiny), "T"
    if gemm:
        # a K-block's share is a difference of two prefix row sums: its error scales with the prefix, i.e. with the
        # scales of all K-blocks up to this one
        prefix_scale = np.cumsum(ob["scale_rowsum_blk"], axis=0)
        assert np.all(np.abs(r["rowsum_blk_k"] - ob["rowsum_blk"]) <= tol * prefix_scale + tiny), "rowsum"
        assert np.all(np.abs(r["E_blk_k"] - ob["E_blk"]) <= 2 * tol * prefix_scale + tiny), "E"
        assert np.all(np.abs(r["E"] - ob["E"]) <= 2 * tol * prefix_scale.sum(axis=(0, 1)) + tiny), "E aggregate"


SHAPES = [("bf16", 512, 768, 512, 0, 128), ("bf16", 256, 512, 640, 1, 256), ("f16", 256, 512, 1024, 1, 256),
          ("f16", 512, 256, 192, 0, 128), ("bf16", 256, 256, 256, 0, 1024)]


@pytest.mark.parametrize("dtype,M,N,K,transB,kblock", SHAPES)
def test_k_blocked_fault_free_parity(dtype, M, N, K, transB, kblock):
    from paper_2602_08043_amd import binding as vb
    W = vb.vabft_block_width(dtype)
    for seed, dist in ((71, "n_1e-6_1"), (72, "n_1_1")):
        A, B = _gen(dtype, M, N, K, transB, seed, dist)
        print(f"k-blocked {dtype} {M}x{N}x{K} transB={transB} kblock={kblock} {dist}", flush=True)
        vg = _session(M, N, K, dtype, transB, kblock)
        assert vg.nkb == (K + kblock - 1) // kblock
        e = _emax(dtype, min(K, kblock), min(N, W))
        vg.run(_dev(A, dtype), _dev(B, dtype), e)
        r = vg.results()
        ob = orc.verify_blocks_k(A, B, dtype, transB, W, kblock, e)
        check_pieces(r, ob, dtype, M, N, K, kblock)
        check_C(r, ob, A, B, dtype, transB)
        assert r["nflag"] == 0 and r["nblockflag"] == 0 and not r["blockflags_k"].any() and not r["flags"].any()
        assert not ob["blockflags"].any()
        assert np.all(np.abs(r["E_blk_k"]) <= r["T_blk_k"])
        # a second run on the same buffers gives the same bits
        first = {k: np.copy(v) for k, v in r.items() if isinstance(v, np.ndarray)}
        vg.run(_dev(A, dtype), _dev(B, dtype), e)
        r2 = vg.results()
        for k, v in first.items():
            assert np.array_equal(r2[k], v), k


def test_k_blocked_exact_arithmetic_and_planted_faults():
    dtype, M, N, K, kblock = "bf16", 512, 512, 512, 128
    g = wl.rng(9, 9)
    A = wl.to_storage(g.integers(-2, 3, size=(M, K)).astype(np.float64), dtype)
    B = wl.to_storage(g.integers(-2, 3, size=(K, N)).astype(np.float64), dtype)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, 0, kblock)
    e = _emax(dtype, kblock, 256)
    vg.run(dA, dB, e)
    r = vg.results()
    ob = orc.verify_blocks_k(A, B, dtype, 0, 256, kblock, e)
    assert np.array_equal(r["rowsum_blk_k"].astype(np.float64), ob["rowsum_blk"])     # small integers: exact
    assert np.array_equal(r["expected_blk_k"].astype(np.float64), ob["expected_blk"])
    assert not r["E_blk_k"].any() and r["nflag"] == 0
    # faults on the finished accumulator land in the last K-block's share of their column block
    faults = [(0, 0, 22), (M - 1, N - 1, 22), (255, 256, 22), (300, 17, 22)]
    faults = [(i, j, b) for (i, j, b) in faults if abs(ob["C"][i, j]) >= 1]
    assert len(faults) >= 2
    vg.gemm(dA, dB, vg.make_inject(mode=1, faults=faults))
    r = vg.results()
    n, recs = vg.inject_records()
    assert n == len(faults) and [x[:3] for x in recs] == sorted(faults)
    rs = orc.replay_faults_blocks_k(ob["rowsum_blk"], recs, 256)
    assert np.array_equal(r["rowsum_blk_k"].astype(np.float64), rs)
    want = np.zeros_like(r["blockflags_k"])
    for (i, j, _b) in faults:
        want[-1, j // 256, i] = 1
    assert np.array_equal(r["blockflags_k"], want)
    assert r["nblockflag"] == len(faults) and r["nflag"] == len({i for (i, _j, _b) in faults})
    assert np.array_equal(np.nonzero(r["flags"])[0], sorted({i for (i, _j, _b) in faults}))


def test_k_blocked_thresholds_are_tighter_than_the_column_block_ones():
    """What the section is after: a piece accumulates fewer terms, so its threshold is a fraction of the column
    block's; a fault between the two is caught only by the K-blocked check."""
    dtype, M, N, K, kblock = "bf16", 256, 512, 2048, 256
    A, B = _gen(dtype, M, N, K, 0, 5, "n_1_1")
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, 0, kblock)
    vg.run(dA, dB)
    r = vg.results()
    from test_gpu_parity import _session as _plain_session
    col = _plain_session(M, N, K, dtype, 0)
    col.run_blocks(dA, dB)
    rc = col.results()
    ratio = rc["T_blk"][None, :, :] / r["T_blk_k"]      # [K-block][column block][row]
    # 8 K-blocks: the first piece's threshold is an eighth of the block's or less; later pieces carry (b + 1) e_max
    # (their share is gained on a running accumulator b blocks deep) and approach the block's threshold from below
    assert np.median(ratio[0]) > 6.0 and np.median(ratio) > 1.5 and np.all(np.median(ratio, axis=(1, 2)) > 0.9)
    assert r["nflag"] == 0 and rc["nflag"] == 0


@pytest.mark.parametrize("dtype,M,N,K,transB,kblock", [("f32", 200, 260, 300, 0, 128), ("f64", 131, 67, 256, 1, 128),
                                                        ("bf16", 300, 520, 200, 1, 128)])
def test_k_blocked_passes_take_any_shape_and_type(dtype, M, N, K, transB, kblock):
    """The encode and threshold passes of the K-blocked route run on every type and shape; the GEMM with K-block
    prefixes exists for BF16 / FP16 problems made of whole tiles and says so otherwise."""
    from paper_2602_08043_amd import binding as vb
    W = vb.vabft_block_width(dtype)
    A, B = _gen(dtype, M, N, K, transB, 31)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    vg = _session(M, N, K, dtype, transB, kblock)
    e = _emax(dtype, kblock, min(N, W))
    vg.encode(dB)
    vg.threshold(dA, e)
    r = vg.results()
    ob = orc.verify_blocks_k(A, B, dtype, transB, W, kblock, e, full_gemm=False)
    check_pieces(r, ob, dtype, M, N, K, kblock, gemm=False)
    with pytest.raises(vb.VabftError) as ei:
        vg.gemm(dA, dB)
    assert ei.value.status == vb.VABFT_EUNSUPPORTED
