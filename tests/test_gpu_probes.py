"""The measurement aids of the library (not steps of the verified path): the register-only matrix-instruction loop
and the read-only / empty kernels that `bench.py` times beside the GEMM and the streaming passes."""
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_mfma_probe_runs_and_counts_its_flops():
    from paper_2602_08043_amd import binding as vb
    out = torch.full((65536,), float("nan"), dtype=torch.float32, device="cuda")
    for dt, per_wave_iter in (("bf16", 64 * 16384), ("f16", 64 * 16384), ("f32", 16 * 4096), ("f64", 16 * 2048)):
        flops = vb.vabft_probe_mfma(dt, 3, out.data_ptr())
        torch.cuda.synchronize()
        assert flops == 256 * 4 * 3 * per_wave_iter
        assert torch.isfinite(out).all()
    with pytest.raises(vb.VabftError):
        vb.vabft_probe_mfma("bf16", 0, out.data_ptr())


def test_read_probe_reads_and_writes_nothing():
    from paper_2602_08043_amd import binding as vb
    buf = torch.randn(1 << 20, dtype=torch.float32, device="cuda")
    ref = buf.clone()
    out = torch.full((4,), 7.0, dtype=torch.float32, device="cuda")
    for nbytes in (buf.numel() * 4, 16 * 1000 + 16, 16, 0):   # whole buffer, a ragged count of pieces, one piece, empty
        vb.vabft_probe_read(buf.data_ptr(), nbytes, out.data_ptr())
    vb.vabft_probe_read(None, 0, out.data_ptr())
    torch.cuda.synchronize()
    assert torch.equal(buf, ref) and torch.equal(out, torch.full_like(out, 7.0))
    with pytest.raises(vb.VabftError):
        vb.vabft_probe_read(buf.data_ptr() + 4, 64, out.data_ptr())   # not 16-byte aligned
