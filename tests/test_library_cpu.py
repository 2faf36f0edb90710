"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
include/vabft.h declares, and rejects bad arguments before launching anything."""
import os
import re

import pytest

from paper_2602_08043_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(vb.LIB_PATH):
        import __graft_entry__ as ge
        ge.build()
    return vb.load()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "vabft.h")).read()
    declared = set(re.findall(r"\b(vabft_[a-z_]+)\s*\(", header))
    assert declared == set(vb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_header():
    import ctypes
    assert ctypes.sizeof(vb.Problem) == 48
    assert ctypes.sizeof(vb.Inject) == 48
    assert ctypes.sizeof(vb.InjectRec) == 32
    assert vb.Problem.lda.offset == 24 and vb.Inject.seed.offset == 16 and vb.Inject.d_list.offset == 32


def test_status_strings_and_default_emax(lib):
    assert vb.status_string(0) == "ok"
    assert "workspace" in vb.status_string(vb.VABFT_EWORKSPACE)
    # larger of the paper's GPU law and the MI355X-calibrated law, n = max(K, N)
    for n in (128, 512, 4096, 8192, 65536):
        paper, meas = 5.0e-9 * n ** 0.5 + 1.2e-7, 3.0e-9 * n ** 0.5 + 4.2e-7
        assert vb.vabft_default_emax("bf16", n, n) == pytest.approx(max(paper, meas))
        paper, meas = 1.0e-17 * n ** 0.5 + 2.5e-16, 8.0e-18 * n ** 0.5 + 7.0e-16
        assert vb.vabft_default_emax("f64", n, n) == pytest.approx(max(paper, meas))
    assert vb.vabft_default_emax("f16", 4096, 11008) == vb.vabft_default_emax("f32", 11008, 4096)


def test_default_emax_keeps_its_margin_over_the_calibration_table(lib):
    """Every row of the committed calibration table (the paper's protocol run with this library's kernels on
    MI355X; the '+20 %' column is the protocol's own margin): the default lies at least 25 % above it."""
    import os
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles",
                        "emax_calibration_mi355x.md")
    rows = 0
    with open(path) as f:
        for line in f:
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) < 7 or cells[0] not in ("bf16", "f16", "f32", "f64", "f8", "f8e5m2"):
                continue
            dtype, n, plus20 = cells[0], int(cells[2]), float(cells[6])
            assert vb.vabft_default_emax(dtype, n, n) >= 1.25 * plus20, line
            rows += 1
    assert rows >= 40


def test_workspace_bytes(lib):
    p = vb.make_problem(4096, 4096, 4096, "bf16")
    assert vb.vabft_workspace_bytes(p) >= 16 * 4096 * 4
    assert vb.vabft_workspace_bytes(vb.make_problem(0, 4, 4, "f32")) == 0
    assert vb.vabft_workspace_bytes(vb.make_problem(4, 4, 4, 9)) == 0
    pt = vb.make_problem(4096, 11008, 4096, "bf16", transB=1)
    assert vb.vabft_workspace_bytes(pt) >= 86 * 3 * 4096 * 4


def test_rejects_bad_arguments_without_a_gpu(lib):
    p = vb.make_problem(8, 8, 8, "f32")
    # null pointers
    assert vb.vabft_encode(p, None, None, None, None, None, 0, None, check=False) == vb.VABFT_EINVAL
    assert vb.vabft_threshold(p, None, None, None, 1e-6, 2.5, None, None, None, None, check=False) == vb.VABFT_EINVAL
    assert vb.vabft_gemm_verified(p, None, None, None, None, None, 1, None, None, None, None, None, None, None, None, 0,
                                  None, check=False) == vb.VABFT_EINVAL
    # leading dimension smaller than the row, unknown dtype, bad transB
    for bad in (vb.make_problem(8, 8, 8, "f32", lda=4), vb.make_problem(8, 8, 8, 7), vb.make_problem(8, 8, 8, "f32", transB=2),
                vb.make_problem(8, 8, 8, "f32", transB=1, ldb=7), vb.make_problem(-1, 8, 8, "f32")):
        assert vb.vabft_encode(bad, 16, 16, 16, 16, 16, 1 << 20, None, check=False) == vb.VABFT_EINVAL
    # misaligned element pointer
    assert vb.vabft_encode(p, 18, 16, 16, 16, None, 0, None, check=False) == vb.VABFT_EINVAL
    with pytest.raises(vb.VabftError):
        vb.vabft_encode(p, None, None, None, None, None, 0, None)


def test_deferred_fold_arguments_without_a_gpu(lib):
    """d_S may be NULL for vabft_encode and vabft_gemm_verified_fused (the fold of S1..S3 deferred to the fused
    call): the argument checks then go on to the workspace, which is what these calls lack."""
    p = vb.make_problem(256, 256, 256, "f32")
    assert vb.vabft_encode(p, 16, 16, 16, None, None, 0, None, check=False) == vb.VABFT_EWORKSPACE
    assert vb.vabft_encode(p, 16, 16, 16, 24, None, 0, None, check=False) == vb.VABFT_EWORKSPACE
    # a misaligned d_S is still rejected when it is given
    assert vb.vabft_encode(p, 16, 16, 16, 20, None, 0, None, check=False) == vb.VABFT_EINVAL
    args = dict(d_astat=16, d_expected=16, d_T=16, inj=None, d_rowsum=16, d_E=16, d_flags=16, d_nflag=16, d_injlog=16,
                d_ninj=16, d_workspace=None, workspace_bytes=0)
    assert vb.vabft_gemm_verified_fused(p, 16, 16, 16, 16, None, 1e-6, 2.5, check=False, **args) == vb.VABFT_EWORKSPACE
    assert vb.vabft_gemm_verified_fused(p, 16, 16, 16, None, None, 1e-6, 2.5, check=False, **args) in (
        vb.VABFT_EINVAL, vb.VABFT_EWORKSPACE)
    # the workspace covers the partials of S1..S3 (three doubles per 16 rows of B) beside the GEMM's areas
    small, big = vb.make_problem(256, 256, 256, "f32"), vb.make_problem(256, 256, 16384, "f32")
    assert vb.vabft_workspace_bytes(big) - vb.vabft_workspace_bytes(small) >= (16384 - 256) // 16 * 24


def test_bench_refuses_more_than_one_gpu():
    """The path is built and measured on one GPU: bench.py --gpus N with N > 1 exits with a message, before
    anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_missing_library_fails_loudly(tmp_path):
    """There is no CPU fallback: loading a library that is not there raises, with the build command in the text."""
    missing = str(tmp_path / "libvabft_not_built.so")
    with pytest.raises(ImportError) as e:
        vb.load(missing)
    assert "has not been built" in str(e.value) and "no fallback" in str(e.value)


def test_asm_lint_flags_the_hazards_it_is_built_for():
    """The build-time hazard pass on the generated assembly of the inline-assembly kernels: each of its three
    rules fires on a planted case and stays quiet on the padded form of the same sequence."""
    from paper_2602_08043_amd import asm_lint

    def kernel(body):
        return "_ZN5vabft18gemm16_fast_kernelIxEEv:\n" + body + "\n\ts_endpgm\n"

    asm = lambda text: "\t;;#ASMSTART\n\t" + text + "\n\t;;#ASMEND\n"
    # a scalar base written by the vector ALU and read by a load from assembly within five wait states
    bad = kernel("\tv_readfirstlane_b32 s4, v1\n" + asm("global_load_lds_dwordx4 v2, s[4:5] offset:0"))
    good = kernel("\tv_readfirstlane_b32 s4, v1\n\ts_nop 4\n" + asm("global_load_lds_dwordx4 v2, s[4:5] offset:0"))
    assert asm_lint.lint(bad) and not asm_lint.lint(good)
    # ... the same for a plain global load issued from assembly
    bad = kernel("\tv_readfirstlane_b32 s6, v1\n" + asm("global_load_dword v3, v2, s[6:7]"))
    good = kernel("\tv_readfirstlane_b32 s6, v1\n\ts_nop 4\n" + asm("global_load_dword v3, v2, s[6:7]"))
    assert asm_lint.lint(bad) and not asm_lint.lint(good)
    # the load directly behind the move that sets M0
    bad = kernel(asm("s_mov_b32 m0, s9") + asm("global_load_lds_dwordx4 v2, s[4:5] offset:0"))
    good = kernel(asm("s_mov_b32 m0, s9") + asm("v_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[8:11], a[0:3]") +
                  asm("global_load_lds_dwordx4 v2, s[4:5] offset:0"))
    assert asm_lint.lint(bad) and not asm_lint.lint(good)
    # an operand of an MFMA from assembly written by the vector ALU within four wait states
    bad = kernel("\tv_cndmask_b32_e32 v4, v20, v21, vcc\n" + asm("v_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[8:11], a[0:3]"))
    good = kernel("\tv_cndmask_b32_e32 v4, v20, v21, vcc\n\ts_nop 4\n" +
                  asm("v_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[8:11], a[0:3]"))
    assert asm_lint.lint(bad) and not asm_lint.lint(good)
