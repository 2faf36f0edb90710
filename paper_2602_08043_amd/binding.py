"""ctypes binding of libvabft.so: the same entry points as include/vabft.h.

Argument marshalling only.  Every step of the path runs in the HIP kernels of the
library; there is no CPU or PyTorch fallback: if the library is missing, loading
fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_int32, c_int64, c_size_t, c_uint64, c_void_p

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libvabft.so")

VABFT_OK, VABFT_EINVAL, VABFT_EUNSUPPORTED, VABFT_EWORKSPACE, VABFT_EDEVICE = range(5)
VABFT_F64, VABFT_F32, VABFT_F16, VABFT_BF16, VABFT_F8E4M3, VABFT_F8E5M2 = range(6)
DTYPE_CODE = {"f64": VABFT_F64, "f32": VABFT_F32, "f16": VABFT_F16, "bf16": VABFT_BF16, "f8": VABFT_F8E4M3,
              "f8e5m2": VABFT_F8E5M2}

EXPORTS = ("vabft_status_string", "vabft_workspace_bytes", "vabft_workspace_init", "vabft_default_emax",
           "vabft_encode", "vabft_threshold", "vabft_gemm_verified", "vabft_gemm_verified_fused",
           "vabft_encode_weighted", "vabft_threshold_weighted", "vabft_gemm_verified_weighted",
           "vabft_locate_correct", "vabft_default_emax_offline", "vabft_check_offline",
           "vabft_encode_a", "vabft_threshold_cols", "vabft_gemm_verified_rc",
           "vabft_block_width", "vabft_encode_blocks", "vabft_threshold_blocks", "vabft_gemm_verified_blocks",
           "vabft_static_scratch_bytes", "vabft_gemm_verified_fused_static", "vabft_probe_mfma", "vabft_probe_read",
           "vabft_kblock_count", "vabft_workspace_bytes_blocks_k", "vabft_encode_blocks_k",
           "vabft_threshold_blocks_k", "vabft_gemm_verified_blocks_k")


class Problem(Structure):
    _fields_ = [("M", c_int32), ("N", c_int32), ("K", c_int32), ("dtype", c_int32), ("transB", c_int32),
                ("reserved", c_int32), ("lda", c_int64), ("ldb", c_int64), ("ldc", c_int64)]


class Inject(Structure):
    _fields_ = [("mode", c_int32), ("bit_lo", c_int32), ("bit_hi", c_int32), ("n_list", c_int32),
                ("seed", c_uint64), ("rate", c_double), ("d_list", c_void_p), ("log_capacity", c_int32),
                ("reserved", c_int32)]


class InjectRec(Structure):
    _fields_ = [("row", c_int32), ("col", c_int32), ("bit", c_int32), ("pad", c_int32),
                ("before", c_double), ("after", c_double)]


class VabftError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def load(path: str | None = None):
    """Load libvabft.so (built in-tree by paper_2602_08043_amd/build.py)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise ImportError(
            f"{p} not found: the HIP library has not been built. Run "
            "`python -c 'import __graft_entry__ as g; g.build()'` (needs hipcc); there is no fallback path.")
    lib = ctypes.CDLL(p)
    lib.vabft_status_string.restype = c_char_p
    lib.vabft_status_string.argtypes = [ctypes.c_int]
    lib.vabft_workspace_bytes.restype = c_size_t
    lib.vabft_workspace_bytes.argtypes = [POINTER(Problem)]
    lib.vabft_default_emax.restype = c_double
    lib.vabft_default_emax.argtypes = [c_int32, c_int32, c_int32]
    lib.vabft_encode.restype = ctypes.c_int
    lib.vabft_encode.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                 c_void_p]
    lib.vabft_threshold.restype = ctypes.c_int
    lib.vabft_threshold.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_double, c_double, c_void_p,
                                    c_void_p, c_void_p, c_void_p]
    lib.vabft_gemm_verified.restype = ctypes.c_int
    lib.vabft_gemm_verified.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int32,
                                        POINTER(Inject), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_size_t, c_void_p]
    lib.vabft_workspace_init.restype = ctypes.c_int
    lib.vabft_workspace_init.argtypes = [c_void_p, c_size_t, c_void_p]
    lib.vabft_gemm_verified_fused.restype = ctypes.c_int
    lib.vabft_gemm_verified_fused.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                              c_double, c_double, c_void_p, c_void_p, c_void_p, POINTER(Inject),
                                              c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                              c_size_t, c_void_p]
    lib.vabft_probe_read.restype = ctypes.c_int
    lib.vabft_probe_read.argtypes = [c_void_p, c_size_t, c_void_p, c_void_p]
    lib.vabft_probe_mfma.restype = ctypes.c_int
    lib.vabft_probe_mfma.argtypes = [c_int32, c_int32, c_void_p, POINTER(c_double), c_void_p]
    lib.vabft_static_scratch_bytes.restype = c_size_t
    lib.vabft_static_scratch_bytes.argtypes = []
    lib.vabft_gemm_verified_fused_static.restype = ctypes.c_int
    lib.vabft_gemm_verified_fused_static.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p,
                                                     c_void_p, c_double, c_double, c_void_p, c_void_p, c_void_p,
                                                     POINTER(Inject), c_void_p, c_void_p, c_void_p, c_void_p,
                                                     c_void_p, c_void_p, c_void_p]
    lib.vabft_encode_weighted.restype = ctypes.c_int
    lib.vabft_encode_weighted.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_size_t, c_void_p]
    lib.vabft_threshold_weighted.restype = ctypes.c_int
    lib.vabft_threshold_weighted.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_double,
                                             c_double, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.vabft_gemm_verified_weighted.restype = ctypes.c_int
    lib.vabft_gemm_verified_weighted.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                                 POINTER(Inject), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                                 c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.vabft_locate_correct.restype = ctypes.c_int
    lib.vabft_locate_correct.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.vabft_default_emax_offline.restype = c_double
    lib.vabft_default_emax_offline.argtypes = [c_int32, c_int32, c_int32]
    lib.vabft_check_offline.restype = ctypes.c_int
    lib.vabft_check_offline.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_void_p]
    lib.vabft_encode_a.restype = ctypes.c_int
    lib.vabft_encode_a.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                   c_void_p]
    lib.vabft_threshold_cols.restype = ctypes.c_int
    lib.vabft_threshold_cols.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_double, c_double, c_void_p,
                                         c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.vabft_gemm_verified_rc.restype = ctypes.c_int
    lib.vabft_gemm_verified_rc.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_void_p, POINTER(Inject), c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_size_t, c_void_p]
    lib.vabft_block_width.restype = c_int32
    lib.vabft_block_width.argtypes = [c_int32]
    lib.vabft_encode_blocks.restype = ctypes.c_int
    lib.vabft_encode_blocks.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.vabft_threshold_blocks.restype = ctypes.c_int
    lib.vabft_threshold_blocks.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_double, c_double,
                                           c_void_p, c_void_p, c_void_p, c_void_p]
    lib.vabft_kblock_count.restype = c_int32
    lib.vabft_kblock_count.argtypes = [POINTER(Problem), c_int32]
    lib.vabft_workspace_bytes_blocks_k.restype = c_size_t
    lib.vabft_workspace_bytes_blocks_k.argtypes = [POINTER(Problem), c_int32]
    lib.vabft_encode_blocks_k.restype = ctypes.c_int
    lib.vabft_encode_blocks_k.argtypes = [POINTER(Problem), c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                          c_void_p]
    lib.vabft_threshold_blocks_k.restype = ctypes.c_int
    lib.vabft_threshold_blocks_k.argtypes = [POINTER(Problem), c_int32, c_void_p, c_void_p, c_void_p, c_double,
                                             c_double, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.vabft_gemm_verified_blocks_k.restype = ctypes.c_int
    lib.vabft_gemm_verified_blocks_k.argtypes = [POINTER(Problem), c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                                 c_void_p, POINTER(Inject), c_void_p, c_void_p, c_void_p, c_void_p,
                                                 c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                                 c_void_p]
    lib.vabft_gemm_verified_blocks.restype = ctypes.c_int
    lib.vabft_gemm_verified_blocks.argtypes = [POINTER(Problem), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                               POINTER(Inject), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                               c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    if path is None:
        _lib = lib
    return lib


def make_problem(M, N, K, dtype, transB=0, lda=None, ldb=None, ldc=None) -> Problem:
    code = DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)
    return Problem(M, N, K, code, int(transB), 0, K if lda is None else lda,
                   (K if transB else N) if ldb is None else ldb, N if ldc is None else ldc)


def status_string(status: int) -> str:
    return load().vabft_status_string(int(status)).decode()


def vabft_workspace_bytes(p: Problem) -> int:
    return int(load().vabft_workspace_bytes(byref(p)))


def vabft_default_emax(dtype, K: int, N: int) -> float:
    code = DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)
    return float(load().vabft_default_emax(code, K, N))


def _check(rc: int, where: str, check: bool):
    if check and rc != VABFT_OK:
        raise VabftError(rc, where)
    return rc


def vabft_encode(p: Problem, dB, d_Be, d_bstat, d_S, d_workspace, workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_encode(byref(p), dB, d_Be, d_bstat, d_S, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_encode", check)


def vabft_threshold(p: Problem, dA, d_Be, d_S, e_max, c_sigma, d_astat, d_expected, d_T, stream=None,
                    check=True) -> int:
    rc = load().vabft_threshold(byref(p), dA, d_Be, d_S, float(e_max), float(c_sigma), d_astat, d_expected, d_T,
                                stream)
    return _check(rc, "vabft_threshold", check)


def vabft_gemm_verified(p: Problem, dA, dB, dC, d_expected, d_T, verify, inj, d_rowsum, d_E, d_flags, d_nflag,
                        d_injlog, d_ninj, d_workspace, workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_gemm_verified(byref(p), dA, dB, dC, d_expected, d_T, int(verify),
                                    byref(inj) if inj is not None else None, d_rowsum, d_E, d_flags, d_nflag,
                                    d_injlog, d_ninj, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_gemm_verified", check)


def vabft_workspace_init(d_workspace, workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_workspace_init(d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_workspace_init", check)


def vabft_gemm_verified_fused(p: Problem, dA, dB, dC, d_Be, d_S, e_max, c_sigma, d_astat, d_expected, d_T, inj,
                              d_rowsum, d_E, d_flags, d_nflag, d_injlog, d_ninj, d_workspace, workspace_bytes,
                              stream=None, check=True) -> int:
    rc = load().vabft_gemm_verified_fused(byref(p), dA, dB, dC, d_Be, d_S, float(e_max), float(c_sigma), d_astat,
                                          d_expected, d_T, byref(inj) if inj is not None else None, d_rowsum, d_E,
                                          d_flags, d_nflag, d_injlog, d_ninj, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_gemm_verified_fused", check)


def vabft_probe_mfma(dtype: str, iters: int, d_out, stream=None) -> float:
    """One launch of the register-only matrix-instruction loop; returns the launch's flop count."""
    flops = c_double(0.0)
    rc = load().vabft_probe_mfma(DTYPE_CODE[dtype], int(iters), d_out, byref(flops), stream)
    _check(rc, "vabft_probe_mfma", True)
    return float(flops.value)


def vabft_probe_read(d_buf, nbytes: int, d_out, stream=None) -> None:
    """One launch of the read-only kernel over nbytes at d_buf (nbytes < 16: an empty kernel)."""
    _check(load().vabft_probe_read(d_buf, int(nbytes), d_out, stream), "vabft_probe_read", True)


def vabft_static_scratch_bytes() -> int:
    return int(load().vabft_static_scratch_bytes())


def vabft_gemm_verified_fused_static(p: Problem, dA, dB, dC, d_Be, d_S, e_max, c_sigma, d_astat, d_expected, d_T,
                                     inj, d_rowsum, d_E, d_flags, d_nflag, d_injlog, d_ninj, stream=None,
                                     check=True) -> int:
    rc = load().vabft_gemm_verified_fused_static(byref(p), dA, dB, dC, d_Be, d_S, float(e_max), float(c_sigma),
                                                 d_astat, d_expected, d_T, byref(inj) if inj is not None else None,
                                                 d_rowsum, d_E, d_flags, d_nflag, d_injlog, d_ninj, stream)
    return _check(rc, "vabft_gemm_verified_fused_static", check)


def vabft_encode_weighted(p: Problem, dB, d_Be, d_Be2, d_bstat, d_S, d_workspace, workspace_bytes, stream=None,
                          check=True) -> int:
    rc = load().vabft_encode_weighted(byref(p), dB, d_Be, d_Be2, d_bstat, d_S, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_encode_weighted", check)


def vabft_threshold_weighted(p: Problem, dA, d_Be, d_Be2, d_S, e_max, c_sigma, d_astat, d_expected, d_expected2, d_T,
                             stream=None, check=True) -> int:
    rc = load().vabft_threshold_weighted(byref(p), dA, d_Be, d_Be2, d_S, float(e_max), float(c_sigma), d_astat,
                                         d_expected, d_expected2, d_T, stream)
    return _check(rc, "vabft_threshold_weighted", check)


def vabft_gemm_verified_weighted(p: Problem, dA, dB, dC, d_expected, d_T, inj, d_rowsum, d_rowsum2, d_E, d_flags,
                                 d_nflag, d_injlog, d_ninj, d_workspace, workspace_bytes, stream=None,
                                 check=True) -> int:
    rc = load().vabft_gemm_verified_weighted(byref(p), dA, dB, dC, d_expected, d_T,
                                             byref(inj) if inj is not None else None, d_rowsum, d_rowsum2, d_E,
                                             d_flags, d_nflag, d_injlog, d_ninj, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_gemm_verified_weighted", check)


def vabft_locate_correct(p: Problem, dC, d_expected, d_expected2, d_rowsum, d_rowsum2, d_flags, correct, d_loc,
                         d_delta, d_ncorrected, stream=None, check=True) -> int:
    rc = load().vabft_locate_correct(byref(p), dC, d_expected, d_expected2, d_rowsum, d_rowsum2, d_flags,
                                     int(correct), d_loc, d_delta, d_ncorrected, stream)
    return _check(rc, "vabft_locate_correct", check)


def vabft_default_emax_offline(dtype, K: int, N: int) -> float:
    code = DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)
    return float(load().vabft_default_emax_offline(code, K, N))


def vabft_check_offline(p: Problem, dC, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, stream=None,
                        check=True) -> int:
    rc = load().vabft_check_offline(byref(p), dC, d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag, stream)
    return _check(rc, "vabft_check_offline", check)


def vabft_encode_a(p: Problem, dA, d_eA, d_acolstat, d_SA, d_workspace, workspace_bytes, stream=None,
                   check=True) -> int:
    rc = load().vabft_encode_a(byref(p), dA, d_eA, d_acolstat, d_SA, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_encode_a", check)


def vabft_threshold_cols(p: Problem, dB, d_eA, d_SA, e_max, c_sigma, d_bcolstat, d_expected_col, d_Tcol, d_workspace,
                         workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_threshold_cols(byref(p), dB, d_eA, d_SA, float(e_max), float(c_sigma), d_bcolstat,
                                     d_expected_col, d_Tcol, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_threshold_cols", check)


def vabft_gemm_verified_rc(p: Problem, dA, dB, dC, d_expected, d_T, d_expected_col, d_Tcol, inj, d_rowsum, d_E,
                           d_flags, d_nflag, d_colsum, d_Ecol, d_colflags, d_ncolflag, d_injlog, d_ninj, d_workspace,
                           workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_gemm_verified_rc(byref(p), dA, dB, dC, d_expected, d_T, d_expected_col, d_Tcol,
                                       byref(inj) if inj is not None else None, d_rowsum, d_E, d_flags, d_nflag,
                                       d_colsum, d_Ecol, d_colflags, d_ncolflag, d_injlog, d_ninj, d_workspace,
                                       workspace_bytes, stream)
    return _check(rc, "vabft_gemm_verified_rc", check)


def vabft_block_width(dtype) -> int:
    code = DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)
    return int(load().vabft_block_width(code))


def vabft_encode_blocks(p: Problem, dB, d_Be_blk, d_S_blk, d_workspace, workspace_bytes, stream=None,
                        check=True) -> int:
    rc = load().vabft_encode_blocks(byref(p), dB, d_Be_blk, d_S_blk, d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_encode_blocks", check)


def vabft_threshold_blocks(p: Problem, dA, d_Be_blk, d_S_blk, e_max, c_sigma, d_astat, d_expected_blk, d_T_blk,
                           stream=None, check=True) -> int:
    rc = load().vabft_threshold_blocks(byref(p), dA, d_Be_blk, d_S_blk, float(e_max), float(c_sigma), d_astat,
                                       d_expected_blk, d_T_blk, stream)
    return _check(rc, "vabft_threshold_blocks", check)


def vabft_kblock_count(p: Problem, kblock: int) -> int:
    return int(load().vabft_kblock_count(byref(p), int(kblock)))


def vabft_workspace_bytes_blocks_k(p: Problem, kblock: int) -> int:
    return int(load().vabft_workspace_bytes_blocks_k(byref(p), int(kblock)))


def vabft_encode_blocks_k(p: Problem, kblock, dB, d_Be_blk_k, d_S_blk_k, d_workspace, workspace_bytes, stream=None,
                          check=True) -> int:
    rc = load().vabft_encode_blocks_k(byref(p), int(kblock), dB, d_Be_blk_k, d_S_blk_k, d_workspace, workspace_bytes,
                                      stream)
    return _check(rc, "vabft_encode_blocks_k", check)


def vabft_threshold_blocks_k(p: Problem, kblock, dA, d_Be_blk_k, d_S_blk_k, e_max, c_sigma, d_astat_k,
                             d_expected_blk_k, d_T_blk_k, stream=None, check=True) -> int:
    rc = load().vabft_threshold_blocks_k(byref(p), int(kblock), dA, d_Be_blk_k, d_S_blk_k, float(e_max),
                                         float(c_sigma), d_astat_k, d_expected_blk_k, d_T_blk_k, stream)
    return _check(rc, "vabft_threshold_blocks_k", check)


def vabft_gemm_verified_blocks_k(p: Problem, kblock, dA, dB, dC, d_expected_blk_k, d_T_blk_k, inj, d_rowsum_blk_k,
                                 d_E_blk_k, d_blockflags_k, d_nblockflag, d_E, d_flags, d_nflag, d_injlog, d_ninj,
                                 d_workspace, workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_gemm_verified_blocks_k(byref(p), int(kblock), dA, dB, dC, d_expected_blk_k, d_T_blk_k,
                                             byref(inj) if inj is not None else None, d_rowsum_blk_k, d_E_blk_k,
                                             d_blockflags_k, d_nblockflag, d_E, d_flags, d_nflag, d_injlog, d_ninj,
                                             d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_gemm_verified_blocks_k", check)


def vabft_gemm_verified_blocks(p: Problem, dA, dB, dC, d_expected_blk, d_T_blk, inj, d_rowsum_blk, d_E_blk,
                               d_blockflags, d_nblockflag, d_E, d_flags, d_nflag, d_injlog, d_ninj, d_workspace,
                               workspace_bytes, stream=None, check=True) -> int:
    rc = load().vabft_gemm_verified_blocks(byref(p), dA, dB, dC, d_expected_blk, d_T_blk,
                                           byref(inj) if inj is not None else None, d_rowsum_blk, d_E_blk,
                                           d_blockflags, d_nblockflag, d_E, d_flags, d_nflag, d_injlog, d_ninj,
                                           d_workspace, workspace_bytes, stream)
    return _check(rc, "vabft_gemm_verified_blocks", check)
