"""Device-buffer plumbing around the C ABI: PyTorch supplies HBM allocations and the
stream handle, nothing else.  All arithmetic happens inside libvabft.so."""
from __future__ import annotations

import ctypes

import numpy as np
import torch

from . import binding as vb

_TORCH_DTYPE = {"f64": torch.float64, "f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16,
                "f8": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}
_OUT_DTYPE = {"f8": "f16", "f8e5m2": "f16"}  # FP8 problems store an FP16 product
_REC_DTYPE = np.dtype([("row", "<i4"), ("col", "<i4"), ("bit", "<i4"), ("pad", "<i4"), ("before", "<f8"),
                       ("after", "<f8")])


def to_device(x: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Storage array (see workloads.py) -> device tensor of the matching torch dtype."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).to(device).view(torch.bfloat16)
    if dtype in ("f8", "f8e5m2"):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint8)).to(device).view(_TORCH_DTYPE[dtype])
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class VerifiedGemm:
    """Buffers of one problem and thin wrappers over the three entry points."""

    def __init__(self, M, N, K, dtype: str, transB=0, device="cuda:0", log_capacity=4096):
        vb.load()
        self.M, self.N, self.K, self.dtype, self.transB = M, N, K, dtype, int(transB)
        self.device = torch.device(device)
        self.problem = vb.make_problem(M, N, K, dtype, transB)
        acc = torch.float64 if dtype == "f64" else torch.float32
        self.acc = acc
        dev = self.device
        self.out_dtype = _OUT_DTYPE.get(dtype, dtype)
        self.C = torch.empty((M, N), dtype=_TORCH_DTYPE[self.out_dtype], device=dev)
        self.Be = torch.empty(K, dtype=acc, device=dev)
        self.bstat = torch.empty((K, 3), dtype=acc, device=dev)
        self.S = torch.empty(3, dtype=torch.float64, device=dev)
        self.astat = torch.empty((M, 3), dtype=acc, device=dev)
        self.expected = torch.empty(M, dtype=acc, device=dev)
        self.T = torch.empty(M, dtype=acc, device=dev)
        self.rowsum = torch.empty(M, dtype=acc, device=dev)
        self.E = torch.empty(M, dtype=acc, device=dev)
        self.flags = torch.empty(M, dtype=torch.int32, device=dev)
        self.nflag = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ninj = torch.zeros(1, dtype=torch.int32, device=dev)
        self.log_capacity = int(log_capacity)
        self.injlog = torch.zeros(max(1, self.log_capacity) * _REC_DTYPE.itemsize, dtype=torch.uint8, device=dev)
        # position-weighted checksum / localisation buffers
        self.Be2 = torch.empty(K, dtype=acc, device=dev)
        self.expected2 = torch.empty(M, dtype=acc, device=dev)
        self.rowsum2 = torch.empty(M, dtype=acc, device=dev)
        self.loc = torch.empty(M, dtype=torch.int32, device=dev)
        self.delta = torch.empty(M, dtype=acc, device=dev)
        self.ncorrected = torch.zeros(1, dtype=torch.int32, device=dev)
        # column-checksum buffers
        self.eA = torch.empty(K, dtype=acc, device=dev)
        self.acolstat = torch.empty((K, 3), dtype=acc, device=dev)
        self.SA = torch.empty(3, dtype=torch.float64, device=dev)
        self.bcolstat = torch.empty((N, 3), dtype=acc, device=dev)
        self.expected_col = torch.empty(N, dtype=acc, device=dev)
        self.T_col = torch.empty(N, dtype=acc, device=dev)
        self.colsum = torch.empty(N, dtype=acc, device=dev)
        self.E_col = torch.empty(N, dtype=acc, device=dev)
        self.colflags = torch.empty(N, dtype=torch.int32, device=dev)
        self.ncolflag = torch.zeros(1, dtype=torch.int32, device=dev)
        # block-wise verification buffers
        self.W = vb.vabft_block_width(dtype)
        self.nblocks = (N + self.W - 1) // self.W
        nb = self.nblocks
        self.Be_blk = torch.empty((nb, K), dtype=acc, device=dev)
        self.S_blk = torch.empty((nb, 3), dtype=torch.float64, device=dev)
        self.expected_blk = torch.empty((nb, M), dtype=acc, device=dev)
        self.T_blk = torch.empty((nb, M), dtype=acc, device=dev)
        self.rowsum_blk = torch.empty((nb, M), dtype=acc, device=dev)
        self.E_blk = torch.empty((nb, M), dtype=acc, device=dev)
        self.blockflags = torch.empty((nb, M), dtype=torch.int32, device=dev)
        self.nblockflag = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ws_bytes = vb.vabft_workspace_bytes(self.problem)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        vb.vabft_workspace_init(self.ws.data_ptr(), self.ws_bytes, self._stream())
        self._list = None

    @staticmethod
    def _stream():
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def encode(self, B: torch.Tensor, defer_S: bool = False):
        """defer_S: leave S1..S3 as partials in the workspace for gemm_fused(..., deferred_S=True)."""
        return vb.vabft_encode(self.problem, B.data_ptr(), self.Be.data_ptr(), self.bstat.data_ptr(),
                               None if defer_S else self.S.data_ptr(), self.ws.data_ptr(), self.ws_bytes,
                               self._stream())

    def threshold(self, A: torch.Tensor, e_max=None, c_sigma=2.5):
        if e_max is None:
            e_max = vb.vabft_default_emax(self.dtype, self.K, self.N)
        self.e_max = e_max
        return vb.vabft_threshold(self.problem, A.data_ptr(), self.Be.data_ptr(), self.S.data_ptr(), e_max, c_sigma,
                                  self.astat.data_ptr(), self.expected.data_ptr(), self.T.data_ptr(), self._stream())

    def make_inject(self, mode=0, faults=None, seed=0, rate=0.0, bit_lo=0, bit_hi=0) -> vb.Inject:
        """mode 1: faults = [(row, col, bit), ...]; mode 2: Bernoulli(seed, rate, bit_lo..bit_hi)."""
        inj = vb.Inject()
        inj.mode = mode
        inj.bit_lo, inj.bit_hi = bit_lo, bit_hi
        inj.seed, inj.rate = seed, rate
        inj.log_capacity = self.log_capacity
        if mode == 1:
            arr = np.asarray(faults, dtype=np.int32).reshape(-1, 3)
            self._list = torch.from_numpy(arr.copy()).to(self.device)
            inj.n_list = arr.shape[0]
            inj.d_list = self._list.data_ptr()
        return inj

    def gemm(self, A: torch.Tensor, B: torch.Tensor, verify=1, inj: vb.Inject | None = None):
        return vb.vabft_gemm_verified(self.problem, A.data_ptr(), B.data_ptr(), self.C.data_ptr(),
                                      self.expected.data_ptr(), self.T.data_ptr(), verify, inj,
                                      self.rowsum.data_ptr(), self.E.data_ptr(), self.flags.data_ptr(),
                                      self.nflag.data_ptr(), self.injlog.data_ptr(), self.ninj.data_ptr(),
                                      self.ws.data_ptr(), self.ws_bytes, self._stream())

    def gemm_fused(self, A: torch.Tensor, B: torch.Tensor, e_max=None, c_sigma=2.5, inj: vb.Inject | None = None,
                   deferred_S: bool = False):
        """A-side pass, GEMM and check in one call (needs encode(B) first; deferred_S after encode(B, defer_S=True))."""
        if e_max is None:
            e_max = vb.vabft_default_emax(self.dtype, self.K, self.N)
        self.e_max = e_max
        return vb.vabft_gemm_verified_fused(self.problem, A.data_ptr(), B.data_ptr(), self.C.data_ptr(),
                                            self.Be.data_ptr(), None if deferred_S else self.S.data_ptr(), e_max,
                                            c_sigma, self.astat.data_ptr(), self.expected.data_ptr(),
                                            self.T.data_ptr(), inj,
                                            self.rowsum.data_ptr(), self.E.data_ptr(), self.flags.data_ptr(),
                                            self.nflag.data_ptr(), self.injlog.data_ptr(), self.ninj.data_ptr(),
                                            self.ws.data_ptr(), self.ws_bytes, self._stream())

    def run(self, A, B, e_max=None, c_sigma=2.5, inj=None):
        """One pass of the whole path: encode, threshold, verified GEMM (three calls)."""
        self.encode(B)
        self.threshold(A, e_max, c_sigma)
        self.gemm(A, B, 1, inj)

    def run_fused(self, A, B, e_max=None, c_sigma=2.5, inj=None, defer_S: bool = False):
        """One pass of the whole path in two calls: encode, fused threshold + verified GEMM.
        defer_S: S1..S3 travel as partials through the workspace and are folded inside the second call."""
        self.encode(B, defer_S)
        self.gemm_fused(A, B, e_max, c_sigma, inj, deferred_S=defer_S)

    # ---- weighted checksum, localisation, correction ---------------------------------
    def encode_weighted(self, B: torch.Tensor):
        return vb.vabft_encode_weighted(self.problem, B.data_ptr(), self.Be.data_ptr(), self.Be2.data_ptr(),
                                        self.bstat.data_ptr(), self.S.data_ptr(), self.ws.data_ptr(), self.ws_bytes,
                                        self._stream())

    def threshold_weighted(self, A: torch.Tensor, e_max=None, c_sigma=2.5):
        if e_max is None:
            e_max = vb.vabft_default_emax(self.dtype, self.K, self.N)
        self.e_max = e_max
        return vb.vabft_threshold_weighted(self.problem, A.data_ptr(), self.Be.data_ptr(), self.Be2.data_ptr(),
                                           self.S.data_ptr(), e_max, c_sigma, self.astat.data_ptr(),
                                           self.expected.data_ptr(), self.expected2.data_ptr(), self.T.data_ptr(),
                                           self._stream())

    def gemm_weighted(self, A: torch.Tensor, B: torch.Tensor, inj: vb.Inject | None = None):
        return vb.vabft_gemm_verified_weighted(self.problem, A.data_ptr(), B.data_ptr(), self.C.data_ptr(),
                                               self.expected.data_ptr(), self.T.data_ptr(), inj,
                                               self.rowsum.data_ptr(), self.rowsum2.data_ptr(), self.E.data_ptr(),
                                               self.flags.data_ptr(), self.nflag.data_ptr(), self.injlog.data_ptr(),
                                               self.ninj.data_ptr(), self.ws.data_ptr(), self.ws_bytes,
                                               self._stream())

    def locate_correct(self, correct=1):
        return vb.vabft_locate_correct(self.problem, self.C.data_ptr(), self.expected.data_ptr(),
                                       self.expected2.data_ptr(), self.rowsum.data_ptr(), self.rowsum2.data_ptr(),
                                       self.flags.data_ptr(), correct, self.loc.data_ptr(), self.delta.data_ptr(),
                                       self.ncorrected.data_ptr(), self._stream())

    def run_weighted(self, A, B, e_max=None, c_sigma=2.5, inj=None, correct=1):
        """Detect, locate, correct: weighted encode, weighted threshold, weighted verified GEMM,
        then localisation (and correction of the stored C)."""
        self.encode_weighted(B)
        self.threshold_weighted(A, e_max, c_sigma)
        self.gemm_weighted(A, B, inj)
        self.locate_correct(correct)

    # ---- column checksums --------------------------------------------------------------
    def encode_a(self, A: torch.Tensor):
        return vb.vabft_encode_a(self.problem, A.data_ptr(), self.eA.data_ptr(), self.acolstat.data_ptr(),
                                 self.SA.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self._stream())

    def threshold_cols(self, B: torch.Tensor, e_max=None, c_sigma=2.5):
        if e_max is None:
            e_max = vb.vabft_default_emax(self.dtype, self.K, max(self.N, self.M))
        return vb.vabft_threshold_cols(self.problem, B.data_ptr(), self.eA.data_ptr(), self.SA.data_ptr(), e_max,
                                       c_sigma, self.bcolstat.data_ptr(), self.expected_col.data_ptr(),
                                       self.T_col.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self._stream())

    def gemm_rc(self, A: torch.Tensor, B: torch.Tensor, inj: vb.Inject | None = None):
        return vb.vabft_gemm_verified_rc(self.problem, A.data_ptr(), B.data_ptr(), self.C.data_ptr(),
                                         self.expected.data_ptr(), self.T.data_ptr(), self.expected_col.data_ptr(),
                                         self.T_col.data_ptr(), inj, self.rowsum.data_ptr(), self.E.data_ptr(),
                                         self.flags.data_ptr(), self.nflag.data_ptr(), self.colsum.data_ptr(),
                                         self.E_col.data_ptr(), self.colflags.data_ptr(), self.ncolflag.data_ptr(),
                                         self.injlog.data_ptr(), self.ninj.data_ptr(), self.ws.data_ptr(),
                                         self.ws_bytes, self._stream())

    def run_rc(self, A, B, e_max=None, e_max_col=None, c_sigma=2.5, inj=None):
        """Row and column check of one GEMM: both encodes, both threshold passes, one GEMM launch."""
        self.encode(B)
        self.threshold(A, e_max, c_sigma)
        self.encode_a(A)
        self.threshold_cols(B, e_max_col, c_sigma)
        self.gemm_rc(A, B, inj)

    # ---- block-wise verification --------------------------------------------------------
    def encode_blocks(self, B: torch.Tensor):
        return vb.vabft_encode_blocks(self.problem, B.data_ptr(), self.Be_blk.data_ptr(), self.S_blk.data_ptr(),
                                      self.ws.data_ptr(), self.ws_bytes, self._stream())

    def threshold_blocks(self, A: torch.Tensor, e_max=None, c_sigma=2.5):
        if e_max is None:
            e_max = vb.vabft_default_emax(self.dtype, self.K, min(self.N, self.W))
        return vb.vabft_threshold_blocks(self.problem, A.data_ptr(), self.Be_blk.data_ptr(), self.S_blk.data_ptr(),
                                         e_max, c_sigma, self.astat.data_ptr(), self.expected_blk.data_ptr(),
                                         self.T_blk.data_ptr(), self._stream())

    def gemm_blocks(self, A: torch.Tensor, B: torch.Tensor, inj: vb.Inject | None = None):
        return vb.vabft_gemm_verified_blocks(self.problem, A.data_ptr(), B.data_ptr(), self.C.data_ptr(),
                                             self.expected_blk.data_ptr(), self.T_blk.data_ptr(), inj,
                                             self.rowsum_blk.data_ptr(), self.E_blk.data_ptr(),
                                             self.blockflags.data_ptr(), self.nblockflag.data_ptr(),
                                             self.E.data_ptr(), self.flags.data_ptr(), self.nflag.data_ptr(),
                                             self.injlog.data_ptr(), self.ninj.data_ptr(), self.ws.data_ptr(),
                                             self.ws_bytes, self._stream())

    def run_blocks(self, A, B, e_max=None, c_sigma=2.5, inj=None):
        self.encode_blocks(B)
        self.threshold_blocks(A, e_max, c_sigma)
        self.gemm_blocks(A, B, inj)

    # ---- offline (post-quantisation) check ---------------------------------------------
    def check_offline(self, C: torch.Tensor | None = None):
        """Row sums of a stored product (default: this session's C) against expected / T."""
        C = self.C if C is None else C
        return vb.vabft_check_offline(self.problem, C.data_ptr(), self.expected.data_ptr(), self.T.data_ptr(),
                                      self.rowsum.data_ptr(), self.E.data_ptr(), self.flags.data_ptr(),
                                      self.nflag.data_ptr(), self._stream())

    def run_offline(self, A, B, e_max=None, c_sigma=2.5, inj=None):
        """Plain (or fault-injected) GEMM, then the post-hoc check on the stored C with an e_max for
        the output precision."""
        if e_max is None:
            e_max = vb.vabft_default_emax_offline(self.dtype, self.K, self.N)
        self.encode(B)
        self.threshold(A, e_max, c_sigma)
        if inj is None:
            self.gemm(A, B, 0)
        else:
            self.gemm(A, B, 1, inj)  # the injector lives in the verified kernel; its check is overwritten below
        self.check_offline()

    def inject_records(self):
        """Downloaded injection log as a list of (row, col, bit, before, after), sorted."""
        n = int(self.ninj.item())
        m = min(n, self.log_capacity)
        raw = self.injlog.cpu().numpy()[: m * _REC_DTYPE.itemsize].view(_REC_DTYPE)
        recs = sorted((int(r["row"]), int(r["col"]), int(r["bit"]), float(r["before"]), float(r["after"]))
                      for r in raw)
        return n, recs

    def results(self):
        torch.cuda.synchronize(self.device)
        out = {k: getattr(self, k).cpu().numpy() for k in
               ("Be", "bstat", "S", "astat", "expected", "T", "rowsum", "E", "flags", "Be2", "expected2", "rowsum2",
                "loc", "delta", "eA", "acolstat", "SA", "bcolstat", "expected_col", "T_col", "colsum", "E_col",
                "colflags", "Be_blk", "S_blk", "expected_blk", "T_blk", "rowsum_blk", "E_blk", "blockflags")}
        out["nblockflag"] = int(self.nblockflag.item())
        out["ncolflag"] = int(self.ncolflag.item())
        out["ncorrected"] = int(self.ncorrected.item())
        out["nflag"] = int(self.nflag.item())
        out["C"] = to_host(self.C, self.out_dtype)
        return out


class KBlockedGemm:
    """Buffers and thin wrappers of the block-wise route with K split as well (vabft_*_blocks_k): device memory and
    the stream handle only, like VerifiedGemm."""

    def __init__(self, M, N, K, dtype: str, transB=0, kblock=1024, device="cuda:0", log_capacity=256):
        vb.load()
        self.M, self.N, self.K, self.dtype, self.transB, self.kblock = M, N, K, dtype, int(transB), int(kblock)
        self.device = dev = torch.device(device)
        self.problem = vb.make_problem(M, N, K, dtype, transB)
        acc = torch.float64 if dtype == "f64" else torch.float32
        self.W = vb.vabft_block_width(dtype)
        self.nblocks = nb = (N + self.W - 1) // self.W
        self.nkb = nkb = vb.vabft_kblock_count(self.problem, kblock)
        self.out_dtype = _OUT_DTYPE.get(dtype, dtype)
        self.C = torch.empty((M, N), dtype=_TORCH_DTYPE[self.out_dtype], device=dev)
        self.Be_blk_k = torch.empty(nb * K, dtype=acc, device=dev)  # piece b: [nb][len_b] at offset b * nb * kblock
        self.S_blk_k = torch.empty((nkb, nb, 3), dtype=torch.float64, device=dev)
        self.astat_k = torch.empty((nkb, M, 3), dtype=acc, device=dev)
        self.expected_blk_k = torch.empty((nkb, nb, M), dtype=acc, device=dev)
        self.T_blk_k = torch.empty((nkb, nb, M), dtype=acc, device=dev)
        self.rowsum_blk_k = torch.empty((nkb, nb, M), dtype=acc, device=dev)
        self.E_blk_k = torch.empty((nkb, nb, M), dtype=acc, device=dev)
        self.blockflags_k = torch.empty((nkb, nb, M), dtype=torch.int32, device=dev)
        self.nblockflag = torch.zeros(1, dtype=torch.int32, device=dev)
        self.E = torch.empty(M, dtype=acc, device=dev)
        self.flags = torch.empty(M, dtype=torch.int32, device=dev)
        self.nflag = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ninj = torch.zeros(1, dtype=torch.int32, device=dev)
        self.log_capacity = int(log_capacity)
        self.injlog = torch.zeros(max(1, self.log_capacity) * _REC_DTYPE.itemsize, dtype=torch.uint8, device=dev)
        self.ws_bytes = vb.vabft_workspace_bytes_blocks_k(self.problem, kblock)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        vb.vabft_workspace_init(self.ws.data_ptr(), self.ws_bytes, self._stream())
        self._list = None

    _stream = staticmethod(VerifiedGemm._stream)
    make_inject = VerifiedGemm.make_inject
    inject_records = VerifiedGemm.inject_records

    def encode(self, B: torch.Tensor):
        return vb.vabft_encode_blocks_k(self.problem, self.kblock, B.data_ptr(), self.Be_blk_k.data_ptr(),
                                        self.S_blk_k.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self._stream())

    def threshold(self, A: torch.Tensor, e_max=None, c_sigma=2.5):
        if e_max is None:
            e_max = vb.vabft_default_emax(self.dtype, min(self.K, self.kblock), min(self.N, self.W))
        return vb.vabft_threshold_blocks_k(self.problem, self.kblock, A.data_ptr(), self.Be_blk_k.data_ptr(),
                                           self.S_blk_k.data_ptr(), e_max, c_sigma, self.astat_k.data_ptr(),
                                           self.expected_blk_k.data_ptr(), self.T_blk_k.data_ptr(), self._stream())

    def gemm(self, A: torch.Tensor, B: torch.Tensor, inj: vb.Inject | None = None):
        return vb.vabft_gemm_verified_blocks_k(self.problem, self.kblock, A.data_ptr(), B.data_ptr(), self.C.data_ptr(),
                                               self.expected_blk_k.data_ptr(), self.T_blk_k.data_ptr(), inj,
                                               self.rowsum_blk_k.data_ptr(), self.E_blk_k.data_ptr(),
                                               self.blockflags_k.data_ptr(), self.nblockflag.data_ptr(),
                                               self.E.data_ptr(), self.flags.data_ptr(), self.nflag.data_ptr(),
                                               self.injlog.data_ptr(), self.ninj.data_ptr(), self.ws.data_ptr(),
                                               self.ws_bytes, self._stream())

    def run(self, A, B, e_max=None, c_sigma=2.5, inj=None):
        self.encode(B)
        self.threshold(A, e_max, c_sigma)
        self.gemm(A, B, inj)

    def results(self):
        torch.cuda.synchronize(self.device)
        out = {k: getattr(self, k).cpu().numpy() for k in
               ("Be_blk_k", "S_blk_k", "astat_k", "expected_blk_k", "T_blk_k", "rowsum_blk_k", "E_blk_k", "blockflags_k",
                "E", "flags")}
        out["C"] = to_host(self.C, self.out_dtype)
        out["nflag"] = int(self.nflag.item())
        out["nblockflag"] = int(self.nblockflag.item())
        return out
