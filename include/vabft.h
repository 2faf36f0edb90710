/*
 * vabft.h - C ABI of the V-ABFT verified-GEMM hot path for AMD MI355X (gfx950).
 *
 * The library computes C = A x B on the matrix cores with the fused row-checksum
 * verification of ABFT (paper section 2.2, "ABFT for Matrix Multiplication") and
 * the variance-based adaptive threshold of V-ABFT (section 3.4 boxed T_bound,
 * Algorithm 1, section 3.5 extrema-variance bound).
 *
 * Conventions common to every entry point
 *   - Pointers whose name starts with d_ / dA / dB / dC are DEVICE pointers owned by
 *     the caller; everything else is a host pointer read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every
 *     call only enqueues work on that stream: it never synchronises, allocates or
 *     frees device memory.
 *   - Matrices are row-major with leading dimensions in ELEMENTS.
 *       A: M x K (lda >= K);  C: M x N (ldc >= N)
 *       B: transB == 0 -> K x N (ldb >= N);  transB == 1 -> stored N x K (ldb >= K),
 *          the layout in which a linear layer keeps its weight.
 *   - Element type `dtype` applies to A, B and C.  The accumulator type ("acc") is
 *     double for VABFT_F64 and float otherwise (section 3.6: low-precision inputs are
 *     accumulated in FP32 and verified before output quantisation).  Vectors
 *     described as "acc" have that element type.
 *   - bf16 is the upper half of an IEEE binary32 word; conversions from the
 *     accumulator round to nearest even.
 *   - Return value: a vabft_status.  Argument errors are detected on the host before
 *     anything is launched (null pointer, non-positive size, leading dimension
 *     smaller than the row length, unknown dtype, workspace too small).
 *   - Calls that share a workspace must be ordered on one stream.  The head of the
 *     workspace holds arrival counters that must be zero when a call starts: zero-fill the
 *     workspace once after allocating it (vabft_workspace_init, or any fill); every call
 *     leaves the counters zero again.
 *   - A workspace sized for one problem serves every problem with the same dtype, transB, N
 *     and K and at most as many rows M: what vabft_encode leaves in it (the deferred partials
 *     of S1..S3) sits at a place that depends on B's shape only.
 */
#ifndef VABFT_H
#define VABFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VABFT_OK = 0,
    VABFT_EINVAL = 1,       /* bad argument */
    VABFT_EUNSUPPORTED = 2, /* valid but not implemented for this dtype/layout */
    VABFT_EWORKSPACE = 3,   /* workspace missing or smaller than vabft_workspace_bytes */
    VABFT_EDEVICE = 4       /* the HIP runtime reported an error at launch */
} vabft_status;

/* VABFT_F8E4M3, VABFT_F8E5M2: A and B are OCP FP8 (one byte per element, both in the same encoding), the
 * accumulator is FP32 and C is FP16 ("FP8 inputs -> FP32 accumulation -> FP16 output", section 3.6, which names
 * both encodings).  Every entry point takes these types for any shape and either layout of B.  Problems made of
 * whole 256 x 256 x 256 tiles with 16-byte aligned rows and B stored N x K (transB = 1) run on the FP8 matrix
 * instruction; all others run on the guarded kernel, which widens the operands to FP16 on load (exact) and
 * multiplies them with the FP16 matrix instruction: the same products, the same FP32 accumulation. */
typedef enum { VABFT_F64 = 0, VABFT_F32 = 1, VABFT_F16 = 2, VABFT_BF16 = 3, VABFT_F8E4M3 = 4, VABFT_F8E5M2 = 5 } vabft_dtype;

typedef struct {
    int32_t M, N, K;
    int32_t dtype;  /* vabft_dtype of A, B and C (C is FP16 for the FP8 types) */
    int32_t transB; /* 0: B is K x N row-major; 1: B is stored N x K row-major */
    int32_t reserved;
    int64_t lda, ldb, ldc; /* leading dimensions in elements */
} vabft_problem;

/* Fault injector (section 6.1 "Error injection": single bit flips).  The flip is applied
 * to the accumulator word of C[i][j] after the K loop, before the row sum and before
 * output quantisation; the corrupted value is also what is stored to C.
 *   mode 0: off.
 *   mode 1: explicit list: d_list holds n_list int32 triples (row, col, bit).
 *   mode 2: Bernoulli: element e = i*N + j draws z = splitmix64(seed + (e+1)*0x9E3779B97F4A7C15)
 *           (the e-th output of the splitmix64 stream seeded with `seed`); it is hit iff
 *           (z >> 11) < floor(rate * 2^53); the flipped bit is
 *           bit_lo + (z & 0x7FF) % (bit_hi - bit_lo + 1).
 * Bits are numbered from the least significant bit of the accumulator word (0..31 for
 * float, 0..63 for double). */
typedef struct {
    int32_t mode;
    int32_t bit_lo, bit_hi; /* mode 2 */
    int32_t n_list;         /* mode 1 */
    uint64_t seed;          /* mode 2 */
    double rate;            /* mode 2: probability per element, 0 <= rate <= 1 */
    const int32_t* d_list;  /* mode 1: device pointer, 3 * n_list int32 */
    int32_t log_capacity;   /* records d_injlog can hold */
    int32_t reserved;
} vabft_inject;

typedef struct {
    int32_t row, col, bit, pad;
    double before, after; /* accumulator value before / after the flip */
} vabft_inject_rec;

const char* vabft_status_string(int status);

/* Bytes of device scratch that vabft_encode and vabft_gemm_verified need for this
 * problem (0 is never returned for a valid problem; returns 0 for an invalid one). */
size_t vabft_workspace_bytes(const vabft_problem* p);

/* Zero-fill a freshly allocated workspace (a small fill kernel on `stream`; safe to capture
 * in a HIP graph).  Needed once per allocation, before the first vabft_gemm_verified*. */
int vabft_workspace_init(void* d_workspace, size_t workspace_bytes, void* stream);

/* Recommended e_max for a check made on accumulator values (section 3.6), with n = max(K, N):
 * the larger of the paper's GPU law (table "Recommended e_max across platforms":
 * 5.0e-9*sqrt(n)+1.2e-7 for a float accumulator, 1.0e-17*sqrt(n)+2.5e-16 for double) and the
 * law measured on MI355X with this library's kernels by the paper's calibration protocol
 * (3.0e-9*sqrt(n)+4.2e-7, resp. 8.0e-18*sqrt(n)+7.0e-16: at least 25 % above every value that
 * protocol produced, its own 20 % margin included).  FP8 inputs: the constant 6.5e-6 measured
 * the same way (the FP8 matrix instruction accumulates its 64-term dot products with less than FP32
 * precision). */
double vabft_default_emax(int32_t dtype, int32_t K, int32_t N);

/* Checksum encode and B-side statistics (section 2.2 Eq. for r1 and the encoded matrix
 * B^r; Algorithm 1, loop over k).  One streaming pass over B.
 *   d_Be    [K] acc : Be[k] = sum_n B[k][n]                (the column B r1)
 *   d_bstat [3K] acc: (max, min, mean) of row k of the logical K x N matrix, k-major
 *   d_S     [3] double: S1 = sum_k |mu_Bk|, S2 = sum_k sigma_Bk^2, S3 = sum_k mu_Bk^2 with
 *           sigma_Bk^2 = max(0, (max - mu)(mu - min))      (section 3.5 theorem)
 * Results are bit-reproducible from run to run (no floating-point atomics).  The aggregates are
 * folded by the last workgroup to finish (partials and an arrival counter in the workspace), so
 * the call needs the workspace (vabft_workspace_bytes, zero-filled once) for either layout of B.
 * d_S may be NULL: then the fold is deferred -- S1..S3 stay as the per-workgroup partials in the
 * workspace, where they remain valid until the next encode call (vabft_encode, vabft_encode_weighted,
 * vabft_encode_a) on that workspace, for GEMMs with any number of rows M (the workspace sized for the
 * largest of them; every region of the workspace that outlives a call sits at a place that depends on the
 * shape of B only, for up to a million rows), and
 * vabft_gemm_verified_fused called with d_S = NULL folds them itself (same order, same bits).
 * This takes the arrival-counter round trips out of the encode's tail. */
int vabft_encode(const vabft_problem* p, const void* dB, void* d_Be, void* d_bstat, double* d_S,
                 void* d_workspace, size_t workspace_bytes, void* stream);

/* A-side statistics, expected checksum and threshold (Algorithm 1 for every row m;
 * section 2.2 C^{r1} = A (B r1)).  One streaming pass over A.
 *   d_astat    [3M] acc: (max, min, mean) of row m of A
 *   d_expected [M] acc : sum_k A[m][k] * Be[k], accumulated in acc
 *   d_T        [M] acc : e_max * (T_det + T_var23 + T_var4), evaluated in double
 * e_max > 0 and c_sigma >= 0 are the "precision parameters" of Algorithm 1
 * (c_sigma = 2.5 in the paper). */
int vabft_threshold(const vabft_problem* p, const void* dA, const void* d_Be, const double* d_S,
                    double e_max, double c_sigma, void* d_astat, void* d_expected, void* d_T,
                    void* stream);

/* GEMM on the matrix cores with the fused check (section 2.2 Eq. abft-check and the
 * verification difference E_i; section 3.6 "Online (Fused Kernel) ABFT").
 *   verify == 0: plain C = A x B from the same kernel with the check compiled out;
 *                d_expected, d_T, d_rowsum, d_E, d_flags, d_nflag and inj may be NULL.
 *   verify == 1: additionally
 *     d_rowsum [M] acc : sum_j acc[i][j] taken on the accumulator tile before quantisation,
 *                        partial sums combined in a fixed order
 *     d_E      [M] acc : expected[i] - rowsum[i]
 *     d_flags  [M] int32: !( |E_i| <= T_i )   (equals |E_i| > T_i for finite values and
 *                        also flags NaN / Inf row sums)
 *     d_nflag  [1] int32: number of flagged rows
 *   inj (host pointer, may be NULL = off): fault injector; d_injlog / d_ninj receive up to
 *   inj->log_capacity records and the number of flips applied (which may exceed the
 *   capacity; records beyond it are dropped).  Record order is unspecified.
 * dC [M x N] receives the product rounded to `dtype`. */
int vabft_gemm_verified(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                        const void* d_expected, const void* d_T, int32_t verify,
                        const vabft_inject* inj, void* d_rowsum, void* d_E, int32_t* d_flags,
                        int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                        void* d_workspace, size_t workspace_bytes, void* stream);

/* The same check with the A-side pass of Algorithm 1 folded into the GEMM launch: one call
 * computes what vabft_threshold followed by vabft_gemm_verified(verify = 1) computes
 * (Algorithm 1 for every row of A; section 2.2 C^{r1} = A (B r1); Eq. abft-check), reading A
 * once.  Inputs d_Be / d_S come from vabft_encode (d_S = NULL: the preceding vabft_encode on this
 * workspace was called with d_S = NULL and its partials are folded here; without such a call the
 * thresholds are undefined); e_max, c_sigma as in vabft_threshold.
 * Outputs: d_astat [3M], d_expected [M], d_T [M] (as vabft_threshold) and d_rowsum, d_E,
 * d_flags, d_nflag, dC, injection log (as vabft_gemm_verified).  For BF16 / FP16 problems made
 * of whole 256 x 256 x 128 tiles (FP8: 256 x 256 x 256, B stored N x K), and FP32 / FP64 problems
 * made of whole 128 x 128 x 16 tiles,
 * with 16-byte aligned rows the statistics ride on the operand tiles inside the GEMM kernel
 * and the compare-and-flag step runs in the last workgroup of each row block (a single
 * launch); other problems run the two passes back to back.  The
 * summation order of the A-side sums differs between the two routes (both are fixed and
 * bit-reproducible). */
int vabft_gemm_verified_fused(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                              const void* d_Be, const double* d_S, double e_max, double c_sigma,
                              void* d_astat, void* d_expected, void* d_T, const vabft_inject* inj,
                              void* d_rowsum, void* d_E, int32_t* d_flags, int32_t* d_nflag,
                              vabft_inject_rec* d_injlog, int32_t* d_ninj, void* d_workspace,
                              size_t workspace_bytes, void* stream);

/* The fused call for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as vabft_gemm_verified_fused, but
 * without a workspace argument: the partials and arrival counters live in a fixed array of
 * VABFT_STATIC_SCRATCH_BYTES (16 MiB) of device memory inside the library, one copy per GPU, held until the
 * process ends.  The call allocates nothing and frees nothing.
 *   - d_S must not be NULL (no encode runs on this array, so there are no deferred partials to fold).
 *   - A problem whose workspace need (vabft_workspace_bytes) exceeds the array returns VABFT_EWORKSPACE;
 *     every benchmark configuration fits (the largest, FP16 8192^3, needs 8.4 MB).
 *   - Every call on a GPU shares that GPU's array, which keeps the previous call's contents; the call clears
 *     the arrival counters itself.  Calls that overlap on one GPU (two streams, two threads) race: order them.
 *   - VABFT_EDEVICE if the array's address cannot be obtained on the current device. */
#define VABFT_STATIC_SCRATCH_BYTES (16u << 20)
size_t vabft_static_scratch_bytes(void);
int vabft_gemm_verified_fused_static(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                                     const void* d_Be, const double* d_S, double e_max, double c_sigma,
                                     void* d_astat, void* d_expected, void* d_T, const vabft_inject* inj,
                                     void* d_rowsum, void* d_E, int32_t* d_flags, int32_t* d_nflag,
                                     vabft_inject_rec* d_injlog, int32_t* d_ninj, void* stream);

/* Measurement aid (not a step of the verified path): one launch of a register-only loop of the matrix
 * instruction that the GEMM of `dtype` issues (BF16 / FP16: v_mfma_f32_16x16x32; FP32: 32x32x2; FP64: 16x16x4),
 * 256 workgroups of 4 wavefronts, `iters` iterations, pseudo-random operands.  On N(0,1)-like data the chip
 * sustains a lower clock under matrix load than the one its published peak assumes; the benchmark times this
 * launch and reports the verified GEMM as a fraction of the rate it reaches, beside the published peak.
 *   d_out [65536] float (device): a value per thread, so that the loop is not removed
 *   flops (host): floating-point operations of the launch */
int vabft_probe_mfma(int32_t dtype, int32_t iters, void* d_out, double* flops, void* stream);

/* Measurement aid: one launch of a kernel that only reads `bytes` bytes at d_buf (device, 16-byte aligned;
 * 8192 workgroups of 256 threads, grid-stride 16-byte loads, four in flight per lane) -- what a streaming pass
 * can reach on the chip, to set beside the encode / threshold passes and the 8 TB/s figure.  bytes < 16: an
 * empty kernel (one wavefront that does nothing), whose back-to-back launch time is the floor of any pass.
 *   d_out [16 bytes] (device): never written for ordinary data; keeps the loads alive */
int vabft_probe_read(const void* d_buf, size_t bytes, void* d_out, void* stream);

/* ---- Position-weighted checksum, localisation and correction (section 2.2: r2 = [1..N]^T,
 * C^{r2} = A (B r2), C^{r2'} = C r2, "Error localization and correction") -------------------
 * The three calls below are the weighted forms of vabft_encode, vabft_threshold and
 * vabft_gemm_verified(verify = 1): same arguments, same results, plus one more vector each,
 * produced in the same pass over the data.  All weighted vectors are in the accumulator type. */

/*   d_Be2 [K] acc : Be2[k] = sum_n (n + 1) * B[k][n]       (the column B r2) */
int vabft_encode_weighted(const vabft_problem* p, const void* dB, void* d_Be, void* d_Be2,
                          void* d_bstat, double* d_S, void* d_workspace, size_t workspace_bytes,
                          void* stream);

/*   d_expected2 [M] acc : sum_k A[m][k] * Be2[k]            (C^{r2}) */
int vabft_threshold_weighted(const vabft_problem* p, const void* dA, const void* d_Be,
                             const void* d_Be2, const double* d_S, double e_max, double c_sigma,
                             void* d_astat, void* d_expected, void* d_expected2, void* d_T,
                             void* stream);

/*   d_rowsum2 [M] acc : sum_j (j + 1) * acc[i][j] on the accumulator tile before quantisation
 *                       (C^{r2'}), after the injector if one is given */
int vabft_gemm_verified_weighted(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                                 const void* d_expected, const void* d_T, const vabft_inject* inj,
                                 void* d_rowsum, void* d_rowsum2, void* d_E, int32_t* d_flags,
                                 int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                                 void* d_workspace, size_t workspace_bytes, void* stream);

/* Localise and (correct == 1) correct the error of every flagged row under the paper's
 * single-error-per-row model: D1 = rowsum - expected, D2 = rowsum2 - expected2,
 * column j = D2 / D1 - 1 (linear weights w(k) = k + 1), correction C[i][j] <- C[i][j] - D1.
 *   d_loc   [M] int32: -1 row not flagged; -2 flagged, but D2 / D1 - 1 is not finite, is further
 *                      than 0.25 from an integer, or lies outside 0..N-1 (more than one error in
 *                      the row, or an error too close to the rounding noise of the weighted
 *                      sums): such a row has to be recomputed; otherwise the column j.
 *   d_delta [M] acc  : D1 for flagged rows, 0 otherwise.
 *   d_ncorrected [1] : number of elements rewritten (0 when correct == 0).
 * The correction acts on the stored C: the element is read, converted to the accumulator type,
 * D1 is subtracted and the result is rounded back to `dtype`.  For a 16-bit C the corrupted
 * value was already rounded to 8 (BF16) or 11 (FP16) significant bits, so the corrected
 * element is only as accurate as one unit in the last place of the CORRUPTED value.  Run after
 * vabft_gemm_verified_weighted on the same stream. */
int vabft_locate_correct(const vabft_problem* p, void* dC, const void* d_expected,
                         const void* d_expected2, const void* d_rowsum, const void* d_rowsum2,
                         const int32_t* d_flags, int32_t correct, int32_t* d_loc, void* d_delta,
                         int32_t* d_ncorrected, void* stream);

/* ---- Column checksums (section 2.2: c1 = [1 .. 1], A^c = [A; c1 A], C^{c1} = c1 A B, C^{c1'} = c1 C).
 * A faulty element then raises the flag of its row AND of its column: the intersection localises it
 * without the weighted checksum.  By the symmetry C^T = B^T A^T the column threshold is Algorithm 1 with
 * the roles exchanged: column j of B (K entries) plays the row of A, column k of A (M entries) plays the
 * row of B, M replaces N. */

/* c1 A and the column statistics of A.  One streaming pass over A.
 *   d_eA       [K] acc : sum_m A[m][k]
 *   d_acolstat [3K] acc: (max, min, mean) of column k of A
 *   d_SA       [3] double: S1, S2, S3 of Algorithm 1 formed from the columns of A
 * The call uses the workspace area in which an encode of B with d_S = NULL leaves its partials: such a
 * deferred fold is lost if this call comes between that encode and its fused GEMM. */
int vabft_encode_a(const vabft_problem* p, const void* dA, void* d_eA, void* d_acolstat,
                   double* d_SA, void* d_workspace, size_t workspace_bytes, void* stream);

/* Column statistics of B, expected column checksum and column thresholds.  One pass over B.
 *   d_bcolstat     [3N] acc: (max, min, mean) of column n of the logical K x N matrix
 *   d_expected_col [N] acc : sum_k eA[k] * B[k][n]
 *   d_Tcol         [N] acc : e_max * (T_det + T_var23 + T_var4) with the roles exchanged */
int vabft_threshold_cols(const vabft_problem* p, const void* dB, const void* d_eA,
                         const double* d_SA, double e_max, double c_sigma, void* d_bcolstat,
                         void* d_expected_col, void* d_Tcol, void* d_workspace,
                         size_t workspace_bytes, void* stream);

/* vabft_gemm_verified(verify = 1) plus the column check in the same launch:
 *   d_colsum [N] acc : sum_i acc[i][j] on the accumulator tile before quantisation (after the injector)
 *   d_Ecol [N] acc, d_colflags [N] int32, d_ncolflag [1] int32: as their row counterparts. */
int vabft_gemm_verified_rc(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                           const void* d_expected, const void* d_T, const void* d_expected_col,
                           const void* d_Tcol, const vabft_inject* inj, void* d_rowsum, void* d_E,
                           int32_t* d_flags, int32_t* d_nflag, void* d_colsum, void* d_Ecol,
                           int32_t* d_colflags, int32_t* d_ncolflag, vabft_inject_rec* d_injlog,
                           int32_t* d_ninj, void* d_workspace, size_t workspace_bytes, void* stream);

/* ---- Block-wise verification (section 5.2 "Integration with Block-wise ABFT").  The product is checked
 * in blocks of W = vabft_block_width(dtype) columns (256; 64 for FP32 / FP64): block t holds columns
 * [tW, min(N, (t+1)W)), nblocks = ceil(N / W).  Per block: row statistics of the block of B, Algorithm 1 with
 * the block's width in place of N, block checksums compared on their own; a row's aggregate difference is
 * the sum of its block differences and its flag the OR of its block flags.  K is not split here (the *_k entry
 * points further down split it as well).
 * All block arrays are [nblocks][len] (block-major), in the accumulator type unless stated. */
int32_t vabft_block_width(int32_t dtype);

/*   d_Be_blk [nblocks][K] acc   : Be_t[k] = sum of B[k][n] over the block's columns
 *   d_S_blk  [nblocks][3] double: S1, S2, S3 of Algorithm 1 over the block's columns */
int vabft_encode_blocks(const vabft_problem* p, const void* dB, void* d_Be_blk, double* d_S_blk,
                        void* d_workspace, size_t workspace_bytes, void* stream);

/*   d_astat [3M] acc (as vabft_threshold); d_expected_blk [nblocks][M]: sum_k A[m][k] * Be_t[k];
 *   d_T_blk [nblocks][M]: the block thresholds */
int vabft_threshold_blocks(const vabft_problem* p, const void* dA, const void* d_Be_blk,
                           const double* d_S_blk, double e_max, double c_sigma, void* d_astat,
                           void* d_expected_blk, void* d_T_blk, void* stream);

/* GEMM with the per-block check:
 *   d_rowsum_blk, d_E_blk [nblocks][M] acc; d_blockflags [nblocks][M] int32; d_nblockflag [1] int32;
 *   d_E [M] acc: sum over blocks of E_blk (the full-row difference); d_flags [M]: OR of the block flags;
 *   d_nflag [1]: number of flagged rows. */
int vabft_gemm_verified_blocks(const vabft_problem* p, const void* dA, const void* dB, void* dC,
                               const void* d_expected_blk, const void* d_T_blk,
                               const vabft_inject* inj, void* d_rowsum_blk, void* d_E_blk,
                               int32_t* d_blockflags, int32_t* d_nblockflag, void* d_E,
                               int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog,
                               int32_t* d_ninj, void* d_workspace, size_t workspace_bytes,
                               void* stream);

/* ---- Block-wise verification with K split as well (section 5.2: row statistics "for each block of A and B",
 * the threshold formula per block, tile (M, K, N) = (128, 1024, 256)).  K-block b holds k in
 * [b*kblock, min(K, (b+1)*kblock)), nkb = ceil(K / kblock) = vabft_kblock_count; kblock is a positive multiple of
 * 128.  Piece (b, t) is the product of the K-block of A (all rows) with the (K-block, column block) piece of B,
 * verified on its own: its checksum column, its expected row sums, the row sums of the partial product, and
 * Algorithm 1 with the statistics of the K-block of A's rows and of the piece of B's rows, with (b + 1) * e_max
 * for K-block b (its share is gained on a running accumulator that already holds b blocks, so its rounding error
 * goes with a sum (b + 1) blocks deep).  A row's aggregate
 * difference is the sum of its piece differences and its flag the OR of its piece flags.
 * Arrays are [nkb][nblocks][len] unless stated.  The workspace for these calls is
 * vabft_workspace_bytes_blocks_k bytes (it holds the workspace of the whole problem in front, so the other entry
 * points can share it).
 *   d_Be_blk_k: nkb pieces one after the other, piece b = [nblocks][len_b] acc at element offset b*nblocks*kblock
 *   d_S_blk_k [nkb][nblocks][3] double;  d_astat_k [nkb][3M] acc
 * vabft_encode_blocks_k and vabft_threshold_blocks_k take every type and shape (they run the column-block passes
 * on the K-blocks).  vabft_gemm_verified_blocks_k takes BF16 / FP16 problems made of whole 256 x 256 x 64 tiles
 * with 16-byte aligned rows (VABFT_EUNSUPPORTED otherwise): the kernel leaves the row sums of its accumulator tile
 * at every K-block boundary, in double, and a piece's row sum is the difference of two consecutive ones.  The
 * injector acts on the finished accumulator, i.e. on the last K-block's share. */
int32_t vabft_kblock_count(const vabft_problem* p, int32_t kblock);
size_t vabft_workspace_bytes_blocks_k(const vabft_problem* p, int32_t kblock);
int vabft_encode_blocks_k(const vabft_problem* p, int32_t kblock, const void* dB, void* d_Be_blk_k,
                          double* d_S_blk_k, void* d_workspace, size_t workspace_bytes, void* stream);
int vabft_threshold_blocks_k(const vabft_problem* p, int32_t kblock, const void* dA, const void* d_Be_blk_k,
                             const double* d_S_blk_k, double e_max, double c_sigma, void* d_astat_k,
                             void* d_expected_blk_k, void* d_T_blk_k, void* stream);
int vabft_gemm_verified_blocks_k(const vabft_problem* p, int32_t kblock, const void* dA, const void* dB, void* dC,
                                 const void* d_expected_blk_k, const void* d_T_blk_k,
                                 const vabft_inject* inj, void* d_rowsum_blk_k, void* d_E_blk_k,
                                 int32_t* d_blockflags_k, int32_t* d_nblockflag, void* d_E,
                                 int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog,
                                 int32_t* d_ninj, void* d_workspace, size_t workspace_bytes,
                                 void* stream);

/* ---- Offline (post-hoc) verification (section 3.6 "Verification output precision: Offline vs.
 * Online ABFT"): the check is made on a product that already sits in memory in the output type,
 * whoever computed it.  d_expected / d_T come from vabft_threshold, called with an e_max for the
 * output precision (vabft_default_emax_offline: 2 u_output for BF16 / FP16 outputs, i.e. 2^-7 and
 * 2^-10, the paper's "e_max ~ 2 u_output"; the accumulator-level default for FP32 / FP64).
 *   d_rowsum [M] acc : sum_j C[i][j] over the stored elements, accumulated in acc
 *   d_E, d_flags, d_nflag as in vabft_gemm_verified.
 * One streaming pass over C. */
double vabft_default_emax_offline(int32_t dtype, int32_t K, int32_t N);
int vabft_check_offline(const vabft_problem* p, const void* dC, const void* d_expected,
                        const void* d_T, void* d_rowsum, void* d_E, int32_t* d_flags,
                        int32_t* d_nflag, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VABFT_H */
