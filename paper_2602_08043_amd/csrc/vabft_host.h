// Host-side declarations shared by the translation units of libvabft.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vabft.h"

namespace vabft {

// encode.hip
size_t encode_workspace_bytes(const vabft_problem* p);
int s_partial_count(const vabft_problem* p);  // per-workgroup partials of S1..S3 an encode leaves: [count][3] double
// d_Be2 / d_expected2 may be null (no position-weighted checksum); d_S null: S1..S3 stay as partials in s_partial
int encode_dispatch(const vabft_problem* p, const void* dB, void* d_Be, void* d_Be2, void* d_bstat, double* d_S,
                    double* s_partial, void* ws, int32_t* ticket, hipStream_t st);
// folds the partials an encode left into S[3] (the same fixed order the encode itself uses)
void fold_s_launch(const double* s_partial, int count, double* S, hipStream_t st);
int threshold_dispatch(const vabft_problem* p, const void* dA, const void* d_Be, const void* d_Be2, const double* d_S,
                       double e_max, double c_sigma, void* d_astat, void* d_expected, void* d_expected2, void* d_T,
                       hipStream_t st);
// column checksums (c1 A, per-column thresholds)
size_t cols_workspace_bytes(const vabft_problem* p);
int encode_a_dispatch(const vabft_problem* p, const void* dA, void* d_eA, void* d_acolstat, double* d_SA,
                      double* s_partial, void* ws, int32_t* ticket, hipStream_t st);
int threshold_cols_dispatch(const vabft_problem* p, const void* dB, const void* d_eA, const double* d_SA, double e_max,
                            double c_sigma, void* d_bcolstat, void* d_expected_col, void* d_Tcol, void* ws,
                            hipStream_t st);
// blocks.hip: block-wise verification
int block_width(int dtype);
size_t blocks_workspace_bytes(const vabft_problem* p);
int encode_blocks_dispatch(const vabft_problem* p, const void* dB, void* d_Be_blk, double* d_S_blk, void* ws,
                           hipStream_t st);
int threshold_blocks_dispatch(const vabft_problem* p, const void* dA, const void* d_Be_blk, const double* d_S_blk,
                              double e_max, double c_sigma, void* d_astat, void* d_expected_blk, void* d_T_blk,
                              hipStream_t st);
int finalize_blocks_dispatch(const vabft_problem* p, const void* rowpart, const void* d_expected_blk,
                             const void* d_T_blk, void* d_rowsum_blk, void* d_E_blk, int32_t* d_blockflags, void* d_E,
                             int32_t* d_flags, int32_t* d_nflag, int32_t* d_nblockflag, hipStream_t st);
int finalize_blocks_k_dispatch(const vabft_problem* p, int nkb, const double* kprefix, const void* d_expected_blk,
                               const void* d_T_blk, void* d_rowsum_blk, void* d_E_blk, int32_t* d_blockflags,
                               void* d_E, int32_t* d_flags, int32_t* d_nflag, int32_t* d_nblockflag, hipStream_t st);
int check_offline_dispatch(const vabft_problem* p, const void* dC, const void* d_expected, const void* d_T,
                           void* d_rowsum, void* d_E, int32_t* d_flags, int32_t* d_nflag, hipStream_t st);

// gemm*.hip
struct InjectArgs {
    int32_t mode;
    int32_t bit_lo, bit_span;
    int32_t n_list;
    uint64_t seed;
    uint64_t hit_limit;  // floor(rate * 2^53)
    const int32_t* d_list;
    int32_t log_capacity;
    vabft_inject_rec* d_log;
    int32_t* d_ninj;
};

struct GemmArgs {
    const void* A;
    const void* B;
    void* C;
    int32_t M, N, K;
    int64_t lda, ldb, ldc;
    int32_t tiles_m, tiles_n;
    int32_t a_vec_ok, b_vec_ok, c_vec_ok;
    void* rowpart;    // [tiles_n][M] acc: per-tile-column partial row sums
    int32_t* d_nflag; // number of flagged rows
    InjectArgs inj;
    // in-kernel compare-and-flag (whole-tile kernels): the last workgroup to finish a
    // tile-row combines the partials of that row block
    const void* expected;  // [M] acc: input, or output when fused_stats
    const void* T;         // [M] acc: input, or output when fused_stats
    void* rowsum;          // [M] acc
    void* E;               // [M] acc
    int32_t* flags;        // [M]
    int32_t* tickets;      // [tiles_m] arrival counters, then (8-byte aligned) one 64-bit word:
                           // finished row blocks << 32 | flagged rows; all zero between launches
    // fused A-side statistics (Algorithm 1 for the rows of A, inside the GEMM)
    int32_t fused_stats;
    const void* Be;   // [K] acc
    const double* S;  // [3]; null: fold s_partial[s_nparts][3] (left by an encode with a deferred fold)
    const double* s_partial;
    int32_t s_nparts;
    double e_max, c_sigma;
    void* astat;      // [M][3] acc, output
    void* apart;      // [tiles_n][4][M] acc: per-K-slice (sum, dot, max, min) of the rows of A (fused_stats)
    // position-weighted row sums C r2 (kernel modes 2 and 3)
    void* rowpart2;   // partials, same shape as rowpart
    void* rowsum2;    // [M] acc, output; may be null
    // column sums c1 C (kernel modes 2 and 4): [tiles_m][N] acc partials (wide kernels: [2 * tiles_m][N])
    void* colpart;
    int32_t* d_ncolflag;  // zeroed by the GEMM kernel for the column compare that follows it; may be null
    // block-wise check: the kernels only leave their partial row sums; a kernel of its own compares per block
    int32_t block_mode;
    int32_t* d_nblockflag;  // block mode: zeroed (with d_nflag) by the GEMM kernel for the compare that follows
    // block-wise check with K split as well (kernel modes 6 and 7 of the 16-bit whole-tile kernel): the row sums of
    // the accumulator tile taken every kblock_tiles k-tiles, in double
    double* kprefix;        // [K-blocks][2 * tiles_n][M]: prefix row sums (one per wavefront column of a tile-column)
    int32_t kblock_tiles;   // k-tiles (of 64) per K-block; even
};

size_t gemm_workspace_bytes(const vabft_problem* p);
struct FusedArgs {  // non-null d_Be selects the fused A-side path
    const void* d_Be;
    const double* d_S;  // null: S1..S3 are still the partials of the preceding encode
    double e_max, c_sigma;
    void* d_astat;
};
// d_rowsum2 non-null selects the kernels that also form the position-weighted row sums; cols non-null those
// that also form the column sums and compares them
struct BlockArgs {
    const void* d_expected_blk;  // [nblocks][M] acc
    const void* d_T_blk;         // [nblocks][M] acc
    void* d_rowsum_blk;          // [nblocks][M] acc
    void* d_E_blk;               // [nblocks][M] acc
    int32_t* d_blockflags;       // [nblocks][M]
    int32_t* d_nblockflag;       // [1]
    // K split as well: kblock > 0, every array above is [K-blocks][nblocks][M], kprefix as in GemmArgs
    int32_t kblock = 0;
    double* kprefix = nullptr;
};
struct ColArgs {
    const void* d_expected_col;  // [N] acc
    const void* d_Tcol;          // [N] acc
    void* d_colsum;              // [N] acc
    void* d_Ecol;                // [N] acc
    int32_t* d_colflags;         // [N]
    int32_t* d_ncolflag;         // [1]
};
int gemm_dispatch(const vabft_problem* p, const void* dA, const void* dB, void* dC, void* d_expected, void* d_T,
                  int verify, const FusedArgs* fused, const vabft_inject* inj, void* d_rowsum, void* d_rowsum2,
                  void* d_E, int32_t* d_flags, int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj,
                  void* ws, hipStream_t st, const ColArgs* cols = nullptr, const BlockArgs* blocks = nullptr);
void workspace_init_launch(void* ws, size_t bytes, hipStream_t st);

// per-dtype launchers (one translation unit each, to compile in parallel)
// mode: 0 plain, 1 check, 2 check + injector + weighted row sums + column sums, 3 check + weighted row
// sums, 4 check + column sums, 5 row-sum partials only (block-wise check, whole-tile kernels).
// With edge == false the kernels do the compare-and-flag step themselves (and, with
// GemmArgs::fused_stats, the A-side statistics and thresholds); otherwise the caller launches the
// finalize kernel.
int gemm16_launch_bf16_nn(const GemmArgs& a, int mode, bool edge, hipStream_t st);
int gemm16_launch_bf16_nt(const GemmArgs& a, int mode, bool edge, hipStream_t st);
int gemm16_launch_f16_nn(const GemmArgs& a, int mode, bool edge, hipStream_t st);
int gemm16_launch_f16_nt(const GemmArgs& a, int mode, bool edge, hipStream_t st);
int gemm8_launch_f8_nt(const GemmArgs& a, int mode, hipStream_t st);   // E4M3, whole tiles only
int gemm8_launch_bf8_nt(const GemmArgs& a, int mode, hipStream_t st);  // E5M2, whole tiles only
// FP8 problems of any shape and either layout of B (guarded kernel, operands widened to FP16 on load)
int gemm16_launch_f8_edge(const GemmArgs& a, int mode, int e5m2, int transB, hipStream_t st);
// wave_tile: 64 (128 x 128 tiles per workgroup) or 32 (64 x 64 tiles); a.tiles_m / a.tiles_n must count tiles of that size
int gemmw_launch_f32(const GemmArgs& a, int transB, int mode, bool edge, int wave_tile, hipStream_t st);
int gemmw_launch_f64(const GemmArgs& a, int transB, int mode, bool edge, int wave_tile, hipStream_t st);

}  // namespace vabft
