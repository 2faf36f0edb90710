// Host-side declarations shared by the translation units of libvabft.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vabft.h"

namespace vabft {

// encode.hip
size_t encode_workspace_bytes(const vabft_problem* p);
int encode_dispatch(const vabft_problem* p, const void* dB, void* d_Be, void* d_bstat, double* d_S, void* ws,
                    hipStream_t st);
int threshold_dispatch(const vabft_problem* p, const void* dA, const void* d_Be, const double* d_S, double e_max,
                       double c_sigma, void* d_astat, void* d_expected, void* d_T, hipStream_t st);

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
    void* rowpart;    // [tiles_n][M] acc
    int32_t* d_nflag; // zeroed by the GEMM kernel, accumulated by the finalize kernel
    InjectArgs inj;
};

size_t gemm_workspace_bytes(const vabft_problem* p);
int gemm_dispatch(const vabft_problem* p, const void* dA, const void* dB, void* dC, const void* d_expected,
                  const void* d_T, int verify, const vabft_inject* inj, void* d_rowsum, void* d_E, int32_t* d_flags,
                  int32_t* d_nflag, vabft_inject_rec* d_injlog, int32_t* d_ninj, void* ws, hipStream_t st);

// per-dtype launchers (one translation unit each, to compile in parallel)
int gemm16_launch_bf16(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st);
int gemm16_launch_f16(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st);
int gemmw_launch_f32(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st);
int gemmw_launch_f64(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st);

}  // namespace vabft
