// FP8 (E4M3 / E5M2) verified GEMM for shapes and layouts the whole-tile FP8 kernel does not take: the guarded
// FP16 kernel with the operands widened on load (FP32 accumulation, FP16 output).
#include "gemm16.h"
namespace vabft {
int gemm16_launch_f8_edge(const GemmArgs& a, int mode, int e5m2, int transB, hipStream_t st) {
    if (e5m2) return transB ? gemm16_edge_launch_tb<f16_t, 1, 2>(a, mode, st) : gemm16_edge_launch_tb<f16_t, 0, 2>(a, mode, st);
    return transB ? gemm16_edge_launch_tb<f16_t, 1, 1>(a, mode, st) : gemm16_edge_launch_tb<f16_t, 0, 1>(a, mode, st);
}
}  // namespace vabft
