// FP16 instantiation of the 16-bit verified GEMM: whole-tile problems take the
// direct-to-LDS pipelined kernel, everything else the guarded kernel.
#include "gemm16_fast.h"
namespace vabft {
int gemm16_launch_f16(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st) {
    if (!edge) return gemm16_fast_launch<f16_t>(a, transB, mode, st);
    return gemm16_edge_launch<f16_t>(a, transB, mode, st);
}
}  // namespace vabft
