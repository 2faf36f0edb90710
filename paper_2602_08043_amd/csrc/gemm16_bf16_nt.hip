// BF16 verified GEMM, B stored N x K: whole-tile problems take the direct-to-LDS
// pipelined kernel, everything else the guarded kernel.
#include "gemm16_fast.h"
namespace vabft {
int gemm16_launch_bf16_nt(const GemmArgs& a, int mode, bool edge, hipStream_t st) {
    if (!edge) return gemm16_fast_launch_tb<bf16_t, 1>(a, mode, st);
    return gemm16_edge_launch_tb<bf16_t, 1>(a, mode, st);
}
}  // namespace vabft
