// FP16 instantiation of the 16-bit verified GEMM.
#include "gemm16.h"
namespace vabft {
int gemm16_launch_f16(const GemmArgs& a, int transB, int mode, bool edge, hipStream_t st) {
    return gemm16_launch<f16_t>(a, transB, mode, edge, st);
}
}  // namespace vabft
