// FP8 (E4M3) x FP8 -> FP16 verified GEMM, B stored N x K.
#include "gemm8_fast.h"

namespace vabft {
int gemm8_launch_f8_nt(const GemmArgs& a, int mode, hipStream_t st) { return gemm8_fast_launch<0>(a, mode, st); }
}  // namespace vabft
