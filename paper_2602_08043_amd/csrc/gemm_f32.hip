// FP32 instantiation of the wide verified GEMM.
#include "gemm_wide.h"
namespace vabft {
int gemmw_launch_f32(const GemmArgs& a, int transB, int mode, bool edge, int wave_tile, hipStream_t st) {
    return gemmw_launch<float>(a, transB, mode, edge, wave_tile, st);
}
}  // namespace vabft
