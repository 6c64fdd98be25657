// Kernel instantiations: K split across the four waves of a workgroup, 64x64 tile.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_KSPLIT(_Float16, 64, 64)
GEMM_INSTANTIATE_KSPLIT(__bf16, 64, 64)
GEMM_INSTANTIATE_KSPLIT(float, 64, 64)
}
