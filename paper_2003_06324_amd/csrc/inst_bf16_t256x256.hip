// Kernel instantiations: bfloat16 operands, 256x256 workgroup tile, 2x2 waves.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(__bf16, 256, 256, 2, 2)
}
