// Kernel instantiations: bf16 operands, 128x256 workgroup tile, 2x2 waves.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(__bf16, 128, 256, 2, 2)
}
