// Kernel instantiations: bf16 operands, 256x128 workgroup tile, 2x2 waves.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(__bf16, 256, 128, 2, 2)
}
