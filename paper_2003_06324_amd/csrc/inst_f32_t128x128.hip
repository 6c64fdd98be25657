// Kernel instantiations: f32 operands, 128x128 workgroup tile, 2x2 waves.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(float, 128, 128, 2, 2)
}
