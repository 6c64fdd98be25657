// Kernel instantiations: f32 operands, 128x256 workgroup tile, 2x2 waves.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(float, 128, 256, 2, 2)
}
