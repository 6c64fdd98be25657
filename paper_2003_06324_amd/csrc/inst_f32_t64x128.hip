// Kernel instantiations: f32 operands, 64x128 workgroup tile, 2x2 waves.
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(float, 64, 128, 2, 2)
}
