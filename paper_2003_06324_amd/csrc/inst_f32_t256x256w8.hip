// Kernel instantiations: f32 operands, 256x256 workgroup tile, 2x4 waves (two waves per SIMD).
#include "gemm_launch.h"
namespace gemm_gfx950 {
GEMM_INSTANTIATE_TILE(float, 256, 256, 2, 4)
}
