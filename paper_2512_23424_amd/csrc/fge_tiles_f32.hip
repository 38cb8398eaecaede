// Tile-kernel instantiations for fp32 operands on the fp32 matrix instruction
// (v_mfma_f32_32x32x2_f32).
#include "fge_launch.h"
namespace fge {
hipError_t launch_tile_f32(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_tile_any<float, false>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
