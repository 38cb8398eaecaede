// Tile-kernel instantiations for fp16 operands (v_mfma_f32_32x32x16_f16).
#include "fge_launch.h"
namespace fge {
hipError_t launch_tile_f16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_tile_any<f16_t, false>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
