// Tile-kernel instantiations for 8-bit E4M3 operands (v_mfma_f32_32x32x64_f8f6f4).
#include "fge_launch.h"
namespace fge {
hipError_t launch_tile_f8(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_tile_any<f8_t, false>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
