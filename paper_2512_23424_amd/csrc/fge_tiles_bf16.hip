// Tile-kernel instantiations for bf16 operands (v_mfma_f32_32x32x16_bf16).
#include "fge_launch.h"
namespace fge {
hipError_t launch_tile_bf16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_tile_any<bf16_t, false>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
