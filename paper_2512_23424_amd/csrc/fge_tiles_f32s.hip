// Tile-kernel instantiations for fp32 operands with the split-bf16 product (three
// v_mfma_f32_32x32x16_bf16 per 16 k instead of eight v_mfma_f32_32x32x2_f32).
#include "fge_launch.h"
namespace fge {
hipError_t launch_tile_f32s(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_tile_any<float, true>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
