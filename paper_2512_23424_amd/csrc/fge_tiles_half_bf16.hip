// Half-tile configurations (128x256, 256x128) for bf16 operands.
#include "fge_launch.h"
namespace fge {
hipError_t launch_half_bf16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_half_any<bf16_t>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
