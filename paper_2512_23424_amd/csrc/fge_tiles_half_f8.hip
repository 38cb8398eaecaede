// Half-tile configurations (128x256, 256x128) for f8 operands.
#include "fge_launch.h"
namespace fge {
hipError_t launch_half_f8(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_half_any<f8_t>(tile, out_dtype, grid, s, a);
}
}  // namespace fge
