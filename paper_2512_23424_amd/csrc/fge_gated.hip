// Gated tile-kernel instantiations (bf16, fp16 and 8-bit operands).
#include "fge_launch.h"
namespace fge {
hipError_t launch_gated_bf16(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_gated_any<bf16_t>(out_dtype, grid, s, a);
}
hipError_t launch_gated_f16(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_gated_any<f16_t>(out_dtype, grid, s, a);
}
hipError_t launch_gated_f8(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    return launch_gated_any<f8_t>(out_dtype, grid, s, a);
}
}  // namespace fge
