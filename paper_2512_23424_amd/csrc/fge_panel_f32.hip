// Instantiations of the persistent narrow-K kernel (fp32 operands, split-bf16 MFMA).
#include "fge_launch.h"
#include "fge_panel_kernel.h"
namespace fge {
hipError_t launch_panel_f32(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    if (out_dtype == FGE_BF16)
        hipLaunchKernelGGL((panel_kernel<bf16_t>), grid, dim3(PanelShape::THREADS), 0, s, a);
    else
        hipLaunchKernelGGL((panel_kernel<float>), grid, dim3(PanelShape::THREADS), 0, s, a);
    return hipGetLastError();
}
}  // namespace fge
