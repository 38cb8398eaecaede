// Instantiations of the persistent narrow-K kernel (fp32 operands, split-bf16 MFMA).
#include "fge_launch.h"
#include "fge_panel_kernel.h"
namespace fge {
hipError_t launch_panel_f32(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    const bool full = a.M % PanelShape::BM == 0 && a.N == PanelShape::BN;
    const dim3 block(PanelShape::THREADS);
    if (out_dtype == FGE_BF16) {
        if (full) hipLaunchKernelGGL((panel_kernel<bf16_t, true>), grid, block, 0, s, a);
        else      hipLaunchKernelGGL((panel_kernel<bf16_t, false>), grid, block, 0, s, a);
    } else {
        if (full) hipLaunchKernelGGL((panel_kernel<float, true>), grid, block, 0, s, a);
        else      hipLaunchKernelGGL((panel_kernel<float, false>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}
}  // namespace fge
