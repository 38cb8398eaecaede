// Instantiations of the persistent narrow-K kernel (fp32 operands, split-bf16 MFMA).
#include "fge_launch.h"
#include "fge_panel_kernel.h"
namespace fge {
namespace {
constexpr size_t LLC_BYTES = (size_t)256 << 20;     // memory-side cache in front of HBM

template <typename OutT>
void launch(dim3 grid, hipStream_t s, const TileArgs &a) {
    const bool full = a.M % PanelShape::BM == 0 && a.N == PanelShape::BN;
    const bool stream = (size_t)a.M * a.N * sizeof(OutT) >= LLC_BYTES;
    const dim3 block(PanelShape::THREADS);
    // the chain this kernel exists for - clamp to a narrow range, then the row logsumexp - with
    // activation and row op fixed at compile time (fp32 results, tiles inside the matrix)
    if constexpr (sizeof(OutT) == 4) {
        if (full && a.act == FGE_ACT_CLAMP && a.norm == FGE_NORM_LOGSUMEXP && a.hi - a.lo <= 64.0f) {
            if (stream) hipLaunchKernelGGL((panel_kernel<OutT, true, true, FGE_ACT_CLAMP, FGE_NORM_LOGSUMEXP, true>), grid, block, 0, s, a);
            else        hipLaunchKernelGGL((panel_kernel<OutT, true, false, FGE_ACT_CLAMP, FGE_NORM_LOGSUMEXP, true>), grid, block, 0, s, a);
            return;
        }
    }
    if (full) {
        if (stream) hipLaunchKernelGGL((panel_kernel<OutT, true, true>), grid, block, 0, s, a);
        else        hipLaunchKernelGGL((panel_kernel<OutT, true, false>), grid, block, 0, s, a);
    } else {
        if (stream) hipLaunchKernelGGL((panel_kernel<OutT, false, true>), grid, block, 0, s, a);
        else        hipLaunchKernelGGL((panel_kernel<OutT, false, false>), grid, block, 0, s, a);
    }
}
}  // namespace

hipError_t launch_panel_f32(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    if (out_dtype == FGE_BF16) launch<bf16_t>(grid, s, a);
    else                       launch<float>(grid, s, a);
    return hipGetLastError();
}
}  // namespace fge
