// Host-side table of tile configurations and the launchers each translation unit provides.
#pragma once
#include "fge_tile_kernel.h"

namespace fge {

enum TileId { TILE_64x64 = 0, TILE_64x512 = 1, TILE_128x128 = 2, TILE_256x256 = 3, TILE_PANEL = 4, TILE_64x128 = 5, TILE_COUNT = 6 };

struct TileInfo { int bm, bn, threads, waves_n; const char *name; };

inline const TileInfo &tile_info(int id) {
    static const TileInfo t[TILE_COUNT] = {
        {64, 64, 256, 2, "64x64_w2x2"},
        {64, 512, 256, 4, "64x512_w1x4"},
        {128, 128, 256, 2, "128x128_w2x2"},
        {256, 256, 512, 4, "256x256_w2x4"},
        {64, 512, 512, 8, "panel64x512_w1x8_splitbf16"},   // persistent narrow-K kernel, fp32 operands
        {64, 128, 256, 2, "64x128_w2x2"},
    };
    return t[id];
}

// Defined in fge_tiles_f32.hip / fge_tiles_bf16.hip (split so they compile in parallel).
hipError_t launch_tile_f32(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_tile_bf16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
// Defined in fge_panel_f32.hip: the persistent narrow-K kernel (grid = number of workgroups).
hipError_t launch_panel_f32(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);

template <typename InT>
inline hipError_t launch_tile_any(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
#define FGE_LAUNCH(BM, BN, WM, WN)                                                              \
    do {                                                                                        \
        if (out_dtype == FGE_BF16)                                                              \
            hipLaunchKernelGGL((tile_kernel<InT, bf16_t, BM, BN, WM, WN>), grid,                \
                               dim3(64 * WM * WN), 0, s, a);                                    \
        else                                                                                    \
            hipLaunchKernelGGL((tile_kernel<InT, float, BM, BN, WM, WN>), grid,                 \
                               dim3(64 * WM * WN), 0, s, a);                                    \
    } while (0)
    switch (tile) {
    case TILE_64x64:   FGE_LAUNCH(64, 64, 2, 2); break;
    case TILE_64x512:  FGE_LAUNCH(64, 512, 1, 4); break;
    case TILE_128x128: FGE_LAUNCH(128, 128, 2, 2); break;
    case TILE_256x256: FGE_LAUNCH(256, 256, 2, 4); break;
    case TILE_64x128:  FGE_LAUNCH(64, 128, 2, 2); break;
    default: return hipErrorInvalidValue;
    }
#undef FGE_LAUNCH
    return hipGetLastError();
}

}  // namespace fge
