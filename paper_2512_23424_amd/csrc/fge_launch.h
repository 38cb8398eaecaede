// Host-side table of tile configurations and the launchers each translation unit provides.
#pragma once
#include "fge_tile_kernel.h"

namespace fge {

enum TileId { TILE_64x64 = 0, TILE_64x512 = 1, TILE_128x128 = 2, TILE_256x256 = 3, TILE_PANEL = 4, TILE_64x128 = 5, TILE_COUNT = 6 };

// coop_per_cu: workgroups of this tile's cooperative kernel that are resident on one CU at the
// same time (from the compiler's register / LDS report; a lower bound is safe), 0 if the tile
// has no cooperative kernel.
struct TileInfo { int bm, bn, threads, waves_n, coop_per_cu; const char *name; };

inline const TileInfo &tile_info(int id) {
    static const TileInfo t[TILE_COUNT] = {
        {64, 64, 256, 2, 0, "64x64_w2x2"},
        {64, 512, 256, 4, 0, "64x512_w1x4"},
        {128, 128, 256, 2, 1, "128x128_w2x2"},
        {256, 256, 512, 4, 1, "256x256_w2x4"},
        {64, 512, 512, 8, 0, "panel64x512_w1x8_splitbf16"},   // persistent narrow-K kernel, fp32 operands
        {64, 128, 256, 2, 2, "64x128_w2x2"},
    };
    return t[id];
}

// Defined in fge_tiles_f32.hip / fge_tiles_bf16.hip (split so they compile in parallel).
hipError_t launch_tile_f32(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_tile_bf16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
// Defined in fge_panel_f32.hip: the persistent narrow-K kernel (grid = number of workgroups).
hipError_t launch_panel_f32(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);

// Workgroups of `kernel` the current device holds at the same time (0 if the query fails).
inline int resident_workgroups(const void *kernel, int threads) {
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess) return 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return per_cu * cus;
}

template <typename InT>
inline hipError_t launch_tile_any(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
#define FGE_LAUNCH(BM, BN, WM, WN, COOP, FULL)                                                  \
    do {                                                                                        \
        if (out_dtype == FGE_BF16)                                                              \
            hipLaunchKernelGGL((tile_kernel<InT, bf16_t, BM, BN, WM, WN, COOP, FULL>), grid,    \
                               dim3(64 * WM * WN), 0, s, a);                                    \
        else                                                                                    \
            hipLaunchKernelGGL((tile_kernel<InT, float, BM, BN, WM, WN, COOP, FULL>), grid,     \
                               dim3(64 * WM * WN), 0, s, a);                                    \
    } while (0)
    // cooperative kernel of a tile.  All workgroups of the grid must be resident at once; a launch that the device cannot hold
    // that way is refused instead of being left to run into its wait limit.
#define FGE_LAUNCH_COOP1(BM, BN, WM, WN, OT, FULL)                                              \
    do {                                                                                        \
        auto kern = tile_kernel<InT, OT, BM, BN, WM, WN, true, FULL>;                           \
        static const int resident = resident_workgroups(reinterpret_cast<const void *>(kern), 64 * WM * WN); \
        if ((int)grid.x > resident) return hipErrorCooperativeLaunchTooLarge;                   \
        hipLaunchKernelGGL(kern, grid, dim3(64 * WM * WN), 0, s, a);                            \
    } while (0)
#define FGE_LAUNCH_COOP(BM, BN, WM, WN)                                                         \
    do {                                                                                        \
        if (out_dtype == FGE_BF16) FGE_LAUNCH_COOP1(BM, BN, WM, WN, bf16_t, false);             \
        else                       FGE_LAUNCH_COOP1(BM, BN, WM, WN, float, false);              \
    } while (0)
    // the cooperative form exists for the tiles large problems use: bf16 256x256 and 128x128,
    // fp32 64x128 (tile_has_coop below must agree)
    constexpr bool BF = sizeof(InT) == 2;
    switch (tile) {
    case TILE_64x64:   FGE_LAUNCH(64, 64, 2, 2, false, false); break;
    case TILE_64x512:  FGE_LAUNCH(64, 512, 1, 4, false, false); break;
    case TILE_128x128:
        if constexpr (BF) { if (a.coop) { FGE_LAUNCH_COOP(128, 128, 2, 2); break; } }
        FGE_LAUNCH(128, 128, 2, 2, false, false); break;
    case TILE_256x256:
        if constexpr (BF) { if (a.coop) { FGE_LAUNCH_COOP(256, 256, 2, 4); break; } }
        FGE_LAUNCH(256, 256, 2, 4, false, false); break;
    case TILE_64x128:
        if constexpr (!BF) { if (a.coop) { FGE_LAUNCH_COOP(64, 128, 2, 2); break; } }
        FGE_LAUNCH(64, 128, 2, 2, false, false); break;
    default: return hipErrorInvalidValue;
    }
#undef FGE_LAUNCH_COOP
#undef FGE_LAUNCH_COOP1
#undef FGE_LAUNCH
    return hipGetLastError();
}

// Whether launch_tile_any has a cooperative kernel for this tile and operand type.
inline bool tile_has_coop(int tile, int in_dtype) {
    return in_dtype == FGE_BF16 ? (tile == TILE_128x128 || tile == TILE_256x256) : tile == TILE_64x128;
}

}  // namespace fge
