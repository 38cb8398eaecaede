// Host-side table of tile configurations and the launchers each translation unit provides.
#pragma once
#include "fge_tile_kernel.h"

namespace fge {

enum TileId { TILE_64x64 = 0, TILE_64x512 = 1, TILE_128x128 = 2, TILE_256x256 = 3, TILE_PANEL = 4, TILE_64x128 = 5,
              TILE_GATED = 6, TILE_128x256 = 7, TILE_256x128 = 8, TILE_128x128_W8 = 9, TILE_128x128_S3 = 10, TILE_COUNT = 11 };

// coop_per_cu: workgroups of this tile's cooperative kernel that are resident on one CU at the
// same time (from the compiler's register / LDS report; a lower bound is safe), 0 if the tile
// has no cooperative kernel.
struct TileInfo { int bm, bn, threads, waves_n, coop_per_cu; const char *name, *name_split; };

inline const TileInfo &tile_info(int id) {
    static const TileInfo t[TILE_COUNT] = {
        {64, 64, 256, 2, 0, "64x64_w2x2", "64x64_w2x2_splitbf16"},
        {64, 512, 256, 4, 0, "64x512_w1x4", "64x512_w1x4_splitbf16"},
        {128, 128, 256, 2, 2, "128x128_w2x2", "128x128_w2x2_splitbf16"},
        {256, 256, 512, 4, 1, "256x256_w2x4", nullptr},
        // persistent narrow-K kernel, fp32 operands, always the split product
        {64, 512, 512, 8, 0, "panel64x512_w1x8_splitbf16", "panel64x512_w1x8_splitbf16"},
        {64, 128, 256, 2, 2, "64x128_w2x2", "64x128_w2x2_splitbf16"},
        // gated form, 16-bit operands: 256 rows x 128 output columns (two 256x128 products)
        {256, 128, 512, 4, 1, "gated256x128_w2x4", nullptr},
        // 16-bit and 8-bit operands: half a 256x256 tile either way, eight waves of 64x64 - twice the
        // workgroups of the 256x256 tiling for problems that leave it short of them
        {128, 256, 512, 4, 1, "128x256_w2x4", nullptr},
        {256, 128, 512, 2, 1, "256x128_w4x2", nullptr},
        // fp32 operands, split product: the 128x128 tile on eight waves of 64x32 (one workgroup per
        // CU) - for problems that give a CU one tile only, where the four-wave form leaves each
        // SIMD a single wave and nothing to run under its stalls
        {128, 128, 512, 4, 1, nullptr, "128x128_w2x4_splitbf16"},
        // 16- and 8-bit operands, at most one 128x128 tile per CU: eight waves of 64x32 and three
        // stage buffers (no second workgroup shares the CU, so a second K-tile copy in flight and a
        // second wave per SIMD hide the latencies instead); the plan puts it in the place of
        // 128x128_w2x2 wherever that tile is chosen for such a problem
        {128, 128, 512, 4, 1, "128x128_w2x4_s3", nullptr},
    };
    return t[id];
}

// Defined in fge_tiles_f32.hip / fge_tiles_f32s.hip / fge_tiles_bf16.hip (separate units so they
// compile in parallel).  f32: fp32 matrix instruction; f32s: split-bf16 product.
hipError_t launch_tile_f32(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_tile_f32s(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_tile_bf16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_tile_f16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_tile_f8(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
// Defined in fge_panel_f32.hip: the persistent narrow-K kernel (grid = number of workgroups).
hipError_t launch_panel_f32(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);

// Element-granular kernels (fge_generic.hip) for shapes the vectorised kernels do not take.
// gemm: dst = act(post*(alpha*X.W^T + b)); act: dst = act(X) [* W if W is set] with X (and W) laid
// out like dst; row:
// dst = rowop(X) with X rows x N at strides (ldx, bsx).  M rows per problem, `batch` problems.
struct GenArgs {
    const void *X, *W;
    const float *b, *gamma, *beta;
    const float *b2;            // slice sum with a gate: bias of the second product
    void *dst;
    float *aux;
    int M, N, K, batch;
    int64_t ldx, ldw, ldd, bsx, bsd;
    float alpha, post, lo, hi, eps;
    int act, norm;
};
hipError_t launch_generic_gemm(int in_dtype, int dst_dtype, hipStream_t s, const GenArgs &a);
hipError_t launch_generic_act(int dtype, hipStream_t s, const GenArgs &a);
hipError_t launch_generic_row(int src_dtype, int out_dtype, hipStream_t s, const GenArgs &a);
// X: a.K dense fp32 slices of M x N, a.bsx elements apart; dst = act(post*(alpha*sum + b)),
// times post*(alpha*sum2 + b2) when W points to the slices of a second product (gated form)
hipError_t launch_splitk_sum(int dst_dtype, hipStream_t s, const GenArgs &a);

// Dense, zero-padded copy of an operand (fge_generic.hip): dst is rows_dst x Kp of the same
// element type, Kp a multiple of the 16-byte chunk; source: batch problems of M rows x K.
struct PadArgs {
    const void *src;
    void *dst;
    int M, batch, K, Kp;
    int64_t ld, bs;             // source row stride / stride between problems, in elements
    int64_t rows_dst;           // >= batch * M; the rows beyond are zero
};
hipError_t launch_pad_rows(int dtype, hipStream_t s, const PadArgs &a);
hipError_t launch_pad_vec(const float *src, float *dst, int n, int np, hipStream_t s);

// Workgroups of `kernel` the current device holds at the same time (0 if the query fails).
inline int resident_workgroups(const void *kernel, int threads) {
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess) return 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return per_cu * cus;
}

// Which tiles exist for which operand type (tile selection on the host must agree):
//   bf16, fp16, fp8: 64x64, 64x512, 128x128 (+ cooperative; four waves, and eight with three
//         stage buffers for one tile per CU), 256x256 and its halves 128x256, 256x128 (+ cooperative)
//   fp32: 64x64, 64x512, 64x128 (+ cooperative) - once with the fp32 matrix instruction and once
//         with the split-bf16 product (SPLIT); 128x128 (+ cooperative; four waves, and eight for one
//         tile per CU) with the split product only
// The 16-bit output type that goes with an operand type (the other output type is fp32).
template <typename InT> struct NarrowOut { typedef bf16_t type; };
template <> struct NarrowOut<f16_t> { typedef f16_t type; };

template <typename InT, bool SPLIT>
inline hipError_t launch_tile_any(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    typedef typename NarrowOut<InT>::type NarrowT;
#define FGE_LAUNCH(BM, BN, WM, WN)                                                              \
    do {                                                                                        \
        if (out_dtype != FGE_F32)                                                               \
            hipLaunchKernelGGL((tile_kernel<InT, NarrowT, BM, BN, WM, WN, false, false, SPLIT>), grid, \
                               dim3(64 * WM * WN), 0, s, a);                                    \
        else                                                                                    \
            hipLaunchKernelGGL((tile_kernel<InT, float, BM, BN, WM, WN, false, false, SPLIT>), grid, \
                               dim3(64 * WM * WN), 0, s, a);                                    \
    } while (0)
    // cooperative kernel of a tile.  All workgroups of the grid must be resident at once; a
    // launch that the device cannot hold that way is refused instead of being left to run into
    // its wait limit.
#define FGE_LAUNCH_COOP2(BM, BN, WM, WN, OT, FULL)                                              \
    do {                                                                                        \
        auto kern = tile_kernel<InT, OT, BM, BN, WM, WN, true, FULL, SPLIT>;                    \
        static const int resident = resident_workgroups(reinterpret_cast<const void *>(kern), 64 * WM * WN); \
        if ((int)grid.x > resident) return hipErrorCooperativeLaunchTooLarge;                   \
        hipLaunchKernelGGL(kern, grid, dim3(64 * WM * WN), 0, s, a);                            \
    } while (0)
    /* guard-free epilogue where every tile lies inside the matrix (256x256 tiles only) */      \
#define FGE_LAUNCH_COOP1(BM, BN, WM, WN, OT)                                                    \
    do {                                                                                        \
        if (BM == 256 && a.M % BM == 0 && a.N % BN == 0) FGE_LAUNCH_COOP2(BM, BN, WM, WN, OT, (BM == 256)); \
        else                                             FGE_LAUNCH_COOP2(BM, BN, WM, WN, OT, false); \
    } while (0)
#define FGE_LAUNCH_COOP(BM, BN, WM, WN)                                                         \
    do {                                                                                        \
        if (out_dtype != FGE_F32)  FGE_LAUNCH_COOP1(BM, BN, WM, WN, NarrowT);                   \
        else                       FGE_LAUNCH_COOP1(BM, BN, WM, WN, float);                     \
    } while (0)
    // 128x128 tiles on eight waves with three stage buffers (one workgroup per CU), ordinary and cooperative launch
#define FGE_LAUNCH_DEEP128(OT)                                                                  \
    do {                                                                                        \
        if (a.coop) {                                                                           \
            auto kern = tile_kernel<InT, OT, 128, 128, 2, 4, true, false, false, false, 3>;     \
            static const int resident = resident_workgroups(reinterpret_cast<const void *>(kern), 512); \
            if ((int)grid.x > resident) return hipErrorCooperativeLaunchTooLarge;               \
            hipLaunchKernelGGL(kern, grid, dim3(512), 0, s, a);                                 \
        } else {                                                                                \
            hipLaunchKernelGGL((tile_kernel<InT, OT, 128, 128, 2, 4, false, false, false, false, 3>), grid, \
                               dim3(512), 0, s, a);                                             \
        }                                                                                       \
    } while (0)
    constexpr bool BF = sizeof(InT) <= 2;
    switch (tile) {
    case TILE_64x64:   FGE_LAUNCH(64, 64, 2, 2); break;
    case TILE_64x512:  FGE_LAUNCH(64, 512, 1, 4); break;
    case TILE_128x128:
        if constexpr (BF || SPLIT) {
            if (a.coop) FGE_LAUNCH_COOP(128, 128, 2, 2);
            else        FGE_LAUNCH(128, 128, 2, 2);
            break;
        }
        return hipErrorInvalidValue;
    case TILE_128x128_S3:
        if constexpr (BF && !SPLIT) {
            if (out_dtype != FGE_F32) FGE_LAUNCH_DEEP128(NarrowT);
            else                      FGE_LAUNCH_DEEP128(float);
            break;
        }
        return hipErrorInvalidValue;
    case TILE_256x256:
        if constexpr (BF) {
            if (a.coop) FGE_LAUNCH_COOP(256, 256, 2, 4);
            else        FGE_LAUNCH(256, 256, 2, 4);
            break;
        }
        return hipErrorInvalidValue;
    case TILE_128x128_W8:
        if constexpr (SPLIT) {
            if (a.coop) FGE_LAUNCH_COOP(128, 128, 2, 4);
            else        FGE_LAUNCH(128, 128, 2, 4);
            break;
        }
        return hipErrorInvalidValue;
    case TILE_64x128:
        if constexpr (!BF) {
            if (a.coop) FGE_LAUNCH_COOP(64, 128, 2, 2);
            else        FGE_LAUNCH(64, 128, 2, 2);
            break;
        }
        return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
    }
#undef FGE_LAUNCH
#undef FGE_LAUNCH_DEEP128
#undef FGE_LAUNCH_COOP
#undef FGE_LAUNCH_COOP1
#undef FGE_LAUNCH_COOP2
    return hipGetLastError();
}

// The gated tile kernel (16-bit and 8-bit operands): ordinary or cooperative launch.
template <typename InT>
inline hipError_t launch_gated_any(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    typedef typename NarrowOut<InT>::type NarrowT;
#define FGE_GATED(OT, COOP)                                                                     \
    do {                                                                                        \
        auto kern = tile_kernel<InT, OT, 256, 256, 2, 4, COOP, false, false, true>;             \
        if (COOP) {                                                                             \
            static const int resident = resident_workgroups(reinterpret_cast<const void *>(kern), 512); \
            if ((int)grid.x > resident) return hipErrorCooperativeLaunchTooLarge;               \
        }                                                                                       \
        hipLaunchKernelGGL(kern, grid, dim3(512), 0, s, a);                                     \
    } while (0)
    if (out_dtype != FGE_F32) { if (a.coop) FGE_GATED(NarrowT, true); else FGE_GATED(NarrowT, false); }
    else                      { if (a.coop) FGE_GATED(float, true);   else FGE_GATED(float, false); }
#undef FGE_GATED
    return hipGetLastError();
}
// The half-tile configurations (TILE_128x256, TILE_256x128), ordinary or cooperative launch;
// defined in fge_tiles_half.hip.
template <typename InT>
inline hipError_t launch_half_any(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a) {
    typedef typename NarrowOut<InT>::type NarrowT;
#define FGE_HALF(BM, BN, WM, WN, OT)                                                            \
    do {                                                                                        \
        if (a.coop) {                                                                           \
            auto kern = tile_kernel<InT, OT, BM, BN, WM, WN, true, false>;                      \
            static const int resident = resident_workgroups(reinterpret_cast<const void *>(kern), 512); \
            if ((int)grid.x > resident) return hipErrorCooperativeLaunchTooLarge;               \
            hipLaunchKernelGGL(kern, grid, dim3(512), 0, s, a);                                 \
        } else {                                                                                \
            hipLaunchKernelGGL((tile_kernel<InT, OT, BM, BN, WM, WN, false, false>), grid, dim3(512), 0, s, a); \
        }                                                                                       \
    } while (0)
    if (tile == TILE_128x256) {
        if (out_dtype != FGE_F32) FGE_HALF(128, 256, 2, 4, NarrowT); else FGE_HALF(128, 256, 2, 4, float);
    } else if (tile == TILE_256x128) {
        if (out_dtype != FGE_F32) FGE_HALF(256, 128, 4, 2, NarrowT); else FGE_HALF(256, 128, 4, 2, float);
    } else {
        return hipErrorInvalidValue;
    }
#undef FGE_HALF
    return hipGetLastError();
}
hipError_t launch_half_bf16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_half_f16(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_half_f8(int tile, int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_gated_bf16(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_gated_f16(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);
hipError_t launch_gated_f8(int out_dtype, dim3 grid, hipStream_t s, const TileArgs &a);

// Whether launch_tile_any has a cooperative kernel for this tile and operand type.
inline bool tile_has_coop(int tile, int in_dtype) {
    if (tile == TILE_GATED) return true;
    if (tile == TILE_128x256 || tile == TILE_256x128) return in_dtype != FGE_F32;
    return in_dtype != FGE_F32 ? (tile == TILE_128x128 || tile == TILE_128x128_S3 || tile == TILE_256x256)
                               : (tile == TILE_64x128 || tile == TILE_128x128 || tile == TILE_128x128_W8);
}

}  // namespace fge
