// Narrow-K whole-row kernel for fp32 operands: K <= 64, N <= 512, many rows.
//
// Such a problem is bound by the output stream (every row reads K*4 bytes and writes N*4), so
// the kernel is organised around HBM, not around the matrix cores:
//   * persistent workgroups (one per CU, 8 waves side by side along N) walk over 64-row tiles;
//     W never leaves the registers: each wave keeps the MFMA B fragments of its 64 columns,
//     already split, for the whole launch;
//   * the X tile of the next step is copied global -> LDS asynchronously while the current one
//     is multiplied and its epilogue runs; the stores of a tile are queued only after that copy
//     has landed, so nothing ever waits on a store;
//   * the product uses the bf16 matrix instruction on a two-term split of the fp32 operands,
//         x = xh + xl,  w = wh + wl  (xh, wh: bf16 roundings; xl, wl: bf16 roundings of the rest)
//         x*w ~= xh*wh + xh*wl + xl*wh          (fp32 accumulate)
//     which leaves a relative error of about 2^-17 per product - 16x the rate of the fp32
//     matrix instruction, at an accuracy the 1e-4 tolerance of the fp32 path covers by an order
//     of magnitude.  With the fp32 instruction the MFMA time alone would exceed the time HBM
//     needs for the output.
// Scale, bias, activation, row statistics and stores are the shared register epilogue.
#pragma once
#include "fge_epilogue.h"

namespace fge {

// 8 fp32 values -> bf16 high parts and bf16 roundings of the remainders, packed two per word.
__device__ __forceinline__ void split_bf16x8(const float (&f)[8], u32x4 &hi, u32x4 &lo) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t hh = f32x2_to_bf16x2(f[2 * p], f[2 * p + 1]);
        const float r0 = f[2 * p] - as_f32(hh << 16), r1 = f[2 * p + 1] - as_f32(hh & 0xFFFF0000u);
        hi[p] = hh;
        lo[p] = f32x2_to_bf16x2(r0, r1);
    }
}

__device__ __forceinline__ void mfma_bf16(const u32x4 &a, const u32x4 &b, floatx16 &c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

struct PanelShape {
    static constexpr int BM = 64, BN = 512, WAVES_N = 8, MB = 2, NB = 2, KMAX = 64;
    static constexpr int THREADS = 64 * WAVES_N;
};

// FULL: M is a multiple of 64 and N == 512, so the epilogue needs no row or column guards.
// STREAM: the output is larger than the last-level cache and is stored with the streaming hint.
template <typename OutT, bool FULL, bool STREAM>
__global__ __launch_bounds__(PanelShape::THREADS)
void panel_kernel(const TileArgs a) {
    constexpr int BM = PanelShape::BM, BN = PanelShape::BN, WAVES_N = PanelShape::WAVES_N;
    constexpr int MB = PanelShape::MB, NB = PanelShape::NB, NT = PanelShape::THREADS;
    constexpr int WTN = NB * 32;
    constexpr int XROWB = 256;                        // LDS bytes per X row: 64 fp32
    constexpr int XTILE = BM * XROWB;                 // 16 KB
    constexpr int X_LD = BM * 16 / NT;                // 16-byte chunks per thread per tile (2)
    using Epi = TileEpilogue<OutT, MB, NB, WAVES_N, 16, false, true, false, FULL, STREAM>;

    __shared__ __attribute__((aligned(16))) unsigned char xs[2 * XTILE];
    __shared__ __attribute__((aligned(16))) float2 xch[2 * BM * WAVES_N];
    __shared__ __attribute__((aligned(16))) float patches[(NT / 64) * Epi::PATCH_FLOATS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_n = wave;
    const int h = lane >> 5, l32 = lane & 31;
    const float *X = reinterpret_cast<const float *>(a.X);
    const float *W = reinterpret_cast<const float *>(a.W);
    OutT *out = reinterpret_cast<OutT *>(a.out);

    // zero both X buffers once: chunks past K are never written by the copies below
#pragma unroll
    for (int i = 0; i < 2 * XTILE / 16 / NT; ++i)
        *reinterpret_cast<u32x4 *>(xs + (i * NT + tid) * 16) = u32x4{0u, 0u, 0u, 0u};

    // ---------------- W fragments of this wave's 64 columns, split once, kept in registers
    // fragment (j, t): column wave_n*64 + j*32 + l32, k = 16t + 8h .. +7
    u32x4 whi[NB][4], wlo[NB][4];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const float *wr = W + (int64_t)min(wave_n * WTN + j * 32 + l32, a.N - 1) * a.ldw;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int k0 = 16 * t + 8 * h;
            float f[8];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                floatx4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (k0 + 4 * c < a.K) v = *reinterpret_cast<const floatx4 *>(wr + k0 + 4 * c);
                f[4 * c] = v[0]; f[4 * c + 1] = v[1]; f[4 * c + 2] = v[2]; f[4 * c + 3] = v[3];
            }
            split_bf16x8(f, whi[j][t], wlo[j][t]);
        }
    }

    // ---------------- X tile copy plan.  LDS image: row-major, 16 chunks of 16 bytes per row,
    // chunk c stored at c ^ (row & 15) so that the 16 rows read by a quarter wave hit all 64
    // banks.  A wave's copy instruction fills 1024 contiguous bytes (4 rows), lane l at +16*l.
    int x_row[X_LD], x_gc[X_LD];
#pragma unroll
    for (int i = 0; i < X_LD; ++i) {
        x_row[i] = (i * (NT / 64) + wave) * 4 + (lane >> 4);
        x_gc[i] = (lane & 15) ^ (x_row[i] & 15);
    }
    auto dma_x = [&](int buf, int m0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < X_LD; ++i) {
            if (x_gc[i] * 4 < a.K) {
                const float *g = X + (int64_t)min(m0 + x_row[i], a.M - 1) * a.ldx + x_gc[i] * 4;
                unsigned char *s = xs + buf * XTILE + (i * (NT / 64) + wave) * 1024;
                lds_dma16(g, s);
            }
        }
    };

    // A fragment (i, t): row i*32 + l32, k = 16t + 8h .. +7 = chunks 4t + 2h and 4t + 2h + 1
    // (every wave needs all 64 rows; the split of a fragment is recomputed per wave)
    int fa_off[MB][4][2];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                fa_off[i][t][c] = (i * 32 + l32) * XROWB + (((4 * t + 2 * h + c) ^ (l32 & 15)) << 4);

    Epi epi(a, out, xch, patches + wave * Epi::PATCH_FLOATS, BM, 0, 0, 0, 0, wave_n, lane);

    // ---------------- persistent loop over 64-row tiles
    const int ntiles = a.tiles_m;
    int tile = blockIdx.x;
    __syncthreads();                                  // zero fill is complete
    if (tile < ntiles) dma_x(0, tile * BM);
    lds_dma_wait();
    // Whole-row logsumexp leaves `out` final without any exchange between the waves; only aux
    // needs all strips of a row.  The strips' pairs are parked in LDS and merged one iteration
    // later, behind the barrier the loop has anyway.
    epi.defer_lse = a.norm == FGE_NORM_LOGSUMEXP;
    int it = 0;
    for (; tile < ntiles; tile += gridDim.x, ++it) {
        const int buf = it & 1;
        __syncthreads();    // tile `it` has landed for every wave; reads of the other buffer are over
        if (epi.defer_lse && it > 0) epi.flush_lse(tid, (it - 1) & 1, (tile - (int)gridDim.x) * BM);
        const int next = tile + gridDim.x;
        if (next < ntiles) dma_x(buf ^ 1, next * BM);

        floatx16 acc[MB][NB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            u32x4 ahi[MB], alo[MB];
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const floatx4 x0 = *reinterpret_cast<const floatx4 *>(xs + buf * XTILE + fa_off[i][t][0]);
                const floatx4 x1 = *reinterpret_cast<const floatx4 *>(xs + buf * XTILE + fa_off[i][t][1]);
                const float f[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
                split_bf16x8(f, ahi[i], alo[i]);
            }
            // small terms first; the MB*NB accumulators keep successive MFMAs independent
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) mfma_bf16(alo[i], whi[j][t], acc[i][j]);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) mfma_bf16(ahi[i], wlo[j][t], acc[i][j]);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) mfma_bf16(ahi[i], whi[j][t], acc[i][j]);
        }
        // the epilogue waits for the copy of the next tile before it queues its stores
        epi.m0 = tile * BM;
        epi.lse_par = buf;
        epi.template tile<NT>(acc, 0, 0, tid);
    }
    if (epi.defer_lse && it > 0) {
        __syncthreads();
        epi.flush_lse(tid, (it - 1) & 1, (tile - (int)gridDim.x) * BM);
    }
}

}  // namespace fge
