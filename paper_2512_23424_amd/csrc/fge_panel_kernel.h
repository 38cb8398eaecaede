// Narrow-K whole-row kernel for fp32 operands: K <= 64, N <= 512, many rows.
//
// Such a problem is bound by the output stream (every row reads K*4 bytes and writes N*4), so
// the kernel is organised around HBM, not around the matrix cores:
//   * persistent workgroups (one per CU, 8 waves side by side along N) walk over 64-row tiles;
//     W never leaves the registers: each wave keeps the MFMA B fragments of its 64 columns,
//     already split, for the whole launch;
//   * every wave multiplies all 64 rows of a tile, so the fp32 X tile is split into its bf16
//     parts once per workgroup (each thread fetches and splits 8 values) and parked in LDS as
//     two bf16 images; a tile's values are fetched a whole iteration before they are parked (the
//     fetch of the tile after next is issued right behind the parking of the next one, ahead of
//     the current tile's stores), so neither memory latency nor a store queue is waited for;
//   * scale and bias cost nothing per element: post_scale*alpha is folded into the register-
//     resident W fragments before they are split (one fp32 rounding per weight, none when the
//     factor is a power of two) and post_scale*b is the initial value of the accumulators;
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
// ACT_CT / NORM_CT / BOUNDED_CT: the chain fixed at compile time (see TileEpilogue), -1 to take
// it from the arguments.
template <typename OutT, bool FULL, bool STREAM, int ACT_CT = -1, int NORM_CT = -1, bool BOUNDED_CT = false>
__global__ __launch_bounds__(PanelShape::THREADS)
void panel_kernel(const TileArgs a) {
    constexpr int BM = PanelShape::BM, WAVES_N = PanelShape::WAVES_N;
    constexpr int MB = PanelShape::MB, NB = PanelShape::NB, NT = PanelShape::THREADS;
    constexpr int WTN = NB * 32;
    constexpr int SROWB = 128;                        // LDS bytes per row of a bf16 image: 64 values
    constexpr int SIMG = BM * SROWB;                  // 8 KB; an X buffer is the image of the high
    constexpr int XBUF = 2 * SIMG;                    // parts followed by the image of the low parts
    using Epi = TileEpilogue<OutT, MB, NB, WAVES_N, 16, false, false, false, FULL, STREAM, ACT_CT, NORM_CT, BOUNDED_CT, true>;
    static_assert(NT == BM * 8, "one thread per (row, 8 values of k) of an X tile");

    __shared__ __attribute__((aligned(16))) unsigned char xs[2 * XBUF];
    __shared__ __attribute__((aligned(16))) float2 xch[2 * BM * WAVES_N];
    __shared__ __attribute__((aligned(16))) float patches[(NT / 64) * Epi::PATCH_FLOATS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_n = wave;
    const int h = lane >> 5, l32 = lane & 31;
    const float *X = reinterpret_cast<const float *>(a.X);
    const float *W = reinterpret_cast<const float *>(a.W);
    OutT *out = reinterpret_cast<OutT *>(a.out);

    // ---------------- W fragments of this wave's 64 columns, split once, kept in registers
    // fragment (j, t): column wave_n*64 + j*32 + l32, k = 16t + 8h .. +7
    // scaled by post*alpha on the way in; the accumulators start from post*b (column l32 of block j
    // in every register of the block), so that they end as post*(alpha*x.w + b)
    const float wscale = a.post * a.alpha;
    u32x4 whi[NB][4], wlo[NB][4];
    float binit[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int col = wave_n * WTN + j * 32 + l32;
        binit[j] = (a.b != nullptr && col < a.N) ? a.post * a.b[col] : 0.0f;
        const float *wr = W + (int64_t)min(col, a.w_rows - 1) * a.ldw;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int k0 = 16 * t + 8 * h;
            float f[8];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                floatx4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (k0 + 4 * c < a.K) v = *reinterpret_cast<const floatx4 *>(wr + k0 + 4 * c);
                f[4 * c] = wscale * v[0]; f[4 * c + 1] = wscale * v[1]; f[4 * c + 2] = wscale * v[2]; f[4 * c + 3] = wscale * v[3];
            }
            split_bf16x8(f, whi[j][t], wlo[j][t]);
        }
    }

    // ---------------- X tiles.  Every wave multiplies all 64 rows, so the tile is split once for
    // the workgroup: thread (row, c) = (tid / 8, tid % 8) fetches the 8 values k = 8c .. 8c+7 of
    // its row into registers while the previous tile is multiplied, splits them, and parks the two
    // 16-byte bf16 chunks in LDS.  Image: 128-byte rows, chunk c stored at c ^ ((row >> 1) & 7),
    // which keeps the fragment reads below (32 rows x 2 chunks per instruction) off each other's
    // banks.  Values past K are zero.
    const int s_row = tid >> 3, s_c = tid & 7;
    const int s_off = s_row * SROWB + ((s_c ^ ((s_row >> 1) & 7)) << 4);
    floatx4 xin[2];
    auto load_x = [&](int m0) __attribute__((always_inline)) {
        const float *g = X + (int64_t)min(m0 + s_row, a.M - 1) * a.ldx + s_c * 8;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            xin[c] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
            if (s_c * 8 + 4 * c < a.K) xin[c] = *reinterpret_cast<const floatx4 *>(g + 4 * c);
        }
    };
    auto park_x = [&](int buf) __attribute__((always_inline)) {
        const float f[8] = {xin[0][0], xin[0][1], xin[0][2], xin[0][3], xin[1][0], xin[1][1], xin[1][2], xin[1][3]};
        u32x4 hi, lo;
        split_bf16x8(f, hi, lo);
        *reinterpret_cast<u32x4 *>(xs + buf * XBUF + s_off) = hi;
        *reinterpret_cast<u32x4 *>(xs + buf * XBUF + SIMG + s_off) = lo;
    };

    // A fragment (i, t): row i*32 + l32, k = 16t + 8h .. +7 = chunk 2t + h of that row
    int fa_off[MB][4];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int t = 0; t < 4; ++t)
            fa_off[i][t] = (i * 32 + l32) * SROWB + (((2 * t + h) ^ ((l32 >> 1) & 7)) << 4);

    Epi epi(a, out, xch, patches + wave * Epi::PATCH_FLOATS, BM, 0, 0, 0, 0, wave_n, lane);

    // ---------------- persistent loop over 64-row tiles.  At the top of an iteration the tile is
    // parked in LDS buffer `buf` and the registers hold the values of the next tile, fetched a
    // whole iteration ago; they are parked behind this tile's product, and the fetch of the tile
    // after next follows at once, still ahead of this tile's stores.
    const int ntiles = a.tiles_m;
    int tile = blockIdx.x;
    if (tile < ntiles) {
        load_x(tile * BM);
        park_x(0);
        if (tile + (int)gridDim.x < ntiles) load_x((tile + (int)gridDim.x) * BM);
    }
    // Whole-row logsumexp leaves `out` final without any exchange between the waves; only aux
    // needs all strips of a row.  The strips' pairs are parked in LDS and merged one iteration
    // later, behind the barrier the loop has anyway.
    epi.defer_lse = (NORM_CT >= 0 ? NORM_CT : a.norm) == FGE_NORM_LOGSUMEXP;
    int it = 0;
    for (; tile < ntiles; tile += gridDim.x, ++it) {
        const int buf = it & 1;
        __syncthreads();    // tile `it` is parked by every wave; reads of the other buffer are over
        if (epi.defer_lse && it > 0) epi.flush_lse(tid, (it - 1) & 1, (tile - (int)gridDim.x) * BM);
        const int next = tile + gridDim.x, next2 = next + gridDim.x;

        floatx16 acc[MB][NB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = binit[j];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            u32x4 ahi[MB], alo[MB];
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                ahi[i] = *reinterpret_cast<const u32x4 *>(xs + buf * XBUF + fa_off[i][t]);
                alo[i] = *reinterpret_cast<const u32x4 *>(xs + buf * XBUF + SIMG + fa_off[i][t]);
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
        if (next < ntiles) park_x(buf ^ 1);
        if (next2 < ntiles) load_x(next2 * BM);
        __builtin_amdgcn_sched_barrier(0);
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
