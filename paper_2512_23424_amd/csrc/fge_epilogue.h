// Register epilogue shared by the GEMM kernels: scale + bias + activation on the accumulators,
// in-tile row statistics, and either the final normalised store or the parked tile plus its
// per-tile statistics for the second pass.
//
// It works on one 32-row accumulator block of one wave at a time: `blk[j][r]` is the MFMA
// 32x32 accumulator of column block j, whose element r lives at
//     row = (r / 4) * 8 + (lane / 32) * 4 + r % 4,   column = j * 32 + lane % 32
// of the block.  Scale, bias and activation are applied in that layout.  The block then goes
// through a wave-private LDS patch into a row-wise layout - a lane holds 16 bytes' worth of
// neighbouring columns of one row, LPR neighbouring lanes hold a row segment - in which the row
// statistics need only log2(LPR) cross-lane steps per row (plus one LDS exchange between the
// WAVES_N waves sharing the rows) and the global stores are 16 bytes per lane over whole row
// segments.
#pragma once
#include "fge_device.h"

namespace fge {

struct TileArgs {
    const void *X, *W;
    const float *b, *gamma, *beta;
    void *out;
    float *aux;
    float2 *ws;                 // [batch*M][tiles_n] per-tile row statistics (split rows only)
    int M, N, K;
    int64_t ldx, ldw, ldo, bsx, bso;
    float alpha, post, lo, hi, eps;
    int act, norm;
    int tiles_m, tiles_n, group_m;
};

// OutT: storage type of out.  NB: 32-column blocks per wave.  WAVES_N: waves sharing a row.
// BN: tile width.  PATCH_ROWS (32 or 16): rows staged at a time in the wave's LDS patch.
// WAIT_VM: drain the wave's vector-memory counter before the first global store of a block
// (for callers that have asynchronous global->LDS loads in flight and want them accounted for
// before the stores are queued behind them).
template <typename OutT, int NB, int WAVES_N, int BN, int PATCH_ROWS, bool WAIT_VM>
struct TileEpilogue {
    static constexpr int WTN = NB * 32;
    static constexpr int SSTR = WTN + 8;              // floats per patch row: +8 puts lanes 0-31
                                                      // and 32-63 (four rows apart) on other banks
    static constexpr int VEC = 16 / (int)sizeof(OutT);
    static constexpr int LPR = WTN / VEC, RPP = 64 / LPR;   // lanes per row, rows per pass
    static constexpr int NP = PATCH_ROWS / RPP;             // passes over the patch
    static constexpr int PATCH_FLOATS = PATCH_ROWS * SSTR;  // per wave
    static_assert(PATCH_ROWS == 32 || PATCH_ROWS == 16, "patch");
    static_assert(RPP >= 1 && PATCH_ROWS % RPP == 0 && LPR <= 64, "patch passes");

    const TileArgs &a;
    OutT *out;                  // base of this problem's output
    float *red;                 // LDS, two buffers of [tile rows][WAVES_N], used alternately
    float *patch;               // LDS, this wave's PATCH_FLOATS
    int64_t row_base;           // z * M: offset of this problem in aux / ws
    int m0, n0, tn;             // tile origin and column-tile index
    int tile_rows;              // rows of the tile (stride between the two red buffers)
    int wave_n, lane, h, l32;
    int prow, pcol, gcol;       // row-wise layout: row in a pass, first column in the wave tile / globally
    bool vok;                   // this lane's column vector lies inside N (N is a multiple of VEC)
    bool rlead;                 // first lane of a row segment
    int red_par;                // which red buffer the next exchange uses
    float bias[NB];
    bool whole_row;
    int ncols;

    __device__ __forceinline__ TileEpilogue(const TileArgs &a_, OutT *out_, float *red_, float *patch_,
                                            int tile_rows_, int z, int m0_, int n0_, int tn_,
                                            int wave_n_, int lane_)
        : a(a_), out(out_), red(red_), patch(patch_), row_base((int64_t)z * a_.M), m0(m0_), n0(n0_),
          tn(tn_), tile_rows(tile_rows_), wave_n(wave_n_), lane(lane_), h(lane_ >> 5), l32(lane_ & 31) {
        const int wcol0 = n0 + wave_n * WTN + l32;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            bias[j] = (a.b != nullptr && wcol0 + j * 32 < a.N) ? a.b[wcol0 + j * 32] : 0.0f;
        prow = lane / LPR;
        pcol = (lane % LPR) * VEC;
        gcol = n0 + wave_n * WTN + pcol;
        vok = gcol < a.N;
        rlead = lane % LPR == 0;
        red_par = 0;
        whole_row = a.tiles_n == 1;
        ncols = min(BN, a.N - n0);                    // valid columns of this tile
    }

    // row of accumulator element r inside the block
    __device__ __forceinline__ int brow(int r) const { return (r >> 2) * 8 + h * 4 + (r & 3); }

    template <int ACT> __device__ __forceinline__ void act_block(floatx16 (&blk)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                blk[j][r] = activate<ACT>(a.post * (a.alpha * blk[j][r] + bias[j]), a.lo, a.hi);
    }

    // All-reduce st[p] (one value per row of pass p) over the tile's columns: across the LPR
    // lanes of the row segment, then across the WAVES_N waves through LDS.  The two red buffers
    // alternate, so one barrier per exchange is enough: a buffer is rewritten only after the
    // barrier of the exchange in between.  trow0: tile row of patch row 0.
    template <typename Op> __device__ __forceinline__ void reduce_rows(float (&st)[NP], int trow0) {
#pragma unroll
        for (int p = 0; p < NP; ++p) st[p] = allreduce_lanes<Op, LPR>(st[p]);
        if constexpr (WAVES_N > 1) {
            float *rb = red + red_par * tile_rows * WAVES_N;
            red_par ^= 1;
            if (rlead) {
#pragma unroll
                for (int p = 0; p < NP; ++p) rb[(trow0 + p * RPP + prow) * WAVES_N + wave_n] = st[p];
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const float *q = rb + (trow0 + p * RPP + prow) * WAVES_N;
                float v;
                if constexpr (WAVES_N % 4 == 0) {     // 16-byte LDS reads (red is 16-byte aligned)
                    floatx4 x = *reinterpret_cast<const floatx4 *>(q);
#pragma unroll
                    for (int w = 4; w < WAVES_N; w += 4) {
                        const floatx4 y = *reinterpret_cast<const floatx4 *>(q + w);
                        x[0] = Op::f(x[0], y[0]); x[1] = Op::f(x[1], y[1]);
                        x[2] = Op::f(x[2], y[2]); x[3] = Op::f(x[3], y[3]);
                    }
                    v = Op::f(Op::f(x[0], x[1]), Op::f(x[2], x[3]));
                } else {
                    v = q[0];
#pragma unroll
                    for (int w = 1; w < WAVES_N; ++w) v = Op::f(v, q[w]);
                }
                st[p] = v;
            }
        }
    }

    // Row operation on PATCH_ROWS rows in the row-wise layout: v[p][e] is column gcol + e of
    // patch row p*RPP + prow.  Whole rows are normalised in place; split rows keep the parked
    // value and publish their per-tile statistics (one float2 per row and column tile).
    template <int NORM> __device__ __forceinline__ void norm_rows(float (&v)[NP][VEC], int trow0) {
        float st[NP];
        const bool stat_writer = rlead && wave_n == 0;
        auto put_stats = [&](int p, float s0, float s1) __attribute__((always_inline)) {
            const int grow = m0 + trow0 + p * RPP + prow;
            if (stat_writer && grow < a.M) a.ws[(row_base + grow) * a.tiles_n + tn] = make_float2(s0, s1);
        };
        if constexpr (NORM == FGE_NORM_SOFTMAX || NORM == FGE_NORM_LOGSUMEXP) {
            float mx[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                float m = OpMax::ident();
#pragma unroll
                for (int e = 0; e < VEC; ++e) m = fmaxf(m, v[p][e]);
                st[p] = vok ? m : OpMax::ident();
            }
            reduce_rows<OpMax>(st, trow0);
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                mx[p] = st[p];
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float x = fast_exp(v[p][e] - mx[p]);
                    if constexpr (NORM == FGE_NORM_SOFTMAX) v[p][e] = x;
                    s += x;
                }
                st[p] = vok ? s : 0.0f;
            }
            reduce_rows<OpSum>(st, trow0);
            if (!whole_row) {
                // softmax parks exp(a - m_tile); the second pass rescales by exp(m_tile - m)/s
#pragma unroll
                for (int p = 0; p < NP; ++p) put_stats(p, mx[p], st[p]);
            } else if constexpr (NORM == FGE_NORM_SOFTMAX) {
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const float inv = fast_rcp(st[p]);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) v[p][e] *= inv;
                }
            } else {
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const int grow = m0 + trow0 + p * RPP + prow;
                    if (stat_writer && grow < a.M) a.aux[row_base + grow] = mx[p] + __logf(st[p]);
                }
            }
            return;
        }
        // gamma / beta of this lane's columns (only whole rows are normalised here)
        float gam[VEC], bet[VEC];
#pragma unroll
        for (int e = 0; e < VEC; e += 4) {
            floatx4 g = {1.0f, 1.0f, 1.0f, 1.0f}, b = {0.0f, 0.0f, 0.0f, 0.0f};
            if (whole_row && vok && a.gamma != nullptr) g = *reinterpret_cast<const floatx4 *>(a.gamma + gcol + e);
            if (whole_row && vok && a.beta != nullptr) b = *reinterpret_cast<const floatx4 *>(a.beta + gcol + e);
            gam[e] = g[0]; gam[e + 1] = g[1]; gam[e + 2] = g[2]; gam[e + 3] = g[3];
            bet[e] = b[0]; bet[e + 1] = b[1]; bet[e + 2] = b[2]; bet[e + 3] = b[3];
        }
        if constexpr (NORM == FGE_NORM_LAYERNORM) {
            float mean[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) s += v[p][e];
                st[p] = vok ? s : 0.0f;
            }
            reduce_rows<OpSum>(st, trow0);
            const float inv_n = 1.0f / (float)ncols;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                mean[p] = st[p] * inv_n;
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float d = v[p][e] - mean[p];
                    s += d * d;
                }
                st[p] = vok ? s : 0.0f;
            }
            reduce_rows<OpSum>(st, trow0);
            if (whole_row) {
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const float rstd = rsqrtf(st[p] * inv_n + a.eps);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) v[p][e] = (v[p][e] - mean[p]) * rstd * gam[e] + bet[e];
                }
            } else {
#pragma unroll
                for (int p = 0; p < NP; ++p) put_stats(p, mean[p], st[p]);   // tile (mean, M2)
            }
        } else {  // FGE_NORM_RMSNORM
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) s += v[p][e] * v[p][e];
                st[p] = vok ? s : 0.0f;
            }
            reduce_rows<OpSum>(st, trow0);
            if (whole_row) {
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const float rr = rsqrtf(st[p] / (float)a.N + a.eps);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) v[p][e] *= rr * gam[e];
                }
            } else {
#pragma unroll
                for (int p = 0; p < NP; ++p) put_stats(p, st[p], 0.0f);
            }
        }
    }

    // activation -> LDS patch -> row-wise statistics -> 16-byte global stores, for one 32-row
    // accumulator block; trow0 = first tile row of the block
    __device__ __forceinline__ void block(floatx16 (&blk)[NB], int trow0) {
        dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) { act_block<ACT>(blk); });
#pragma unroll
        for (int half = 0; half < 32 / PATCH_ROWS; ++half) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (PATCH_ROWS == 32 || (r >> 3) == half)
                        patch[(brow(r) - half * PATCH_ROWS) * SSTR + j * 32 + l32] = blk[j][r];
            float v[NP][VEC];
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int e = 0; e < VEC; e += 4) {
                    const floatx4 f = *reinterpret_cast<const floatx4 *>(patch + (p * RPP + prow) * SSTR + pcol + e);
                    v[p][e] = f[0]; v[p][e + 1] = f[1]; v[p][e + 2] = f[2]; v[p][e + 3] = f[3];
                }
            const int hrow0 = trow0 + half * PATCH_ROWS;
            switch (a.norm) {
            case FGE_NORM_NONE:      break;
            case FGE_NORM_SOFTMAX:   norm_rows<FGE_NORM_SOFTMAX>(v, hrow0); break;
            case FGE_NORM_LOGSUMEXP: norm_rows<FGE_NORM_LOGSUMEXP>(v, hrow0); break;
            case FGE_NORM_LAYERNORM: norm_rows<FGE_NORM_LAYERNORM>(v, hrow0); break;
            default:                 norm_rows<FGE_NORM_RMSNORM>(v, hrow0); break;
            }
            if constexpr (WAIT_VM) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int grow = m0 + hrow0 + p * RPP + prow;
                if (grow < a.M && vok)
                    *reinterpret_cast<uint4 *>(out + (int64_t)grow * a.ldo + gcol) = Store<OutT>::pack(v[p]);
            }
        }
    }
};

}  // namespace fge
