// Register epilogue shared by the GEMM kernels: scale + bias + activation on the accumulators,
// in-tile row statistics, and either the final normalised store or the parked tile plus its
// per-tile statistics for the second pass.
//
// It works on one 32-row accumulator block of one wave at a time: `blk[j][r]` is the MFMA
// 32x32 accumulator of column block j, whose element r lives at
//     row = (r / 4) * 8 + (lane / 32) * 4 + r % 4,   column = j * 32 + lane % 32
// of the block.  A row's values are therefore lane-local over j, spread over the 32 lanes with
// equal lane/32, and over the WAVES_N waves of the workgroup that share the rows.
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
    static constexpr int PATCH_FLOATS = PATCH_ROWS * SSTR;  // per wave
    static_assert(PATCH_ROWS == 32 || PATCH_ROWS == 16, "patch");
    static_assert(RPP >= 1 && PATCH_ROWS % RPP == 0, "patch passes");

    const TileArgs &a;
    OutT *out;                  // base of this problem's output
    float *red;                 // LDS, [tile rows][WAVES_N]
    float *patch;               // LDS, this wave's PATCH_FLOATS
    int64_t row_base;           // z * M: offset of this problem in aux / ws
    int m0, n0, tn;             // tile origin and column-tile index
    int wave_n, lane, h, l32;
    int wcol0;                  // first global column of this lane
    bool cok[NB];
    float bias[NB], gam[NB], bet[NB];
    bool whole_row, writer;
    int ncols;

    __device__ __forceinline__ TileEpilogue(const TileArgs &a_, OutT *out_, float *red_, float *patch_,
                                            int z, int m0_, int n0_, int tn_, int wave_n_, int lane_)
        : a(a_), out(out_), red(red_), patch(patch_), row_base((int64_t)z * a_.M), m0(m0_), n0(n0_),
          tn(tn_), wave_n(wave_n_), lane(lane_), h(lane_ >> 5), l32(lane_ & 31) {
        wcol0 = n0 + wave_n * WTN + l32;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            cok[j] = wcol0 + j * 32 < a.N;
            bias[j] = (a.b != nullptr && cok[j]) ? a.b[wcol0 + j * 32] : 0.0f;
            gam[j] = (a.gamma != nullptr && cok[j]) ? a.gamma[wcol0 + j * 32] : 1.0f;
            bet[j] = (a.beta != nullptr && cok[j]) ? a.beta[wcol0 + j * 32] : 0.0f;
        }
        whole_row = a.tiles_n == 1;
        writer = wave_n == 0 && l32 == 0;             // one lane per accumulator row
        ncols = min(BN, a.N - n0);                    // valid columns of this tile
    }

    // row of accumulator element r inside the block
    __device__ __forceinline__ int brow(int r) const { return (r >> 2) * 8 + h * 4 + (r & 3); }

    // All-reduce one value per accumulator row over the tile's columns: across the 32 lanes of
    // the row, then across the WAVES_N waves through LDS.  trow0: first tile row of the block.
    template <typename Op> __device__ __forceinline__ void reduce_rows(float (&st)[16], int trow0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = allreduce32<Op>(st[r]);
        if constexpr (WAVES_N > 1) {
            __syncthreads();                          // previous use of `red` is over
            if (l32 == 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) red[(trow0 + brow(r)) * WAVES_N + wave_n] = st[r];
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float *p = red + (trow0 + brow(r)) * WAVES_N;
                float v = p[0];
#pragma unroll
                for (int w = 1; w < WAVES_N; ++w) v = Op::f(v, p[w]);
                st[r] = v;
            }
        }
    }

    // statistics of split rows: one float2 per (row, column tile)
    __device__ __forceinline__ void put_stats(int trow0, int r, float s0, float s1) {
        const int grow = m0 + trow0 + brow(r);
        if (writer && grow < a.M) a.ws[(row_base + grow) * a.tiles_n + tn] = make_float2(s0, s1);
    }

    template <int ACT> __device__ __forceinline__ void act_block(floatx16 (&blk)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                blk[j][r] = activate<ACT>(a.post * (a.alpha * blk[j][r] + bias[j]), a.lo, a.hi);
    }

    // (Tests of whole_row stay outside the unrolled loops: inside them the compiler keeps the
    // accumulators in scratch memory.)
    template <int NORM> __device__ __forceinline__ void norm_block(floatx16 (&blk)[NB], int trow0) {
        float st[16];
        if constexpr (NORM == FGE_NORM_SOFTMAX || NORM == FGE_NORM_LOGSUMEXP) {
            float mx[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float m = OpMax::ident();
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (cok[j]) m = fmaxf(m, blk[j][r]);
                st[r] = m;
            }
            reduce_rows<OpMax>(st, trow0);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                mx[r] = st[r];
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const float e = cok[j] ? fast_exp(blk[j][r] - mx[r]) : 0.0f;
                    if constexpr (NORM == FGE_NORM_SOFTMAX) blk[j][r] = e;
                    s += e;
                }
                st[r] = s;
            }
            reduce_rows<OpSum>(st, trow0);
            if (!whole_row) {
                // softmax parks exp(a - m_tile); the second pass rescales by exp(m_tile - m)/s
#pragma unroll
                for (int r = 0; r < 16; ++r) put_stats(trow0, r, mx[r], st[r]);
            } else if constexpr (NORM == FGE_NORM_SOFTMAX) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float inv = fast_rcp(st[r]);
#pragma unroll
                    for (int j = 0; j < NB; ++j) blk[j][r] *= inv;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int grow = m0 + trow0 + brow(r);
                    if (writer && grow < a.M) a.aux[row_base + grow] = mx[r] + __logf(st[r]);
                }
            }
        } else if constexpr (NORM == FGE_NORM_LAYERNORM) {
            float mean[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) s += cok[j] ? blk[j][r] : 0.0f;
                st[r] = s;
            }
            reduce_rows<OpSum>(st, trow0);
            const float inv_n = 1.0f / (float)ncols;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                mean[r] = st[r] * inv_n;
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const float d = blk[j][r] - mean[r];
                    s += cok[j] ? d * d : 0.0f;
                }
                st[r] = s;
            }
            reduce_rows<OpSum>(st, trow0);
            if (whole_row) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float rstd = rsqrtf(st[r] * inv_n + a.eps);
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        blk[j][r] = (blk[j][r] - mean[r]) * rstd * gam[j] + bet[j];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) put_stats(trow0, r, mean[r], st[r]);   // tile (mean, M2)
            }
        } else {  // FGE_NORM_RMSNORM
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) s += cok[j] ? blk[j][r] * blk[j][r] : 0.0f;
                st[r] = s;
            }
            reduce_rows<OpSum>(st, trow0);
            if (whole_row) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float rr = rsqrtf(st[r] / (float)a.N + a.eps);
#pragma unroll
                    for (int j = 0; j < NB; ++j) blk[j][r] *= rr * gam[j];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) put_stats(trow0, r, st[r], 0.0f);
            }
        }
    }

    // Store of the block through the wave-private LDS patch, so that global stores are 16 bytes
    // per lane and cover whole row segments: PATCH_ROWS rows at a time are written as fp32
    // [PATCH_ROWS][WTN + 8], read back row-wise, converted and stored.
    __device__ __forceinline__ void store_block(floatx16 (&blk)[NB], int trow0) {
        const int prow = lane / LPR, pcol = (lane % LPR) * VEC;
        const int gcol = n0 + wave_n * WTN + pcol;
        if constexpr (WAIT_VM) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int half = 0; half < 32 / PATCH_ROWS; ++half) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (PATCH_ROWS == 32 || (r >> 3) == half)
                        patch[(brow(r) - half * PATCH_ROWS) * SSTR + j * 32 + l32] = blk[j][r];
#pragma unroll
            for (int p = 0; p < PATCH_ROWS / RPP; ++p) {
                const int row = p * RPP + prow;
                const int grow = m0 + trow0 + half * PATCH_ROWS + row;
                float v[VEC];
#pragma unroll
                for (int e = 0; e < VEC; e += 4) {
                    const floatx4 f = *reinterpret_cast<const floatx4 *>(patch + row * SSTR + pcol + e);
                    v[e] = f[0]; v[e + 1] = f[1]; v[e + 2] = f[2]; v[e + 3] = f[3];
                }
                if (grow < a.M && gcol < a.N)         // N is a multiple of VEC: whole vector or none
                    *reinterpret_cast<uint4 *>(out + (int64_t)grow * a.ldo + gcol) = Store<OutT>::pack(v);
            }
        }
    }

    // activation -> statistics -> store of one block; trow0 = first tile row of the block
    __device__ __forceinline__ void block(floatx16 (&blk)[NB], int trow0) {
        dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) { act_block<ACT>(blk); });
        switch (a.norm) {
        case FGE_NORM_NONE:      break;
        case FGE_NORM_SOFTMAX:   norm_block<FGE_NORM_SOFTMAX>(blk, trow0); break;
        case FGE_NORM_LOGSUMEXP: norm_block<FGE_NORM_LOGSUMEXP>(blk, trow0); break;
        case FGE_NORM_LAYERNORM: norm_block<FGE_NORM_LAYERNORM>(blk, trow0); break;
        default:                 norm_block<FGE_NORM_RMSNORM>(blk, trow0); break;
        }
        store_block(blk, trow0);
    }
};

}  // namespace fge
