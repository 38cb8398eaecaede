// The tile kernel: MFMA mainloop with double-buffered LDS panels, accumulators kept in
// registers through scale + bias + activation, in-tile row statistics, and either the final
// normalised store (tile spans N) or a parked tile plus per-tile statistics for the light
// second pass (row split over several column tiles).
//
// One workgroup computes a BM x BN tile of  act(post_scale*(alpha*X.W^T + b)).
// Waves are laid out WAVES_M x WAVES_N; each owns (BM/WAVES_M) x (BN/WAVES_N) outputs as
// 32x32 MFMA blocks.  X rows feed the MFMA A operand and W rows the B operand, so in every
// accumulator register the 32 lanes with equal lane/32 hold 32 neighbouring columns of one
// output row: stores are 128-byte contiguous and a row reduction is lane-local over the
// wave's column blocks, then 5 cross-lane steps, then one LDS exchange between waves.
//
// LDS panel layout (both operands): row-major, 128 bytes of K per row (64 bf16 / 32 fp32),
// the eight 16-byte chunks of a row stored at chunk ^ (row & 7) so that the 16-byte fragment
// reads of 8 neighbouring rows touch all 32 banks.
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

// Logical tile index for a hardware workgroup id.  Workgroups are handed to the 8 XCDs round
// robin, so ids congruent mod 8 share an L2; give each XCD one contiguous range of logical
// tiles, then walk that range in groups of `group_m` row tiles, column-tile major inside a
// group, so the tiles resident on one XCD at a time share few X and W panels.
__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int group_m,
                                            int &tm, int &tn) {
    const int nt = tiles_m * tiles_n;
    const int q = nt >> 3, rem = nt & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * q + (xcd < rem ? xcd : rem) + slot;
    const int per_group = group_m * tiles_n;
    const int g = logical / per_group;
    const int first_m = g * group_m;
    const int gm = min(group_m, tiles_m - first_m);
    const int idx = logical - g * per_group;
    tm = first_m + idx % gm;
    tn = idx / gm;
}

template <typename InT> struct Mma;
template <> struct Mma<bf16_t> {
    __device__ static __forceinline__ void run(const u32x4 &a, const u32x4 &b, floatx16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                    __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    // A 16-byte fragment holds 4 consecutive k of one row; lanes 0-31 and 32-63 hold different
    // chunks.  The k pairing is the same for both operands, so the sum over k is complete.
    // (as_f32 takes the element by value: a bit cast applied directly to a vector-element
    // lvalue reads element 0 whichever element is named.)
    __device__ static __forceinline__ void run(const u32x4 &a, const u32x4 &b, floatx16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(a.x), as_f32(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(a.y), as_f32(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(a.z), as_f32(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(a.w), as_f32(b.w), c, 0, 0, 0);
    }
};

template <typename InT, typename OutT, int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N)
void tile_kernel(const TileArgs a) {
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int MB = WTM / 32, NB = WTN / 32;
    constexpr int ROWB = 128;                        // bytes of K per LDS row
    constexpr int BK = ROWB / (int)sizeof(InT);      // 64 bf16 / 32 fp32
    constexpr int CW = 16 / (int)sizeof(InT);        // elements per 16-byte chunk
    constexpr int A_LD = BM * 8 / NT, B_LD = BN * 8 / NT;
    constexpr int RSTEP = NT / 8;                    // rows between a thread's successive chunks
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0 && RSTEP % 8 == 0, "load plan");
    constexpr int STAGE = (BM + BN) * ROWB;

    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];
    __shared__ float red[BM * WAVES_N];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int h = lane >> 5, l32 = lane & 31;

    int tm, tn;
    tile_coords(blockIdx.x, a.tiles_m, a.tiles_n, a.group_m, tm, tn);
    const int z = blockIdx.z;
    const int m0 = tm * BM, n0 = tn * BN;

    const InT *X = reinterpret_cast<const InT *>(a.X) + (int64_t)z * a.bsx;
    const InT *W = reinterpret_cast<const InT *>(a.W);
    OutT *out = reinterpret_cast<OutT *>(a.out) + (int64_t)z * a.bso;

    // ---------------- global -> register -> LDS staging plan
    // Thread t stages chunk (t & 7) of rows (t >> 3) + i*RSTEP.  Rows past the end of X / W are
    // clamped to the last valid row: they only feed outputs that are never stored or counted.
    // Only a partial last K tile needs zero fill.
    const int ld_row = tid >> 3, ld_c = tid & 7;
    const int ld_soff = ld_row * ROWB + ((ld_c ^ (ld_row & 7)) << 4);
    const InT *gA[A_LD];
    const InT *gB[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
        gA[i] = X + (int64_t)min(m0 + ld_row + i * RSTEP, a.M - 1) * a.ldx + ld_c * CW;
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
        gB[i] = W + (int64_t)min(n0 + ld_row + i * RSTEP, a.N - 1) * a.ldw + ld_c * CW;
    u32x4 rA[A_LD], rB[B_LD];

    auto load_global = [&]<bool TAIL>(int k0) __attribute__((always_inline)) {
        const bool kok = !TAIL || k0 + ld_c * CW < a.K;   // K is a multiple of CW: chunks are whole
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            rA[i] = u32x4{0u, 0u, 0u, 0u};
            if (kok) rA[i] = *reinterpret_cast<const u32x4 *>(gA[i] + k0);
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            rB[i] = u32x4{0u, 0u, 0u, 0u};
            if (kok) rB[i] = *reinterpret_cast<const u32x4 *>(gB[i] + k0);
        }
    };
    auto store_lds = [&](int buf) __attribute__((always_inline)) {
        unsigned char *sA = smem + buf * STAGE, *sB = sA + BM * ROWB;
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            *reinterpret_cast<u32x4 *>(sA + ld_soff + i * RSTEP * ROWB) = rA[i];
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            *reinterpret_cast<u32x4 *>(sB + ld_soff + i * RSTEP * ROWB) = rB[i];
    };

    // ---------------- fragment read plan
    const int fa_row = wave_m * WTM + l32, fb_row = wave_n * WTN + l32;
    int fsw[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) fsw[t] = ((2 * t + h) ^ (l32 & 7)) << 4;

    floatx16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // ---------------- mainloop
    const int KT = (a.K + BK - 1) / BK;
    const bool ragged_k = (a.K % BK) != 0;            // then the last tile is partial
    if (KT == 1 && ragged_k) load_global.template operator()<true>(0);
    else                     load_global.template operator()<false>(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) {
            if (kt + 2 == KT && ragged_k) load_global.template operator()<true>((kt + 1) * BK);
            else                          load_global.template operator()<false>((kt + 1) * BK);
        }
        const unsigned char *sA = smem + buf * STAGE + fa_row * ROWB;
        const unsigned char *sB = smem + buf * STAGE + BM * ROWB + fb_row * ROWB;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            u32x4 fa[MB], fb[NB];
#pragma unroll
            for (int i = 0; i < MB; ++i)
                fa[i] = *reinterpret_cast<const u32x4 *>(sA + i * 32 * ROWB + fsw[t]);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                fb[j] = *reinterpret_cast<const u32x4 *>(sB + j * 32 * ROWB + fsw[t]);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) Mma<InT>::run(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---------------- epilogue: scale + bias + activation in registers
    // accumulator element (i, j, r): row = wave_m*WTM + i*32 + (r/4)*8 + h*4 + r%4,
    //                                col = wave_n*WTN + j*32 + l32
    const int wrow0 = wave_m * WTM + h * 4;
    const int wcol0 = n0 + wave_n * WTN + l32;
    bool cok[NB];
    float bias[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        cok[j] = wcol0 + j * 32 < a.N;
        bias[j] = (a.b != nullptr && cok[j]) ? a.b[wcol0 + j * 32] : 0.0f;
    }
    auto act_block = [&]<int i>() __attribute__((always_inline)) {
        dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[i][j][r] = activate<ACT>(a.post * (a.alpha * acc[i][j][r] + bias[j]), a.lo, a.hi);
        });
    };
    auto row_of = [&](int i, int r) __attribute__((always_inline)) { return wrow0 + i * 32 + (r >> 2) * 8 + (r & 3); };
    auto store_block = [&]<int i>() __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int grow = m0 + row_of(i, r);
            if (grow < a.M) {
                OutT *o = out + (int64_t)grow * a.ldo + wcol0;
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (cok[j]) Store<OutT>::put(o + j * 32, acc[i][j][r]);
            }
        }
    };

    // ---------------- in-tile row statistics, one 32-row accumulator block at a time
    const bool whole_row = a.tiles_n == 1;
    const int ncols = min(BN, a.N - n0);              // valid columns of this tile
    float gam[NB], bet[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        gam[j] = (a.gamma != nullptr && cok[j]) ? a.gamma[wcol0 + j * 32] : 1.0f;
        bet[j] = (a.beta != nullptr && cok[j]) ? a.beta[wcol0 + j * 32] : 0.0f;
    }
    const bool writer = wave_n == 0 && l32 == 0;      // one lane per accumulator row

    auto norm_block = [&]<int NORM, int i>() __attribute__((always_inline)) {
        float st[16];
        // All-reduce one value per accumulator row over the tile's BN columns: across the 32
        // lanes of the row, then across the WAVES_N waves through LDS.
        auto reduce_rows = [&]<typename Op>(Op) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) st[r] = allreduce32<Op>(st[r]);
            if constexpr (WAVES_N > 1) {
                __syncthreads();                      // previous use of `red` is over
                if (l32 == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[row_of(i, r) * WAVES_N + wave_n] = st[r];
                }
                __syncthreads();
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float *p = red + row_of(i, r) * WAVES_N;
                    float v = p[0];
#pragma unroll
                    for (int w = 1; w < WAVES_N; ++w) v = Op::f(v, p[w]);
                    st[r] = v;
                }
            }
        };
        // statistics of split rows: one float2 per (row, column tile)
        auto put_stats = [&](int r, float s0, float s1) __attribute__((always_inline)) {
            const int grow = m0 + row_of(i, r);
            if (writer && grow < a.M)
                a.ws[((int64_t)z * a.M + grow) * a.tiles_n + tn] = make_float2(s0, s1);
        };

        if constexpr (NORM == FGE_NORM_SOFTMAX || NORM == FGE_NORM_LOGSUMEXP) {
            float mx[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float m = OpMax::ident();
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (cok[j]) m = fmaxf(m, acc[i][j][r]);
                st[r] = m;
            }
            reduce_rows(OpMax{});
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                mx[r] = st[r];
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const float e = cok[j] ? fast_exp(acc[i][j][r] - mx[r]) : 0.0f;
                    if constexpr (NORM == FGE_NORM_SOFTMAX) acc[i][j][r] = e;
                    s += e;
                }
                st[r] = s;
            }
            reduce_rows(OpSum{});
            // (the whole_row test stays outside the unrolled loops: inside them the compiler
            // keeps the accumulators in scratch memory)
            if (!whole_row) {
                // softmax parks exp(a - m_tile); the second pass rescales by exp(m_tile - m)/s
#pragma unroll
                for (int r = 0; r < 16; ++r) put_stats(r, mx[r], st[r]);
            } else if constexpr (NORM == FGE_NORM_SOFTMAX) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float inv = fast_rcp(st[r]);
#pragma unroll
                    for (int j = 0; j < NB; ++j) acc[i][j][r] *= inv;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int grow = m0 + row_of(i, r);
                    if (writer && grow < a.M)
                        a.aux[(int64_t)z * a.M + grow] = mx[r] + __logf(st[r]);
                }
            }
        } else if constexpr (NORM == FGE_NORM_LAYERNORM) {
            float mean[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) s += cok[j] ? acc[i][j][r] : 0.0f;
                st[r] = s;
            }
            reduce_rows(OpSum{});
            const float inv_n = 1.0f / (float)ncols;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                mean[r] = st[r] * inv_n;
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const float d = acc[i][j][r] - mean[r];
                    s += cok[j] ? d * d : 0.0f;
                }
                st[r] = s;
            }
            reduce_rows(OpSum{});
            if (whole_row) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float rstd = rsqrtf(st[r] * inv_n + a.eps);
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j][r] = (acc[i][j][r] - mean[r]) * rstd * gam[j] + bet[j];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) put_stats(r, mean[r], st[r]);   // tile (mean, M2)
            }
        } else {  // FGE_NORM_RMSNORM
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < NB; ++j) s += cok[j] ? acc[i][j][r] * acc[i][j][r] : 0.0f;
                st[r] = s;
            }
            reduce_rows(OpSum{});
            if (whole_row) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float rr = rsqrtf(st[r] / (float)a.N + a.eps);
#pragma unroll
                    for (int j = 0; j < NB; ++j) acc[i][j][r] *= rr * gam[j];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) put_stats(r, st[r], 0.0f);
            }
        }
    };
    // Each 32-row accumulator block goes through activation, statistics and store on its own,
    // so only one block's values are live in the vector registers at a time.
    static_for<0, MB>([&]<int i>() __attribute__((always_inline)) {
        act_block.template operator()<i>();
        switch (a.norm) {
        case FGE_NORM_NONE:      break;
        case FGE_NORM_SOFTMAX:   norm_block.template operator()<FGE_NORM_SOFTMAX, i>(); break;
        case FGE_NORM_LOGSUMEXP: norm_block.template operator()<FGE_NORM_LOGSUMEXP, i>(); break;
        case FGE_NORM_LAYERNORM: norm_block.template operator()<FGE_NORM_LAYERNORM, i>(); break;
        default:                 norm_block.template operator()<FGE_NORM_RMSNORM, i>(); break;
        }
        store_block.template operator()<i>();
    });
}

}  // namespace fge
