// Register epilogue shared by the GEMM kernels: scale + bias + activation on the accumulators,
// in-tile row statistics, and the store - final when the tile spans the row or when the tiles
// of a row block finish their rows together (cooperative form), otherwise the parked tile plus
// its per-strip statistics for the second pass.
//
// It works on one 32-row accumulator block of one wave at a time: `blk[j][r]` is the MFMA
// 32x32 accumulator of column block j, whose element r lives at
//     row = (r / 4) * 8 + (lane / 32) * 4 + r % 4,   column = j * 32 + lane % 32
// of the block.  Scale, bias and activation are applied in that layout.  The block then goes
// through a wave-private LDS patch into a row-wise layout - a lane holds 8 columns of one row,
// LPR neighbouring lanes hold a row segment - in which the row statistics need only log2(LPR)
// cross-lane steps per row and the global stores are 16 bytes per lane over whole row segments.
//
// Every wave first reduces its own strip of WTN columns to a mergeable pair per row:
//     softmax / logsumexp (m, s = sum exp(a - m)),  LayerNorm (mean, M2),  RMSNorm (sum a^2, -).
// Rows that the tile spans are finished in place: the WAVES_N pairs of a row meet in LDS (one
// barrier) and are merged (online-softmax merge, Chan's variance merge, plain sum).  Rows split
// over several column tiles either publish the pair per (row, strip) for the second pass - no
// exchange between waves at all - or, in the cooperative form, merge per tile, exchange one pair
// per (row, tile) through the workspace and finish from registers (see further down).
#pragma once
#include "fge_device.h"

namespace fge {

struct TileArgs {
    const void *X, *W;
    const void *W2;             // gated form: second weight matrix (else unused)
    const float *b, *gamma, *beta;
    const float *b2;            // gated form: bias of the second product (may be null)
    void *out;
    float *aux;
    float2 *ws;                 // split rows: [batch*M][tiles_n * waves across] strip pairs for the
                                // second pass, or [batch*M][tiles_n] tile pairs (cooperative form)
    int M, N, K;
    int w_rows;                 // rows of W that exist (N, or fewer when the columns from there on are padding:
                                // they are fed from row w_rows - 1 and their results are never looked at)
    int64_t ldx, ldw, ldo, bsx, bso;
    int64_t bsw;                // offset of problem z in W (0: W is shared; a K-split gives each slice its own k range)
    float alpha, post, lo, hi, eps;
    int act, norm;
    int tiles_m, tiles_n, group_m, batch;
    // cooperative completion of split rows (coop != 0): persistent grid, the column tiles of a
    // row block run in the same round and finish their rows themselves
    int coop;
    unsigned gen;               // value that marks "arrived" in this launch
    unsigned *arrive;           // [batch * tiles_m][tiles_n] arrival marks
    int *fault;                 // set to 1 if a wait ran out (the rows of that tile are then stored as NaN)
    int stream_out;             // store `out` with the streaming hint
    int stagger, stagger_mask;  // cooperative form: row block rb of the first round starts (rb & mask) * stagger * 1024 clocks late
    unsigned spin_limit;        // polls after which a wait gives up
    int withhold;               // tests only: column tile 0 never marks itself as arrived
};

// OutT: storage type of out.  MB x NB: 32x32 accumulator blocks per wave.  WAVES_N: waves
// sharing a row.  PATCH_ROWS (32 or 16): rows staged at a time in the wave's LDS patch.
// JOINT: all MB blocks of the wave go through one statistics step (one exchange per tile; for
// tiles that span N) instead of one per block (less register pressure; split rows never
// exchange anyway).  WAIT_VM: drain the wave's vector-memory counter before the first global
// store of a group (for callers with asynchronous global->LDS loads in flight that want them
// accounted for before stores are queued behind them).  COOP: the cooperative form only - rows
// are split over column tiles that are all in flight and finish their rows themselves.
// FULL_TILE: the caller guarantees that every tile lies inside the matrix (M and N are multiples
// of the tile shape), so no row or column needs a guard.  STREAM_OUT: the output is too large
// for the last-level cache; it is stored with the streaming hint, which keeps it from displacing
// the operands on its way out (nothing of it would still be cached for a consumer anyway).
// ACT_CT / NORM_CT (>= 0): activation and row op fixed at compile time - the tile's epilogue is
// then one straight line of code the compiler can schedule as a whole, instead of a chain of
// uniform branches; BOUNDED_CT says which softmax / logsumexp variant (see `bounded`) that is.
// PLAIN_ACC: the caller's accumulators already hold post*(alpha*x.w + b) (scale folded into an
// operand, bias into the initial accumulator value), so no scale + bias step is applied.
template <typename OutT, int MB, int NB, int WAVES_N, int PATCH_ROWS, bool JOINT, bool WAIT_VM, bool COOP = false,
          bool FULL_TILE = false, bool STREAM_OUT = false, int ACT_CT = -1, int NORM_CT = -1, bool BOUNDED_CT = false,
          bool PLAIN_ACC = false>
struct TileEpilogue {
    static constexpr int WTN = NB * 32;               // columns of a wave strip
    // Patch layout.  A patch row is written 32 columns at a time by the lanes 0-31 (row R) and
    // 32-63 (row R + 4) of an accumulator register, and read back 16 bytes per lane by 16 lanes
    // at a time.  With 4-byte results and 64-column strips a lane reads two 16-byte groups half a
    // strip apart, so 16 lanes cover one half of two neighbouring rows: writes and reads are both
    // free of bank conflicts (64 banks of 4 bytes) when rows are unpadded (one bank line each)
    // and the two 32-column halves are swapped in the rows whose bits 0 and 2 differ - rows four
    // apart and neighbouring rows then sit in opposite halves of the bank line.  (Measured on
    // the narrow-K kernel: conflicts 30 % -> 2 % of the LDS-active cycles.)  Every other case
    // keeps rows padded by 8 floats: conflict-free writes, two-way conflicts on the reads; the
    // analogous swap of 4-column groups for 16-bit results measured 1.5 % slower on the
    // epilogue-heavy batched workload (two more address registers in a kernel short of them).
    static constexpr bool XORP = WTN == 64 && sizeof(OutT) == 4;
    static constexpr int SSTR = XORP ? WTN : WTN + 8;   // floats per patch row
    static constexpr int VEC = 8;                     // columns per lane in the row-wise layout, as
                                                      // two groups of 4: neighbours for bf16 (one
                                                      // 16-byte store), half a strip apart for fp32
                                                      // (two 16-byte stores, each contiguous over
                                                      // the lanes of a row segment)
    static constexpr int G4STEP = sizeof(OutT) == 2 ? 4 : WTN / 2;   // columns between the groups
    static constexpr int SUBW = sizeof(OutT) == 2 ? 8 : 4;           // columns between lanes
    static constexpr int LPR = WTN / VEC, RPP = 64 / LPR;   // lanes per row, rows per pass
    static constexpr int NPH = PATCH_ROWS / RPP;            // passes per patch fill
    static constexpr int NPB = 32 / RPP;                    // passes per 32-row block
    static constexpr int G = JOINT ? MB : 1;                // blocks per statistics group
    static constexpr int NPG = G * NPB;                     // passes per group
    static constexpr int PATCH_FLOATS = PATCH_ROWS * SSTR;  // per wave
    static_assert(PATCH_ROWS == 32 || PATCH_ROWS == 16, "patch");
    static_assert(RPP >= 1 && PATCH_ROWS % RPP == 0 && LPR <= 64 && LPR >= WAVES_N, "patch passes");

    const TileArgs &a;
    OutT *out;                  // base of this problem's output
    float2 *xch;                // LDS, two buffers of [tile rows][WAVES_N] pairs, used alternately
    float *patch;               // LDS, this wave's PATCH_FLOATS
    int64_t row_base;           // z * M: offset of this problem in aux / ws
    int m0, n0, tn;             // tile origin and column-tile index
    int tile_rows;              // rows of the tile (stride between the two exchange buffers)
    int wave_n, lane, h, l32;
    int prow, pcol, gcol;       // row-wise layout: row in a pass, first column (of group 0) in
                                // the strip / globally; group 1 lies G4STEP columns further
    int sub;                    // lane index inside its row segment
    int wsel[2];                // patch layout: column of this lane in a 32-column write, by (block ^ row bit 0)
    int rsel[2];                // ... and first column of its two 4-column read groups
    bool ok4[2];                // columns gcol..+3 / gcol+4..+7 lie inside N (N is a multiple of 4)
    int xch_par;                // which exchange buffer the next exchange uses
    float scale, bias[NB];      // y = scale * acc + bias  (scale = post*alpha, bias = post*b)
    bool whole_row;
    bool bounded;               // clamp activation with a narrow range feeds softmax / logsumexp
    bool defer_lse = false;     // whole-row logsumexp: park the strip pairs, the caller merges them later
    int lse_par = 0;            // exchange buffer the parked pairs of this tile go to

    __device__ __forceinline__ TileEpilogue(const TileArgs &a_, OutT *out_, float2 *xch_, float *patch_,
                                            int tile_rows_, int z, int m0_, int n0_, int tn_,
                                            int wave_n_, int lane_)
        : a(a_), out(out_), xch(xch_), patch(patch_), row_base((int64_t)z * a_.M), m0(m0_), n0(n0_),
          tn(tn_), tile_rows(tile_rows_), wave_n(wave_n_), lane(lane_), h(lane_ >> 5), l32(lane_ & 31) {
        const int wcol0 = n0 + wave_n * WTN + l32;
        scale = a.post * a.alpha;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            bias[j] = (a.b != nullptr && wcol0 + j * 32 < a.N) ? a.post * a.b[wcol0 + j * 32] : 0.0f;
        prow = lane / LPR;
        sub = lane % LPR;
        pcol = sub * SUBW;
        gcol = n0 + wave_n * WTN + pcol;
        ok4[0] = gcol < a.N;
        ok4[1] = gcol + G4STEP < a.N;
        if constexpr (XORP) {                              // halves swapped where row bits 0 and 2 differ
            const int f = (prow ^ (prow >> 2)) & 1;
            wsel[0] = (h << 5) + l32;        wsel[1] = ((h ^ 1) << 5) + l32;
            rsel[0] = pcol + (f << 5);       rsel[1] = pcol + ((f ^ 1) << 5);
        } else {
            wsel[0] = wsel[1] = l32;
            rsel[0] = pcol;                  rsel[1] = pcol + G4STEP;
        }
        xch_par = 0;
        whole_row = a.tiles_n == 1;
        // (not in the cooperative form, whose registers are too scarce for two more variants)
        bounded = !COOP && a.act == FGE_ACT_CLAMP && a.hi - a.lo <= 64.0f;
    }

    // valid columns of strip w of this tile
    __device__ __forceinline__ int strip_cols(int w) const { return max(0, min(WTN, a.N - (n0 + w * WTN))); }
    // row of accumulator element r inside its block
    __device__ __forceinline__ int brow(int r) const { return (r >> 2) * 8 + h * 4 + (r & 3); }
    // tile row of pass q of a group whose first block starts at tile row grow0
    __device__ __forceinline__ int qrow(int grow0, int q) const { return grow0 + (q / NPB) * 32 + (q % NPB) * RPP + prow; }

    template <int ACT> __device__ __forceinline__ void act_block(floatx16 (&blk)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                blk[j][r] = activate<ACT>(PLAIN_ACC ? blk[j][r] : scale * blk[j][r] + bias[j], a.lo, a.hi);
    }

    // Publish the strip pair of pass q: to the workspace for the second pass, or (cooperative
    // form) to LDS, where the tile's strips are merged before anything leaves the workgroup.
    // FULL (here and below): the tile lies inside the matrix, no row or column needs a guard.
    template <bool FULL> __device__ __forceinline__ void put_stats(int grow0, int q, float s0, float s1) {
        if constexpr (COOP) {
            if (sub == 0) xch[qrow(grow0, q) * WAVES_N + wave_n] = make_float2(s0, s1);
        } else {
            const int grow = m0 + qrow(grow0, q);
            if (sub == 0 && (FULL || grow < a.M))
                a.ws[(row_base + grow) * (a.tiles_n * WAVES_N) + tn * WAVES_N + wave_n] = make_float2(s0, s1);
        }
    }
    // Cooperative form: the pairs travel between workgroups of one launch, possibly on different
    // XCDs with separate L2s.  Both sides use device-scope atomic accesses (which go to the
    // device-coherent level), so no cache-wide write-back or invalidate is needed.
    static __device__ __forceinline__ void put_pair(float2 *slot, float s0, float s1) {
        const uint64_t bits = (uint64_t)as_u32(s0) | ((uint64_t)as_u32(s1) << 32);
        __hip_atomic_store(reinterpret_cast<uint64_t *>(slot), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    static __device__ __forceinline__ float2 get_pair(const float2 *slot) {
        const uint64_t bits = __hip_atomic_load(reinterpret_cast<const uint64_t *>(slot), __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
        return make_float2(as_f32((uint32_t)bits), as_f32((uint32_t)(bits >> 32)));
    }
    // Whole rows: every strip's pair of every row of the group meets in LDS; afterwards lane
    // `sub` of a row segment holds the pair of strip `sub` (identity beyond WAVES_N).  The two
    // buffers alternate, so one barrier per exchange is enough: a buffer is rewritten only
    // after the barrier of the exchange in between.
    __device__ __forceinline__ void exchange(int grow0, float (&s0)[NPG], float (&s1)[NPG], float ident0) {
        if constexpr (WAVES_N > 1) {
            float2 *xb = xch + xch_par * tile_rows * WAVES_N;
            xch_par ^= 1;
            if (sub == 0) {
#pragma unroll
                for (int q = 0; q < NPG; ++q) xb[qrow(grow0, q) * WAVES_N + wave_n] = make_float2(s0[q], s1[q]);
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                float2 e = make_float2(ident0, 0.0f);
                if (sub < WAVES_N) e = xb[qrow(grow0, q) * WAVES_N + sub];
                s0[q] = e.x;
                s1[q] = e.y;
            }
        } else {
#pragma unroll
            for (int q = 0; q < NPG; ++q)
                if (sub != 0) { s0[q] = ident0; s1[q] = 0.0f; }
        }
    }

    // Row operation on one group in the row-wise layout: v[q][e] is column gcol + (e/4)*G4STEP + e%4 of tile row
    // qrow(grow0, q).  Whole rows are normalised in place; split rows keep the parked value.
    // BOUNDED (softmax / logsumexp after a clamp): every value lies in [lo, hi] with hi - lo
    // small, so hi serves as the reference of the exponentials and no maximum is searched.
    template <int NORM, bool FULL, bool BOUNDED>
    __device__ __forceinline__ void norm_group(float (&v)[NPG][VEC], int grow0, float (&mkeep)[NPG]) {
        auto okc = [&](int e) __attribute__((always_inline)) { return FULL || ok4[e >> 2]; };
        float s0[NPG], s1[NPG];
        if constexpr (NORM == FGE_NORM_SOFTMAX || NORM == FGE_NORM_LOGSUMEXP) {
            float ml[NPG];                            // strip maxima (or the common bound)
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                if constexpr (BOUNDED) {
                    ml[q] = a.hi;
                } else {
                    float m = OpMax::ident();
#pragma unroll
                    for (int e = 0; e < VEC; ++e) m = max_nc(m, okc(e) ? v[q][e] : OpMax::ident());
                    ml[q] = allreduce_lanes<OpMax, LPR>(m);
                }
            }
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                const float c = -ml[q] * LOG2E;
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float x = exp_rel(v[q][e], c);
                    if constexpr (NORM == FGE_NORM_SOFTMAX) v[q][e] = x;
                    s += okc(e) ? x : 0.0f;
                }
                s0[q] = ml[q];
                s1[q] = allreduce_lanes<OpSum, LPR>(s);
                mkeep[q] = ml[q];
            }
            if (!whole_row) {
                // softmax parks exp(a - m_strip); the second pass rescales by exp(m_strip - m)/s
#pragma unroll
                for (int q = 0; q < NPG; ++q) put_stats<FULL>(grow0, q, s0[q], s1[q]);
                return;
            }
            if constexpr (NORM == FGE_NORM_LOGSUMEXP) {
                if (defer_lse) {          // out is already final; only aux needs the other strips
                    if (sub == 0) {
#pragma unroll
                        for (int q = 0; q < NPG; ++q)
                            xch[(lse_par * tile_rows + qrow(grow0, q)) * WAVES_N + wave_n] = make_float2(s0[q], s1[q]);
                    }
                    return;
                }
            }
            exchange(grow0, s0, s1, OpMax::ident());
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                float m, s;
                if constexpr (BOUNDED) {                  // all references are equal
                    m = a.hi;
                    s = allreduce_lanes<OpSum, LPR>(s1[q]);
                } else {
                    m = allreduce_lanes<OpMax, LPR>(s0[q]);
                    s = allreduce_lanes<OpSum, LPR>(s1[q] * fast_exp(s0[q] - m));
                }
                if constexpr (NORM == FGE_NORM_SOFTMAX) {
                    const float f = (BOUNDED ? 1.0f : fast_exp(ml[q] - m)) * fast_rcp(s);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) v[q][e] *= f;
                } else {
                    const int grow = m0 + qrow(grow0, q);
                    if (sub == 0 && wave_n == 0 && (FULL || grow < a.M)) a.aux[row_base + grow] = m + __logf(s);
                }
            }
            return;
        }
        // gamma / beta of this lane's columns (only whole rows are normalised here)
        float gam[VEC], bet[VEC];
#pragma unroll
        for (int e = 0; e < VEC; e += 4) {
            floatx4 g = {1.0f, 1.0f, 1.0f, 1.0f}, b = {0.0f, 0.0f, 0.0f, 0.0f};
            const int c = gcol + (e >> 2) * G4STEP;
            if (whole_row && okc(e) && a.gamma != nullptr) g = *reinterpret_cast<const floatx4 *>(a.gamma + c);
            if (whole_row && okc(e) && a.beta != nullptr) b = *reinterpret_cast<const floatx4 *>(a.beta + c);
            gam[e] = g[0]; gam[e + 1] = g[1]; gam[e + 2] = g[2]; gam[e + 3] = g[3];
            bet[e] = b[0]; bet[e + 1] = b[1]; bet[e + 2] = b[2]; bet[e + 3] = b[3];
        }
        if constexpr (NORM == FGE_NORM_LAYERNORM) {
            const int nl = FULL ? WTN : strip_cols(wave_n);
            const float inv_nl = nl > 0 ? 1.0f / (float)nl : 0.0f;
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) s += okc(e) ? v[q][e] : 0.0f;
                s0[q] = allreduce_lanes<OpSum, LPR>(s) * inv_nl;                  // strip mean
                float d2 = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float d = v[q][e] - s0[q];
                    d2 += okc(e) ? d * d : 0.0f;
                }
                s1[q] = allreduce_lanes<OpSum, LPR>(d2);                          // strip M2
            }
            if (!whole_row) {
#pragma unroll
                for (int q = 0; q < NPG; ++q) put_stats<FULL>(grow0, q, s0[q], s1[q]);
                return;
            }
            exchange(grow0, s0, s1, 0.0f);
            const float nw = sub < WAVES_N ? (float)strip_cols(sub) : 0.0f;       // columns behind this lane's pair
            const float inv_n = 1.0f / (float)a.N;
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                const float mean = allreduce_lanes<OpSum, LPR>(nw * s0[q]) * inv_n;
                const float d = s0[q] - mean;
                const float m2 = allreduce_lanes<OpSum, LPR>(s1[q] + nw * d * d);
                const float rstd = rsqrtf(m2 * inv_n + a.eps);
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[q][e] = (v[q][e] - mean) * rstd * gam[e] + bet[e];
            }
        } else {  // FGE_NORM_RMSNORM
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                float s = 0.0f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) s += okc(e) ? v[q][e] * v[q][e] : 0.0f;
                s0[q] = allreduce_lanes<OpSum, LPR>(s);
                s1[q] = 0.0f;
            }
            if (!whole_row) {
#pragma unroll
                for (int q = 0; q < NPG; ++q) put_stats<FULL>(grow0, q, s0[q], 0.0f);
                return;
            }
            exchange(grow0, s0, s1, 0.0f);
#pragma unroll
            for (int q = 0; q < NPG; ++q) {
                const float rr = rsqrtf(allreduce_lanes<OpSum, LPR>(s0[q]) / (float)a.N + a.eps);
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[q][e] *= rr * gam[e];
            }
        }
    }
    // Deferred whole-row logsumexp: merges the strip pairs that a tile (first row m0_prev) parked
    // in exchange buffer `par`.  To be called by all threads after a workgroup barrier that
    // follows that tile's epilogue; the buffer may be parked into again after the next barrier.
    __device__ __forceinline__ void flush_lse(int tid, int par, int m0_prev) {
        if (tid < tile_rows) {
            const float2 *e = xch + (par * tile_rows + tid) * WAVES_N;
            float m = e[0].x;
#pragma unroll
            for (int w = 1; w < WAVES_N; ++w) m = max_nc(m, e[w].x);
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < WAVES_N; ++w) sum += e[w].y * fast_exp(e[w].x - m);
            if (m0_prev + tid < a.M) a.aux[row_base + m0_prev + tid] = m + __logf(sum);
        }
    }

    // norm_group with the runtime row-op code (and the clamp bound) turned into constants
    // (mkeep: the references the exponentials of a softmax / logsumexp group were taken against)
    template <bool FULL> __device__ __forceinline__ void norm_dispatch(float (&v)[NPG][VEC], int grow0, float (&mkeep)[NPG]) {
        if constexpr (NORM_CT >= 0) {
            if constexpr (NORM_CT != FGE_NORM_NONE) norm_group<NORM_CT, FULL, BOUNDED_CT>(v, grow0, mkeep);
            return;
        }
        switch (a.norm + (bounded ? 8 : 0)) {
        case FGE_NORM_NONE: case FGE_NORM_NONE + 8: break;
        case FGE_NORM_SOFTMAX:       norm_group<FGE_NORM_SOFTMAX, FULL, false>(v, grow0, mkeep); break;
        case FGE_NORM_SOFTMAX + 8:   norm_group<FGE_NORM_SOFTMAX, FULL, true>(v, grow0, mkeep); break;
        case FGE_NORM_LOGSUMEXP:     norm_group<FGE_NORM_LOGSUMEXP, FULL, false>(v, grow0, mkeep); break;
        case FGE_NORM_LOGSUMEXP + 8: norm_group<FGE_NORM_LOGSUMEXP, FULL, true>(v, grow0, mkeep); break;
        case FGE_NORM_LAYERNORM: case FGE_NORM_LAYERNORM + 8: norm_group<FGE_NORM_LAYERNORM, FULL, false>(v, grow0, mkeep); break;
        default:                 norm_group<FGE_NORM_RMSNORM, FULL, false>(v, grow0, mkeep); break;
        }
    }

    // accumulator layout -> LDS patch -> row-wise layout, for block B of a group
    template <int B> __device__ __forceinline__ void transpose_block(floatx16 (&blk)[NB], float (&v)[NPG][VEC]) {
#pragma unroll
        for (int half = 0; half < 32 / PATCH_ROWS; ++half) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (PATCH_ROWS == 32 || (r >> 3) == half) {
                        // (row bit 0 is r & 1, row bit 2 is h: see brow)
                        const int col = XORP ? wsel[(j ^ r) & 1] : j * 32 + wsel[0];
                        patch[(brow(r) - half * PATCH_ROWS) * SSTR + col] = blk[j][r];
                    }
#pragma unroll
            for (int p = 0; p < NPH; ++p)
#pragma unroll
                for (int e = 0; e < VEC; e += 4) {
                    const floatx4 f = *reinterpret_cast<const floatx4 *>(patch + (p * RPP + prow) * SSTR + rsel[e >> 2]);
                    v[B * NPB + half * NPH + p][e] = f[0];
                    v[B * NPB + half * NPH + p][e + 1] = f[1];
                    v[B * NPB + half * NPH + p][e + 2] = f[2];
                    v[B * NPB + half * NPH + p][e + 3] = f[3];
                }
        }
    }
    // activation in place (accumulator layout), then the transpose
    template <int B> __device__ __forceinline__ void to_rows(floatx16 (&blk)[NB], float (&v)[NPG][VEC]) {
        if constexpr (ACT_CT >= 0) act_block<ACT_CT>(blk);
        else dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) { act_block<ACT>(blk); });
        transpose_block<B>(blk, v);
    }

    // 16-byte store of output; with STREAM_OUT, or when the launch asks for it (a.stream_out: an
    // output of half the last-level cache or more), stores carry the streaming (non-temporal) hint.
    __device__ __forceinline__ void put16(OutT *o, const uint4 &u) const {
        if (STREAM_OUT || a.stream_out) {
            const u32x4 w = {u.x, u.y, u.z, u.w};
            __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(o));
        } else {
            *reinterpret_cast<uint4 *>(o) = u;
        }
    }
    template <bool FULL> __device__ __forceinline__ void store_group(float (&v)[NPG][VEC], int grow0) {
#pragma unroll
        for (int q = 0; q < NPG; ++q) {
            const int grow = m0 + qrow(grow0, q);
            if (FULL || grow < a.M) {
                OutT *o = out + (int64_t)grow * a.ldo + gcol;
                if constexpr (sizeof(OutT) == 2) {     // N is a multiple of 8: all or nothing
                    if (FULL || ok4[0]) put16(o, Store<OutT>::pack(v[q]));
                } else {
                    if (FULL || ok4[0]) put16(o, Store<OutT>::pack(v[q]));
                    if (FULL || ok4[1]) put16(o + G4STEP, Store<OutT>::pack(v[q] + 4));
                }
            }
        }
    }

    // ---------------------------------------------------------------- cooperative completion
    // Rows split over column tiles whose workgroups are all in flight.  Per tile:
    //   1. every wave activates its blocks in place and leaves its strip pairs in LDS;
    //   2. one thread per row merges the tile's strips and publishes one pair per (row, tile);
    //   3. the workgroup marks its tile as arrived and waits for the other tiles of the row block;
    //   4. NT / tile_rows threads per row merge the pairs of all tiles into the final row
    //      statistics, which go to LDS;
    //   5. every wave normalises its blocks - still in the accumulators - and stores them.
    // Merging pairs: (m, s): m = max, s = sum s_i exp(m_i - m);  (mean, M2) with counts n_i:
    // mean = sum n_i mean_i / n, M2 = sum M2_i + n_i (mean_i - mean)^2;  (sum of squares, -): sum.

    // step 2: tile row `row` (one thread each)
    __device__ __forceinline__ void merge_strips(int row) {
        float2 e[WAVES_N];
#pragma unroll
        for (int w = 0; w < WAVES_N; ++w) e[w] = xch[row * WAVES_N + w];
        float o0, o1 = 0.0f;
        if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
            o0 = e[0].x;
#pragma unroll
            for (int w = 1; w < WAVES_N; ++w) o0 = max_nc(o0, e[w].x);
#pragma unroll
            for (int w = 0; w < WAVES_N; ++w) o1 += e[w].y * fast_exp(e[w].x - o0);   // empty strips: 0 * exp(-inf)
        } else if (a.norm == FGE_NORM_LAYERNORM) {
            const int nt = max(1, min(WAVES_N * WTN, a.N - n0));
            float sm = 0.0f;
#pragma unroll
            for (int w = 0; w < WAVES_N; ++w) sm += (float)strip_cols(w) * e[w].x;
            o0 = sm / (float)nt;
#pragma unroll
            for (int w = 0; w < WAVES_N; ++w) {
                const float d = e[w].x - o0;
                o1 += e[w].y + (float)strip_cols(w) * d * d;
            }
        } else {
            o0 = 0.0f;
#pragma unroll
            for (int w = 0; w < WAVES_N; ++w) o0 += e[w].x;
        }
        if (m0 + row < a.M) put_pair(a.ws + (row_base + m0 + row) * a.tiles_n + tn, o0, o1);
    }

    // step 3.  Only correct when all tiles of the row block are in flight at once (the caller's
    // persistent grid guarantees it); the wait is bounded all the same.  A wait that runs out
    // raises the fault word and is reported to the whole workgroup (return value false), which
    // then stores NaN for its rows instead of values normalised with incomplete statistics: the
    // kernel still terminates and the result cannot be mistaken for a valid one.
    __device__ __forceinline__ bool arrive_and_wait(int rowblock, int tid) {
        // the pair stores are device-scope atomics: once the store counter has drained they are
        // visible to the whole device, and the barrier orders every wave's drain before the mark
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                        // (also: the strip pairs in xch are consumed)
        unsigned *marks = a.arrive + (int64_t)rowblock * a.tiles_n;
        // (withhold: host-side tests make the waits of a row block run out by keeping back the
        // mark of its first column tile)
        if (tid == 0 && !(a.withhold && tn == 0))
            __hip_atomic_store(marks + tn, a.gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tid < 64) {
            bool ok = true;
            for (int t = tid; t < a.tiles_n; t += 64) {
                unsigned spins = 0;
                while (__hip_atomic_load(marks + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != a.gen) {
                    __builtin_amdgcn_s_sleep(8);
                    if (++spins > a.spin_limit) { ok = false; break; }
                }
            }
            const bool all_ok = __all(ok);
            if (!ok) *a.fault = 1;
            if (tid == 0) xch[0].x = all_ok ? 0.0f : __builtin_nanf("");
        }
        __syncthreads();                                        // pairs are read with device-scope loads
        return xch[0].x == 0.0f;
    }

    // step 4: TPR neighbouring threads per tile row; the result lands in fin[row]:
    // (m, 1/s) softmax, (mean, rstd) LayerNorm, (rstd, -) RMSNorm; logsumexp writes aux.
    template <int TPR> __device__ __forceinline__ void merge_tiles(int tid, float2 *fin, bool waited_ok) {
        const int row = tid / TPR, part = tid % TPR;
        const int grow = m0 + row;
        const float2 *pr = a.ws + (row_base + min(grow, a.M - 1)) * a.tiles_n;
        const int BN_ = WAVES_N * WTN;
        constexpr int CH = 8;                 // pairs fetched together (independent loads in flight)
        float o0, o1 = 0.0f;
        if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
            float m = OpMax::ident(), sum = 0.0f;
            for (int t0 = part; t0 < a.tiles_n; t0 += CH * TPR) {
                float2 e[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    e[i] = t0 + i * TPR < a.tiles_n ? get_pair(pr + t0 + i * TPR) : make_float2(OpMax::ident(), 0.0f);
                float mc = e[0].x;
#pragma unroll
                for (int i = 1; i < CH; ++i) mc = max_nc(mc, e[i].x);
                const float mn = max_nc(m, mc);            // finite: slot t0 exists and every tile has columns
                sum *= fast_exp(m - mn);
#pragma unroll
                for (int i = 0; i < CH; ++i) sum += e[i].y * fast_exp(e[i].x - mn);
                m = mn;
            }
            o0 = allreduce_lanes<OpMax, TPR>(m);
            const float sden = allreduce_lanes<OpSum, TPR>(m == OpMax::ident() ? 0.0f : sum * fast_exp(m - o0));
            if (a.norm == FGE_NORM_SOFTMAX) o1 = fast_rcp(sden);
            else if (part == 0 && tn == 0 && grow < a.M) a.aux[row_base + grow] = waited_ok ? o0 + __logf(sden) : __builtin_nanf("");
        } else if (a.norm == FGE_NORM_LAYERNORM) {
            // two sweeps over the pairs: the mean first, then M2 about it
            const float inv_n = 1.0f / (float)a.N;
            float sm = 0.0f;
            for (int t0 = part; t0 < a.tiles_n; t0 += CH * TPR) {
                float2 e[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    e[i] = t0 + i * TPR < a.tiles_n ? get_pair(pr + t0 + i * TPR) : make_float2(0.0f, 0.0f);
#pragma unroll
                for (int i = 0; i < CH; ++i) sm += (float)max(0, min(BN_, a.N - (t0 + i * TPR) * BN_)) * e[i].x;
            }
            o0 = allreduce_lanes<OpSum, TPR>(sm) * inv_n;
            float m2 = 0.0f;
            for (int t0 = part; t0 < a.tiles_n; t0 += CH * TPR) {
                float2 e[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    e[i] = t0 + i * TPR < a.tiles_n ? get_pair(pr + t0 + i * TPR) : make_float2(o0, 0.0f);
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const float d = e[i].x - o0;
                    m2 += e[i].y + (float)max(0, min(BN_, a.N - (t0 + i * TPR) * BN_)) * d * d;
                }
            }
            o1 = rsqrtf(allreduce_lanes<OpSum, TPR>(m2) * inv_n + a.eps);
        } else {
            float ss = 0.0f;
            for (int t0 = part; t0 < a.tiles_n; t0 += CH * TPR) {
                float2 e[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    e[i] = t0 + i * TPR < a.tiles_n ? get_pair(pr + t0 + i * TPR) : make_float2(0.0f, 0.0f);
#pragma unroll
                for (int i = 0; i < CH; ++i) ss += e[i].x;
            }
            o0 = rsqrtf(allreduce_lanes<OpSum, TPR>(ss) / (float)a.N + a.eps);
        }
        if (!waited_ok) o0 = o1 = __builtin_nanf("");          // statistics incomplete: the rows become NaN
        if (part == 0) fin[row] = make_float2(o0, o1);
    }

    // gamma / beta of this lane's columns (ones / zeros where absent or not used by the row op)
    template <bool FULL> __device__ __forceinline__ void load_affine(float (&gam)[VEC], float (&bet)[VEC]) {
#pragma unroll
        for (int e = 0; e < VEC; e += 4) {
            floatx4 g = {1.0f, 1.0f, 1.0f, 1.0f}, b = {0.0f, 0.0f, 0.0f, 0.0f};
            const int c = gcol + (e >> 2) * G4STEP;
            const bool ok = FULL || ok4[e >> 2];
            if (a.norm != FGE_NORM_SOFTMAX && ok && a.gamma != nullptr) g = *reinterpret_cast<const floatx4 *>(a.gamma + c);
            if (a.norm == FGE_NORM_LAYERNORM && ok && a.beta != nullptr) b = *reinterpret_cast<const floatx4 *>(a.beta + c);
            gam[e] = g[0]; gam[e + 1] = g[1]; gam[e + 2] = g[2]; gam[e + 3] = g[3];
            bet[e] = b[0]; bet[e + 1] = b[1]; bet[e + 2] = b[2]; bet[e + 3] = b[3];
        }
    }

    // step 5 for one group
    template <int NORM>
    __device__ __forceinline__ void finish_group(float (&v)[NPG][VEC], int grow0, const float2 *fin, const float (&mkeep)[NPG],
                                                 const float (&gam)[VEC], const float (&bet)[VEC]) {
#pragma unroll
        for (int q = 0; q < NPG; ++q) {
            const float2 r = fin[qrow(grow0, q)];
            if constexpr (NORM == FGE_NORM_SOFTMAX) {      // v holds exp(a - mkeep)
                const float f = exp_rel(mkeep[q], -r.x * LOG2E) * r.y;
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[q][e] *= f;
            } else if constexpr (NORM == FGE_NORM_LAYERNORM) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[q][e] = (v[q][e] - r.x) * r.y * gam[e] + bet[e];
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[q][e] *= r.x * gam[e];
            }
        }
    }

    // the whole epilogue of a wave's MB blocks; trow0 = tile row of the wave's first row;
    // rowblock / tid / NT (threads of the workgroup) are used by the cooperative form only
    template <int NT>
    __device__ __forceinline__ void tile(floatx16 (&acc)[MB][NB], int trow0, int rowblock, int tid) {
        if constexpr (COOP) {
            // step 1.  The accumulators move to the row-wise layout for good: what step 5 needs -
            // the activated values, for softmax already exp(a - strip maximum) - stays in these
            // registers across the wait, so nothing is transposed or exponentiated twice.
            // (logsumexp leaves the activated values as they are: stored right away)
            float vall[MB / G][NPG][VEC], mkeep[MB / G][NPG];
            static_for<0, MB / G>([&]<int g>() __attribute__((always_inline)) {
                static_for<0, G>([&]<int b>() __attribute__((always_inline)) { to_rows<b>(acc[g * G + b], vall[g]); });
                const int grow0 = trow0 + g * G * 32;
                norm_dispatch<FULL_TILE>(vall[g], grow0, mkeep[g]);
                if (a.norm == FGE_NORM_LOGSUMEXP) store_group<FULL_TILE>(vall[g], grow0);
            });
            // the affine vectors are the same for every group: fetched once, behind the wait
            float gam[VEC], bet[VEC];
            load_affine<FULL_TILE>(gam, bet);
            __syncthreads();
            if (tid < tile_rows) merge_strips(tid);
            const bool waited_ok = arrive_and_wait(rowblock, tid);
            float2 *fin = xch + tile_rows * WAVES_N;
            merge_tiles<NT / (MB * 32 * (NT / 64 / WAVES_N))>(tid, fin, waited_ok);
            if (a.norm == FGE_NORM_LOGSUMEXP) return;
            __syncthreads();
            static_for<0, MB / G>([&]<int g>() __attribute__((always_inline)) {
                const int grow0 = trow0 + g * G * 32;
                switch (a.norm) {
                case FGE_NORM_SOFTMAX:   finish_group<FGE_NORM_SOFTMAX>(vall[g], grow0, fin, mkeep[g], gam, bet); break;
                case FGE_NORM_LAYERNORM: finish_group<FGE_NORM_LAYERNORM>(vall[g], grow0, fin, mkeep[g], gam, bet); break;
                default:                 finish_group<FGE_NORM_RMSNORM>(vall[g], grow0, fin, mkeep[g], gam, bet); break;
                }
                store_group<FULL_TILE>(vall[g], grow0);
            });
        } else {
            auto body = [&]<bool FULL>() __attribute__((always_inline)) {
                static_for<0, MB / G>([&]<int g>() __attribute__((always_inline)) {
                    float v[NPG][VEC], mkeep[NPG];
                    static_for<0, G>([&]<int b>() __attribute__((always_inline)) { to_rows<b>(acc[g * G + b], v); });
                    const int grow0 = trow0 + g * G * 32;
                    norm_dispatch<FULL>(v, grow0, mkeep);
                    // (once per tile: a second wait would sit behind the first group's own stores)
                    if constexpr (WAIT_VM && g == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    store_group<FULL>(v, grow0);
                });
            };
            body.template operator()<FULL_TILE>();
        }
    }
};

}  // namespace fge
