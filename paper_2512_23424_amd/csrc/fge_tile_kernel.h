// The tile kernel: MFMA mainloop with double-buffered LDS panels filled by asynchronous
// global -> LDS copies, accumulators kept in registers through scale + bias + activation and the
// in-tile row statistics, then the store: final when the tile spans N or when the launch is the
// cooperative one (the column tiles of a row block finish their rows together), otherwise a
// parked tile plus per-strip statistics for the light second pass.
//
// One workgroup computes a BM x BN tile of  act(post_scale*(alpha*X.W^T + b)).
// Waves are laid out WAVES_M x WAVES_N; each owns (BM/WAVES_M) x (BN/WAVES_N) outputs as
// 32x32 MFMA blocks.  X rows feed the MFMA A operand and W rows the B operand, so in every
// accumulator register the 32 lanes with equal lane/32 hold 32 neighbouring columns of one
// output row.
//
// LDS panel layout (both operands): row-major, 128 bytes of K per row (128 E4M3 / 64 16-bit /
// 32 fp32 values; with the split product the bf16 high and low parts of 32 values in
// alternating chunks),
// the eight 16-byte chunks of a row stored at chunk ^ ((row >> 1) & 7): the 16-byte fragment
// reads of 16 neighbouring rows then touch each of the 64 LDS banks exactly once (measured:
// zero bank-conflict cycles; the 8-row variant chunk ^ (row & 7) conflicts two-way).
// Full K tiles are copied global -> LDS directly (no staging registers): a wave's load
// instruction fills 1024 contiguous LDS bytes, lane l at base + 16*l, so each lane fetches
// the global chunk that belongs at its LDS position.  The split product of fp32 operands stages
// through registers instead, since the operands are split into bf16 parts on the way in.
#pragma once
#include "fge_epilogue.h"

namespace fge {

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

// XOR pattern of the panel swizzle for a panel row.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// 8 fp32 values (two 16-byte chunks) -> their bf16 high parts and the bf16 roundings of the
// remainders, packed two per word in the order the bf16 matrix instruction takes them.
__device__ __forceinline__ void split_bf16x8(const u32x4 &c0, const u32x4 &c1, u32x4 &hi, u32x4 &lo) {
    const float f[8] = {as_f32(c0.x), as_f32(c0.y), as_f32(c0.z), as_f32(c0.w),
                        as_f32(c1.x), as_f32(c1.y), as_f32(c1.z), as_f32(c1.w)};
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t hh = f32x2_to_bf16x2(f[2 * p], f[2 * p + 1]);
        const float r0 = f[2 * p] - as_f32(hh << 16), r1 = f[2 * p + 1] - as_f32(hh & 0xFFFF0000u);
        hi[p] = hh;
        lo[p] = f32x2_to_bf16x2(r0, r1);
    }
}

template <typename InT> struct Mma;
template <> struct Mma<bf16_t> {
    __device__ static __forceinline__ void run(const u32x4 &a, const u32x4 &b, floatx16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                    __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<f16_t> {
    __device__ static __forceinline__ void run(const u32x4 &a, const u32x4 &b, floatx16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                   __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<f8_t> {
    // One instruction takes 64 k: 32 bytes per lane and operand, here two 16-byte chunks of the
    // lane's panel row.  Which k sits in which lane half and byte is the same for both
    // operands, so the sum over k is complete.  (Block scales switched off: both scale
    // operands zero select the unscaled instruction.)
    __device__ static __forceinline__ void run(const u32x4 (&a)[2], const u32x4 (&b)[2], floatx16 &c) {
        const i32x8 av = {(int)a[0].x, (int)a[0].y, (int)a[0].z, (int)a[0].w, (int)a[1].x, (int)a[1].y, (int)a[1].z, (int)a[1].w};
        const i32x8 bv = {(int)b[0].x, (int)b[0].y, (int)b[0].z, (int)b[0].w, (int)b[1].x, (int)b[1].y, (int)b[1].z, (int)b[1].w};
        c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 0, 0, 0, 0, 0, 0);
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

// FULL: M and N are multiples of BM and BN - the epilogue then runs without row or column guards.
// Tiles of up to 64x128 are meant to run two workgroups per CU (second launch bound: waves per
// SIMD), which caps their registers at 256.
// SPLIT (fp32 operands only): the product runs on the bf16 matrix instruction with every fp32
// operand split in two bf16 terms, x = xh + xl (bf16 rounding of the value and of the rest):
//     x*w ~= xl*wh + xh*wl + xh*wh        (fp32 accumulate, the xl*wl term is dropped)
// Relative error per product <= about 2^-16.5, against 2^-24 of the fp32 instruction, at less
// than a fifth of its matrix-pipe time (3 x 8 passes per 16 k instead of 8 x 16 passes).  The
// split product has a mainloop of its own (operands are split on their way into LDS).
// STAGES: 0 for the tile's usual number of stage buffers, else that many (see DEEP below).
template <typename InT, typename OutT, int BM, int BN, int WAVES_M, int WAVES_N, bool COOP = false, bool FULL = false,
          bool SPLIT = false, bool GATED = false, int STAGES = 0>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, (BM * BN <= 64 * 128 ? 2 : 1))
void tile_kernel(const TileArgs a) {
    static_assert(!SPLIT || sizeof(InT) == 4, "only fp32 operands are split");
    // GATED: the tile is act(X.W1^T + b1) * (X.W2^T + b2) over BN/2 output columns.  The B panel
    // holds the BN/2 rows of W1 and, below them, the same rows of W2; each wave's column blocks
    // are 32 columns of the first product and the same 32 columns of the second, so the gate is
    // applied register by register before the shared epilogue sees a tile of BN/2 columns.
    static_assert(!GATED || (sizeof(InT) <= 2 && BN / WAVES_N == 64 && !SPLIT), "gated form: two 32-column blocks per wave");
    constexpr int BNO = GATED ? BN / 2 : BN;         // output columns per tile
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int MB = WTM / 32, NB = WTN / 32;
    constexpr int ROWB = 128;                        // bytes of K per LDS row
    constexpr int BK = ROWB / (int)sizeof(InT);      // 128 fp8 / 64 bf16 / 32 fp32
    constexpr int CW = 16 / (int)sizeof(InT);        // elements per 16-byte chunk
    constexpr int A_LD = BM * 8 / NT, B_LD = BN * 8 / NT;
    constexpr bool F8 = sizeof(InT) == 1;            // 64 k per matrix instruction
    constexpr int FR = F8 ? 2 : 1;                   // 16-byte chunks per fragment per k-step
    constexpr int KS = 4 / FR;                       // k-steps per staged tile (the split product has its own loop)
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "load plan");
    constexpr int STAGE = (BM + BN) * ROWB;
    // DEEP: a K tile of a small tile is multiplied in a fraction of the time its copy takes to
    // arrive, so one tile of lookahead leaves the loop waiting on memory latency.  The 64x64 tile
    // always runs with four stage buffers (three copies in flight, two workgroups per CU); the
    // 128x128 tile has a variant with three (STAGES = 3, one workgroup per CU) for launches that
    // give a CU no second workgroup to hide the latency with.
    static_assert(STAGES == 0 || (STAGES > 2 && !SPLIT && !GATED), "extra stage buffers: plain 16- and 8-bit tiles");
    constexpr bool DEEP = STAGES > 2 || (BM == 64 && BN == 64 && !SPLIT && !COOP);
    constexpr int NST = STAGES > 2 ? STAGES : DEEP ? 4 : 2;

    __shared__ __attribute__((aligned(16))) unsigned char smem[NST * STAGE];
    __shared__ __attribute__((aligned(16))) float2 xch[2 * BM * WAVES_N];

    // One pass for an ordinary launch.  A cooperative launch is persistent: every round the
    // grid takes the next gridDim.x / tiles_n row blocks (gridDim.x is a multiple of tiles_n), so
    // the column tiles of a row block are always in flight together.  Inside a round, position s
    // (contiguous per XCD) walks the round's tiles in panels of PW column tiles, row block by row
    // block, so that the tiles of an XCD form a patch about as tall as wide: what its L2 has to
    // fetch per k-step is then close to the minimum for that many tiles.
    for (int round = 0;; ++round) {
    // In the persistent form the thread index is made opaque once per round: everything derived
    // from it (staging plan, fragment offsets, epilogue coordinates) is then recomputed per tile
    // instead of being kept in registers across the epilogue, where registers are scarce.
    int tid = threadIdx.x;
    if constexpr (COOP) asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int h = lane >> 5, l32 = lane & 31;
    int tm, tn, z, rowblock;
    if constexpr (COOP) {
        constexpr int PW = 4;
        const int G = gridDim.x, q = G >> 3, rem = G & 7;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int s = xcd * q + (xcd < rem ? xcd : rem) + slot;
        const int rpr = G / a.tiles_n;                                   // row blocks per round
        const int R = min(rpr, a.tiles_m * a.batch - round * rpr);       // ... in this round
        if (R <= 0 || s >= R * a.tiles_n) break;
        const int full = a.tiles_n / PW, panel = s / (R * PW);
        int rb;
        if (panel < full) {
            const int w = s - panel * R * PW;
            rb = w / PW;
            tn = panel * PW + w % PW;
        } else {                                                         // the narrower last panel
            const int wd = a.tiles_n - full * PW, w = s - full * R * PW;
            rb = w / wd;
            tn = full * PW + w % wd;
        }
        rowblock = round * rpr + rb;
        z = rowblock / a.tiles_m;
        tm = rowblock - z * a.tiles_m;
        // Staggered start: the row blocks of the first round begin a little apart (all column
        // tiles of a row block together - they wait for each other).  Equal tiles keep the whole
        // chip in lockstep otherwise, and every round would end in one burst of stores at the
        // memory system's write ceiling, behind which the next round's first loads queue up.
        if (round == 0 && a.stagger > 0) {
            for (int i = (rb & a.stagger_mask) * a.stagger; i > 0; --i) __builtin_amdgcn_s_sleep(16);     // 1024 clocks each
        }
    } else {
        if (round > 0) break;
        tile_coords(blockIdx.x, a.tiles_m, a.tiles_n, a.group_m, tm, tn);
        z = blockIdx.z;
        rowblock = z * a.tiles_m + tm;
    }
    const int m0 = tm * BM, n0 = tn * BNO;

    const InT *X = reinterpret_cast<const InT *>(a.X) + (int64_t)z * a.bsx;
    const InT *W = reinterpret_cast<const InT *>(a.W) + (int64_t)z * a.bsw;
    OutT *out = reinterpret_cast<OutT *>(a.out) + (int64_t)z * a.bso;

    // ---------------- global -> LDS staging plan
    // A copy instruction of a wave fills 1024 contiguous LDS bytes = 8 panel rows (lane l lands at
    // base + 16*l).  Wave w stages the 8*A_LD rows of the A panel from row w*8*A_LD on and the
    // 8*B_LD rows of the B panel from row w*8*B_LD on, copy i the rows 8i .. 8i+7 of those: the
    // copies of an operand land 1024 bytes apart, which the instruction's own 12-bit offset
    // reaches - it moves the LDS address and the global address alike, so the lane offset of copy
    // i is lowered by the same amount -, and one write of the LDS base register serves four
    // copies.  Rows past the end of X / W are clamped to the last valid row: they only feed
    // outputs that are never stored or counted.  Only a partial last K tile needs zero fill; it
    // goes through registers.
    // The lane at (row, physical chunk c) of the panel fetches global chunk c ^ swizzle(row): the
    // LDS image of a wave's 64 chunks is then the 1024 contiguous bytes a copy writes.
    const int ld_r = (tid & 63) >> 3, ld_c = tid & 7;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int PRE = 3072;                         // bytes the scalar bases start early (keeps lane offsets >= 0)
    static_assert(!GATED || BNO % (8 * B_LD) == 0, "a wave's B rows come from one matrix");
    // gated: the waves whose B rows lie at or beyond BNO stage the same rows of W2
    const bool second = GATED && wave_id * 8 * B_LD >= BNO;
    const unsigned char *Xt = reinterpret_cast<const unsigned char *>(X + (int64_t)m0 * a.ldx) - PRE;
    const unsigned char *Wt = reinterpret_cast<const unsigned char *>(
                                  (second ? reinterpret_cast<const InT *>(a.W2) + (int64_t)z * a.bsw : W) + (int64_t)n0 * a.ldw) - PRE;
    // A copy's global address is a scalar base (first row of the tile, current k) plus the lane's
    // byte offset from it, which does not change along K: 32 bits (the host keeps tiles whose
    // rows span 2 GB or more off this kernel).
    uint32_t oA[A_LD], oB[B_LD];
    int rowA[A_LD], rowB[B_LD], gcA[A_LD], gcB[B_LD];  // panel row and global chunk of this lane per copy
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        rowA[i] = wave_id * 8 * A_LD + i * 8 + ld_r;
        gcA[i] = ld_c ^ swz(rowA[i]);
        oA[i] = (uint32_t)((int64_t)(min(m0 + rowA[i], a.M - 1) - m0) * a.ldx + gcA[i] * CW) * (uint32_t)sizeof(InT) + PRE - (i & 3) * 1024;
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        rowB[i] = wave_id * 8 * B_LD + i * 8 + ld_r;
        gcB[i] = ld_c ^ swz(rowB[i]);
        const int prow = rowB[i] - (second ? BNO : 0);   // row of W (gated: or of W2) in the tile
        oB[i] = (uint32_t)((int64_t)(min(n0 + prow, a.w_rows - 1) - n0) * a.ldw + gcB[i] * CW) * (uint32_t)sizeof(InT) + PRE - (i & 3) * 1024;
    }

    // full tile: asynchronous global -> LDS, no registers involved; completion is tracked by
    // the vector-memory counter (wait for it, then barrier, before anyone reads the tile)
    const uint32_t lds_waveA = lds_address(smem) + (uint32_t)(wave_id * A_LD * 1024);
    const uint32_t lds_waveB = lds_address(smem) + (uint32_t)(BM * ROWB + wave_id * B_LD * 1024);
    constexpr int NS = A_LD + B_LD;                  // copy instructions per thread per tile
    static_assert(NS % 2 == 0, "copies are issued in two halves");
    // copy w of the tile at k0 into stage `buf`; `first`: the first copy of a run of copies (the
    // LDS base register is written then and whenever a copy starts another group of four)
    auto dma_chunk = [&](int buf, int k0, int w, bool first) __attribute__((always_inline)) {
        const int i = w < A_LD ? w : w - A_LD;
        const bool set_base = first || (i & 3) == 0 || w == A_LD;
        if (w < A_LD) lds_dma16(Xt + (int64_t)k0 * sizeof(InT), oA[i], lds_waveA + buf * STAGE + (i >> 2) * 4096, i & 3, set_base);
        else          lds_dma16(Wt + (int64_t)k0 * sizeof(InT), oB[i], lds_waveB + buf * STAGE + (i >> 2) * 4096, i & 3, set_base);
    };
    auto dma_tile = [&](int buf, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int w = 0; w < NS; ++w) dma_chunk(buf, k0, w, w == 0);
    };
    // partial last tile: through registers, zero filled past K
    auto stage_tail = [&](int buf, int k0) __attribute__((always_inline)) {
        unsigned char *sA = smem + buf * STAGE + (ld_c << 4), *sB = sA + BM * ROWB;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            u32x4 v = {0u, 0u, 0u, 0u};             // (K is a multiple of CW: chunks are whole)
            if (k0 + gcA[i] * CW < a.K) v = *reinterpret_cast<const u32x4 *>(Xt + (int64_t)k0 * sizeof(InT) + oA[i] + (i & 3) * 1024);
            *reinterpret_cast<u32x4 *>(sA + rowA[i] * ROWB) = v;
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (k0 + gcB[i] * CW < a.K) v = *reinterpret_cast<const u32x4 *>(Wt + (int64_t)k0 * sizeof(InT) + oB[i] + (i & 3) * 1024);
            *reinterpret_cast<u32x4 *>(sB + rowB[i] * ROWB) = v;
        }
    };

    // ---------------- fragment read plan
    // B fragment of column block j sits FB_STEP panel rows below block 0's (gated: the second
    // product's rows start BNO rows down)
    constexpr int FB_STEP = GATED ? BNO : 32;
    const int fa_row = wave_m * WTM + l32, fb_row = wave_n * (GATED ? 32 : WTN) + l32;
    // chunk pair u (0..3) of a panel row: lanes 0-31 take chunk 2u, lanes 32-63 chunk 2u+1.
    // A k-step consumes FR pairs.  Which k land in which lane and slot does not matter as long
    // as both operands use the same assignment - the sum over k is complete either way.
    int fsw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) fsw[u] = ((2 * u + h) ^ swz(l32)) << 4;

    floatx16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    if constexpr (SPLIT) {
    // ---------------- mainloop, split product
    // Every operand value feeds WAVES_N (X) or WAVES_M (W) waves, so the split into bf16 parts is
    // done once per workgroup on the way into LDS instead of once per wave on the way out: thread
    // (row, kg) = (tid / 4, tid % 4) fetches the 8 values k = 8kg .. 8kg+7 of its panel rows into
    // registers while the previous K tile is multiplied, splits them and parks the high and the
    // low parts as 16-byte chunks 2kg and 2kg+1 of the 128-byte panel row (same swizzle as the
    // other kernels' panels).  One barrier per K tile; values past K are zero.
    constexpr int A_IT = BM * 4 / NT, B_IT = BN * 4 / NT, NI = A_IT + B_IT;
    static_assert((BM * 4) % NT == 0 && (BN * 4) % NT == 0 && (NT / 4) % 16 == 0, "split staging plan");
    const int it_row = tid >> 2, it_kg = tid & 3;
    const float *gS[NI];
#pragma unroll
    for (int i = 0; i < A_IT; ++i)
        gS[i] = X + (int64_t)min(m0 + it_row + i * (NT / 4), a.M - 1) * a.ldx + it_kg * 8;
#pragma unroll
    for (int i = 0; i < B_IT; ++i)
        gS[A_IT + i] = W + (int64_t)min(n0 + it_row + i * (NT / 4), a.w_rows - 1) * a.ldw + it_kg * 8;
    u32x4 sreg[NI][2];
    // GUARD: the tile may reach past K (K is a multiple of 4: chunks are whole)
    auto stage_load = [&]<bool GUARD>(int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bool kok = !GUARD || k0 + it_kg * 8 + 4 * c < a.K;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                if constexpr (GUARD) sreg[i][c] = u32x4{0u, 0u, 0u, 0u};
                if (kok) sreg[i][c] = *reinterpret_cast<const u32x4 *>(gS[i] + k0 + 4 * c);
            }
        }
    };
    const int st_off = it_row * ROWB, st_hi = ((2 * it_kg) ^ swz(it_row)) << 4, st_lo = ((2 * it_kg + 1) ^ swz(it_row)) << 4;
    auto stage_store = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            u32x4 hi, lo;
            split_bf16x8(sreg[i][0], sreg[i][1], hi, lo);
            unsigned char *row = smem + buf * STAGE + st_off +
                                 (i < A_IT ? i * (NT / 4) : BM + (i - A_IT) * (NT / 4)) * ROWB;
            *reinterpret_cast<u32x4 *>(row + st_hi) = hi;
            *reinterpret_cast<u32x4 *>(row + st_lo) = lo;
        }
    };
    // fragment (k-step t of the tile's two): lanes 0-31 take k-group 2t, lanes 32-63 k-group 2t+1
    int fq[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int c = 0; c < 2; ++c) fq[t][c] = ((2 * (2 * t + h) + c) ^ swz(l32)) << 4;
    constexpr int NM = MB * NB, NR = MB + NB;
    u32x4 fh[2][NR], fl[2][NR];                       // [register set][A fragments, then B fragments]
    auto read_split = [&](int buf, int t) __attribute__((always_inline)) {
        const unsigned char *sA = smem + buf * STAGE + fa_row * ROWB;
        const unsigned char *sB = smem + buf * STAGE + BM * ROWB + fb_row * ROWB;
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            const unsigned char *r = q < MB ? sA + q * 32 * ROWB : sB + (q - MB) * 32 * ROWB;
            fh[t & 1][q] = *reinterpret_cast<const u32x4 *>(r + fq[t][0]);
            fl[t & 1][q] = *reinterpret_cast<const u32x4 *>(r + fq[t][1]);
        }
    };
    // One K tile: both k-steps' fragments, the MFMAs of k-step 0, then - STORE - the split and
    // parking of the next tile spread between the MFMAs of k-step 1 (a wave issues in order; left
    // in one piece, the vector-ALU work of the split would run after the last MFMA instead of
    // under them).
    constexpr int ST_VALU = 26 * NI;                  // vector-ALU instructions of one stage_store, about
    auto compute = [&]<bool STORE>(int buf) __attribute__((always_inline)) {
        read_split(buf, 0);
        read_split(buf, 1);
        static_for<0, 2>([&]<int t>() __attribute__((always_inline)) {
            if constexpr (t == 1) {
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (STORE) stage_store(buf ^ 1);
            }
#pragma unroll
            for (int m = 0; m < NM; ++m) {            // small terms first
                floatx16 &c = acc[m / NB][m % NB];
                Mma<bf16_t>::run(fl[t][m / NB], fh[t][MB + m % NB], c);
                Mma<bf16_t>::run(fh[t][m / NB], fl[t][MB + m % NB], c);
                Mma<bf16_t>::run(fh[t][m / NB], fh[t][MB + m % NB], c);
            }
            if constexpr (t == 1 && STORE) {
#pragma unroll
                for (int g = 0; g < 3 * NM; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                              // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, (ST_VALU + 3 * NM - 1) / (3 * NM), 0);   // its share of the split
                }
                __builtin_amdgcn_sched_group_barrier(0x200, 2 * NI, 0);                             // the parked chunks
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    // At the top of iteration kt the staging registers hold tile kt+1 (fetched during iteration
    // kt-1, so a whole iteration hides the latency); it is parked during iteration kt, and tile
    // kt+2 is fetched into the same registers right behind.
    const int KT = (a.K + BK - 1) / BK, KF = a.K / BK;    // tiles; tiles that lie inside K
    stage_load.template operator()<true>(0);
    stage_store(0);
    if (KT > 1) stage_load.template operator()<true>(BK);
    __syncthreads();
    int kt = 0;
    for (; kt + 2 < KF; ++kt) {                       // tile kt+2 lies inside K
        compute.template operator()<true>(kt & 1);
        stage_load.template operator()<false>((kt + 2) * BK);
        __syncthreads();                              // tile kt+1 is parked; reads of tile kt are over
    }
    for (; kt + 2 < KT; ++kt) {                       // tile kt+2 is the partial one
        compute.template operator()<true>(kt & 1);
        stage_load.template operator()<true>((kt + 2) * BK);
        __syncthreads();
    }
    for (; kt + 1 < KT; ++kt) {                       // nothing left to fetch
        compute.template operator()<true>(kt & 1);
        __syncthreads();
    }
    compute.template operator()<false>(kt & 1);
    __syncthreads();                                  // the epilogue reuses the panel memory
    } else {
    // ---------------- mainloop
    // Per staged tile: KS k-steps of NM MFMAs.  Fragments of the next k-step are read from LDS
    // behind the first MFMAs of the current one (two register sets).  The single barrier of an
    // iteration sits before the last k-step, and that k-step already prefetches the next tile's
    // first fragments, so no LDS or barrier latency is exposed.  sched_barrier pins this order:
    // left alone, the compiler sinks every fragment read next to its first use.
    constexpr int NM = MB * NB, NR = MB + NB;
    u32x4 fr[2][NR][FR];                              // [0,MB): A fragments, [MB,NR): B fragments
    // 8-bit operands: fragments are twice as large (64 k per instruction), so the A fragments
    // get one register set only - block i's next fragment is fetched right behind the last
    // MFMA of the current k-step that uses it, and is needed again NM - NB MFMAs later.
    u32x4 fa1[F8 ? MB : 1][FR];
    auto read_frag = [&](int buf, int t, int q) __attribute__((always_inline)) {
        const unsigned char *sA = smem + buf * STAGE + fa_row * ROWB;
        const unsigned char *sB = smem + buf * STAGE + BM * ROWB + fb_row * ROWB;
#pragma unroll
        for (int c = 0; c < FR; ++c) {
            const int off = fsw[(t & (KS - 1)) * FR + c];
            if (q < MB) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(sA + q * 32 * ROWB + off);
                if constexpr (F8) fa1[q][c] = v;
                else              fr[t & 1][q][c] = v;
            } else {
                fr[t & 1][q][c] = *reinterpret_cast<const u32x4 *>(sB + (q - MB) * FB_STEP * ROWB + off);
            }
        }
    };
    // prefetch order = order of first use: A0, B0..B(NB-1), A1..A(MB-1)
    auto slot = [&](int s) __attribute__((always_inline)) { return s == 0 ? 0 : (s <= NB ? MB + s - 1 : s - NB); };
    constexpr int RSPAN = NR < NM ? NR : NM;          // reads ride behind the first RSPAN MFMAs
    // one k-step: MFMAs of step t on fragment set t&1; behind MFMA m: reads of (rbuf, t+1)
    // dma_part: 0 none, 1 / 2: first / second half of the copy instructions of the tile at
    // (dbuf, dk0), one behind each of the first MFMAs - a burst of copies would stall the
    // wave's in-order issue, and with it its MFMAs, on the address unit; 3: all of them, spread
    // evenly over the MFMAs of the k-step
    auto kstep = [&]<int DMA_PART>(int t, bool do_read, int rbuf, bool do_dma, int dbuf, int dk0) __attribute__((always_inline)) {
        constexpr int HALF = NS / 2;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            if constexpr (F8) {
                Mma<InT>::run(fa1[m / NB], fr[t & 1][MB + m % NB], acc[m / NB][m % NB]);
            } else {
                Mma<InT>::run(fr[t & 1][m / NB][0], fr[t & 1][MB + m % NB][0], acc[m / NB][m % NB]);
            }
            if constexpr (F8) {
                if (do_read) {
                    if (m < NB) read_frag(rbuf, t + 1, MB + m);                  // B: into the other set
                    if (m % NB == NB - 1) read_frag(rbuf, t + 1, m / NB);        // A: behind its last use
                }
            } else if (do_read) {
#pragma unroll
                for (int s = (m * NR) / RSPAN; s < ((m + 1) * NR) / RSPAN && s < NR; ++s) read_frag(rbuf, t + 1, slot(s));
            }
            if constexpr (DMA_PART == 3) {
#pragma unroll
                for (int w = (m * NS) / NM; w < ((m + 1) * NS) / NM; ++w)
                    if (do_dma) dma_chunk(dbuf, dk0, w, w == 0);
            } else if constexpr (DMA_PART != 0) {
#pragma unroll
                for (int w = (m * HALF) / NM; w < ((m + 1) * HALF) / NM; ++w)
                    if (do_dma) dma_chunk(dbuf, dk0, (DMA_PART - 1) * HALF + w, w == 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto read_t0 = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NR; ++s) read_frag(buf, 0, slot(s));
        __builtin_amdgcn_sched_barrier(0);
    };
    auto compute_last = [&](int buf) __attribute__((always_inline)) {   // fr[0] holds k-step 0
        static_for<0, KS>([&]<int t>() __attribute__((always_inline)) {
            kstep.template operator()<0>(t, t + 1 < KS, buf, false, 0, 0);
        });
    };
    const int KF = a.K / BK;                          // full K tiles
    const bool ragged_k = (a.K % BK) != 0;            // plus one partial tile
    if constexpr (DEEP) {
        // Tile kt lives in buffer kt % NST; the copies of tiles kt+1 .. kt+NST-1 are in flight
        // while tile kt is multiplied.  Copies complete in issue order, so "tile kt has landed"
        // is a wait until only the copies of the later tiles (NS instructions each) are out.
        // One barrier per tile: behind it tile kt is visible to every wave and every wave is
        // done with tile kt-1, whose buffer the copy of tile kt+NST-1 may then overwrite.
        static_assert(NST <= 4 && (NST - 1) * NS <= 32, "copy counter");
#pragma unroll
        for (int d = 0; d < NST - 1; ++d)
            if (d < KF) dma_tile(d, d * BK);
        for (int kt = 0; kt < KF; ++kt) {
            const int later = KF - 1 - kt;            // tiles issued after kt (capped by the depth)
            if (later >= NST - 2)             asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * NS) : "memory");
            else if (NST > 3 && later == 1)   asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS) : "memory");
            else                              lds_dma_wait();
            __syncthreads();
            if (kt + NST - 1 < KF) dma_tile((kt + NST - 1) % NST, (kt + NST - 1) * BK);
            __builtin_amdgcn_sched_barrier(0);
            read_t0(kt % NST);
            compute_last(kt % NST);
        }
        if (ragged_k) {                               // the partial tile, through registers
            stage_tail(KF % NST, KF * BK);
            __syncthreads();
            read_t0(KF % NST);
            compute_last(KF % NST);
        }
        __syncthreads();
    } else {
    // Tile kt lives in buffer kt & 1.  Its copy is issued in two halves - behind the MFMAs of
    // the last k-step of tile kt-2 (right after the barrier that ends the reads of that buffer)
    // and of k-step 0 of tile kt-1 - and is awaited just before the barrier of tile kt-1.
    if (KF > 0) { dma_tile(0, 0); lds_dma_wait(); }
    else        stage_tail(0, 0);
    __syncthreads();
    // 8-bit operands have two k-steps per tile only: the whole copy of tile kt+1 is issued behind
    // the last k-step of tile kt-1 (measured 4 % faster).  With the four k-steps of 16-bit operands
    // the copy stays in two halves: all at once measured 3 % slower there.
    constexpr bool EARLY = F8;
    if (KF > 1) {
#pragma unroll
        for (int w = 0; w < (EARLY ? NS : NS / 2); ++w) dma_chunk(1, BK, w, w == 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    read_t0(0);
    int kt = 0;
    for (; kt + 1 < KF; ++kt) {                       // tile kt+1 is a full one
        const int buf = kt & 1;
        if constexpr (EARLY) kstep.template operator()<0>(0, true, buf, false, 0, 0);
        else                 kstep.template operator()<2>(0, true, buf, true, buf ^ 1, (kt + 1) * BK);
        static_for<1, KS - 1>([&]<int t>() __attribute__((always_inline)) {
            kstep.template operator()<0>(t, true, buf, false, 0, 0);
        });
        lds_dma_wait();                                   // tile kt+1 has landed in buf^1
        __syncthreads();                              // ... for every wave; reads of buf are over
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (EARLY) kstep.template operator()<3>(KS - 1, true, buf ^ 1, kt + 2 < KF, buf, (kt + 2) * BK);
        else                 kstep.template operator()<1>(KS - 1, true, buf ^ 1, kt + 2 < KF, buf, (kt + 2) * BK);   // then k-step 0
    }
    if (KF > 0 && ragged_k) {                         // last full tile, then the partial tile
        compute_last(kt & 1);
        stage_tail((kt & 1) ^ 1, KF * BK);
        __syncthreads();
        ++kt;
        read_t0(kt & 1);
    }
    compute_last(kt & 1);
    if constexpr (WAVES_M * WAVES_N > 1) __syncthreads();
    }
    }

    // ---------------- epilogue.  The store patches live in the panel memory, free once the
    // mainloop's last fragment reads are behind the barrier above.  The 64-row tiles are the
    // ones chosen to span N; they take the joint form (one exchange per tile).
    constexpr bool JOINT = BM == 64;
    if constexpr (GATED) {
        // gate in the accumulator layout; the epilogue then takes finished values (no scale, bias
        // or activation of its own) of a tile that is one 32-column block per wave wide
        const int col = n0 + wave_n * 32 + l32;
        const float scale = a.post * a.alpha;
        const float bias1 = (a.b != nullptr && col < a.N) ? a.post * a.b[col] : 0.0f;
        const float bias2 = (a.b2 != nullptr && col < a.N) ? a.post * a.b2[col] : 0.0f;
        floatx16 gated[MB][1];
        dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    gated[i][0][r] = activate<ACT>(scale * acc[i][0][r] + bias1, a.lo, a.hi) * (scale * acc[i][1][r] + bias2);
        });
        TileArgs ag = a;
        ag.act = FGE_ACT_NONE; ag.alpha = 1.0f; ag.post = 1.0f; ag.b = nullptr;
        using Epi = TileEpilogue<OutT, MB, 1, WAVES_N, 32, false, false, COOP, false>;
        static_assert(WAVES_M * WAVES_N * Epi::PATCH_FLOATS * 4 <= 2 * STAGE, "store patches fit the panels");
        Epi epi(ag, out, xch, reinterpret_cast<float *>(smem) + wave * Epi::PATCH_FLOATS, BM, z, m0, n0, tn,
                wave_n, lane);
        epi.template tile<NT>(gated, wave_m * WTM, rowblock, tid);
    } else {
        using Epi = TileEpilogue<OutT, MB, NB, WAVES_N, 32, JOINT, false, COOP, FULL>;
        static_assert(WAVES_M * WAVES_N * Epi::PATCH_FLOATS * 4 <= 2 * STAGE, "store patches fit the panels");
        Epi epi(a, out, xch, reinterpret_cast<float *>(smem) + wave * Epi::PATCH_FLOATS, BM, z, m0, n0, tn,
                wave_n, lane);
        epi.template tile<NT>(acc, wave_m * WTM, rowblock, tid);
    }
    if constexpr (COOP) __syncthreads();             // patches are panel memory of the next tile
    }
}

}  // namespace fge
