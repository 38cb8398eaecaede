// Row-wise and elementwise kernels: the unfused K2 (activation) and K3 (row operation), and
// the light second pass of the fused path that merges per-strip row statistics.
// One 64-lane wavefront owns one row; data moves in 16-byte chunks per lane.
#pragma once
#include <type_traits>

#include "fge_device.h"

namespace fge {

struct RowArgs {
    const void *in;             // rows x N, element type T, same strides as out
    const void *in2;            // act only: optional second operand, out = act(in) * in2
    void *out;
    const float *gamma, *beta;
    float *aux;
    const float2 *ws;           // finish only: [batch*M][tiles_n] strip pairs
    int M, N, batch;
    int64_t ldo, bso;
    float lo, hi, eps;
    int act, norm;
    int tiles_n, bn;            // finish only: column strips per row and their width
    // row op over a K-split product (rownorm_kernel<float, CH, OutT, true>): `in` holds `slices`
    // dense fp32 M x N partial products, `slice_stride` elements apart; the row is
    // act(scale * sum of the slices + post * b) before the row operation
    const float *b;
    float scale, post;
    int slices;
    int64_t slice_stride;
};

// K2: A = act(Y) (times a second operand in the gated sequence), elementwise, 16 bytes per lane
// per step.
template <typename T>
__global__ __launch_bounds__(256) void act_kernel(const RowArgs a) {
    constexpr int CW = Store<T>::CW;
    const int cpr = a.N / CW;
    const int64_t total = (int64_t)a.batch * a.M * cpr;
    const T *in = reinterpret_cast<const T *>(a.in);
    T *out = reinterpret_cast<T *>(a.out);
    dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
        for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total;
             idx += (int64_t)gridDim.x * 256) {
            const int64_t rowg = idx / cpr;
            const int c = (int)(idx - rowg * cpr);
            const int64_t off = (rowg / a.M) * a.bso + (rowg % a.M) * a.ldo + (int64_t)c * CW;
            float v[CW];
            Store<T>::unpack(*reinterpret_cast<const uint4 *>(in + off), v);
#pragma unroll
            for (int e = 0; e < CW; ++e) v[e] = activate<ACT>(v[e], a.lo, a.hi);
            if (a.in2 != nullptr) {                                   // gate
                float u[CW];
                Store<T>::unpack(*reinterpret_cast<const uint4 *>(reinterpret_cast<const T *>(a.in2) + off), u);
#pragma unroll
                for (int e = 0; e < CW; ++e) v[e] *= u[e];
            }
            *reinterpret_cast<uint4 *>(out + off) = Store<T>::pack(v);
        }
    });
}

// K3: out = rowop(A).  The row lives in registers as loaded - lane l holds the 16-byte chunks l,
// l+64, ... (CH of them) - and is unpacked to fp32 pass by pass, so a 16-bit row costs half the
// registers of its fp32 image (a row of 8192 bf16 values: 64 registers per lane instead of 128,
// which is the difference between two and four rows in flight per SIMD).  The price: a 16-bit
// softmax forms its exponentials twice (for the sum and for the result); an fp32 row keeps
// them in place.
// SLICES (T = float): the row is first formed from the partial products of a K-split GEMM - the
// slices are added in slice order, then scale, bias and activation - and the result is stored
// as OutT; everything else is the same kernel.
template <typename T, int CH, typename OutT = T, bool SLICES = false>
__global__ __launch_bounds__(256) void rownorm_kernel(const RowArgs a) {
    static_assert(SLICES ? std::is_same_v<T, float> : std::is_same_v<T, OutT>, "slices are fp32; otherwise in and out share a type");
    constexpr int CW = Store<T>::CW;
    constexpr bool PACKED = sizeof(T) == 2;
    const int lane = threadIdx.x & 63;
    const int64_t rowg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rowg >= (int64_t)a.batch * a.M) return;           // wave-uniform
    const int64_t off = (rowg / a.M) * a.bso + (rowg % a.M) * a.ldo;
    const T *in = reinterpret_cast<const T *>(a.in) + (SLICES ? rowg * a.N : off);
    OutT *out = reinterpret_cast<OutT *>(a.out) + off;
    const int cpr = a.N / CW;

    uint4 raw[CH];                                        // chunks past the row hold zeros
    bool ok[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int q = lane + 64 * i;
        ok[i] = q < cpr;
        raw[i] = make_uint4(0u, 0u, 0u, 0u);
        if (ok[i]) raw[i] = *reinterpret_cast<const uint4 *>(in + (int64_t)q * CW);
    }
    if constexpr (SLICES) {
        for (int sl = 1; sl < a.slices; ++sl) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                if (ok[i]) {
                    const floatx4 v = *reinterpret_cast<const floatx4 *>(in + sl * a.slice_stride + (int64_t)(lane + 64 * i) * CW);
                    raw[i].x = as_u32(as_f32(raw[i].x) + v[0]); raw[i].y = as_u32(as_f32(raw[i].y) + v[1]);
                    raw[i].z = as_u32(as_f32(raw[i].z) + v[2]); raw[i].w = as_u32(as_f32(raw[i].w) + v[3]);
                }
        }
        dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                if (ok[i]) {
                    floatx4 bb = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (a.b != nullptr) bb = *reinterpret_cast<const floatx4 *>(a.b + (lane + 64 * i) * CW);
                    raw[i].x = as_u32(activate<ACT>(fmaf(a.scale, as_f32(raw[i].x), a.post * bb[0]), a.lo, a.hi));
                    raw[i].y = as_u32(activate<ACT>(fmaf(a.scale, as_f32(raw[i].y), a.post * bb[1]), a.lo, a.hi));
                    raw[i].z = as_u32(activate<ACT>(fmaf(a.scale, as_f32(raw[i].z), a.post * bb[2]), a.lo, a.hi));
                    raw[i].w = as_u32(activate<ACT>(fmaf(a.scale, as_f32(raw[i].w), a.post * bb[3]), a.lo, a.hi));
                }
        });
    }
    const float inv_n = 1.0f / (float)a.N;
    // Called between the passes over a 16-bit row: the compiler must not keep the fp32 image of
    // one pass for the next (it would, as a common subexpression), that is what costs registers.
    auto forget_unpacked = [&]() __attribute__((always_inline)) {
        if constexpr (PACKED) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                asm volatile("" : "+v"(raw[i].x), "+v"(raw[i].y), "+v"(raw[i].z), "+v"(raw[i].w));
        }
    };
    auto put = [&](int i, const float (&v)[CW]) __attribute__((always_inline)) {
        if constexpr (sizeof(OutT) == sizeof(T)) {
            *reinterpret_cast<uint4 *>(out + (int64_t)(lane + 64 * i) * CW) = Store<OutT>::pack(v);
        } else {                                          // four fp32 values to a 16-bit type: 8 bytes
            const float f[8] = {v[0], v[1], v[2], v[3], 0.0f, 0.0f, 0.0f, 0.0f};
            const uint4 u = Store<OutT>::pack(f);
            *reinterpret_cast<uint2 *>(out + (int64_t)(lane + 64 * i) * CW) = make_uint2(u.x, u.y);
        }
    };

    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident();
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) {
                float v[CW];
                Store<T>::unpack(raw[i], v);
#pragma unroll
                for (int e = 0; e < CW; ++e) m = max_nc(m, v[e]);
            }
        m = allreduce64<OpMax>(m);
        const float c = -m * LOG2E;                       // exp(v - m) = exp2(v*log2(e) + c)
        forget_unpacked();
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) {
                float v[CW];
                Store<T>::unpack(raw[i], v);
#pragma unroll
                for (int e = 0; e < CW; ++e) {
                    v[e] = exp_rel(v[e], c);
                    s += v[e];
                }
                if constexpr (!PACKED) {
                    if (a.norm == FGE_NORM_SOFTMAX) raw[i] = Store<T>::pack(v);
                }
            }
        s = allreduce64<OpSum>(s);
        if (a.norm == FGE_NORM_SOFTMAX) {
            const float inv = fast_rcp(s);
            forget_unpacked();
#pragma unroll
            for (int i = 0; i < CH; ++i)
                if (ok[i]) {
                    float v[CW];
                    Store<T>::unpack(raw[i], v);
#pragma unroll
                    for (int e = 0; e < CW; ++e) v[e] = (PACKED ? exp_rel(v[e], c) : v[e]) * inv;
                    put(i, v);
                }
        } else {
            if (lane == 0) a.aux[rowg] = m + __logf(s);
            if (SLICES || a.in != a.out) {
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    if (ok[i]) {
                        if constexpr (SLICES) {
                            float v[CW];
                            Store<T>::unpack(raw[i], v);
                            put(i, v);
                        } else {
                            *reinterpret_cast<uint4 *>(out + (int64_t)(lane + 64 * i) * CW) = raw[i];
                        }
                    }
            }
        }
        return;
    }

    // gamma / beta of a chunk are read when it is written (fp32, 16 bytes at a time)
    auto affine_put = [&](int i, float scale, float shift, bool with_beta) __attribute__((always_inline)) {
        float v[CW];
        Store<T>::unpack(raw[i], v);
        const int col = (lane + 64 * i) * CW;
#pragma unroll
        for (int e4 = 0; e4 < CW; e4 += 4) {
            float4 g = make_float4(1.f, 1.f, 1.f, 1.f), b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (a.gamma) g = *reinterpret_cast<const float4 *>(a.gamma + col + e4);
            if (with_beta && a.beta) b = *reinterpret_cast<const float4 *>(a.beta + col + e4);
            v[e4 + 0] = (v[e4 + 0] - shift) * scale * g.x + b.x;
            v[e4 + 1] = (v[e4 + 1] - shift) * scale * g.y + b.y;
            v[e4 + 2] = (v[e4 + 2] - shift) * scale * g.z + b.z;
            v[e4 + 3] = (v[e4 + 3] - shift) * scale * g.w + b.w;
        }
        put(i, v);
    };
    if (a.norm == FGE_NORM_LAYERNORM) {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            float v[CW];
            Store<T>::unpack(raw[i], v);                              // masked chunks hold zeros
#pragma unroll
            for (int e = 0; e < CW; ++e) s += v[e];
        }
        const float mean = allreduce64<OpSum>(s) * inv_n;
        forget_unpacked();
        float q2 = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) {
                float v[CW];
                Store<T>::unpack(raw[i], v);
#pragma unroll
                for (int e = 0; e < CW; ++e) {
                    const float d = v[e] - mean;
                    q2 += d * d;
                }
            }
        const float rstd = rsqrtf(allreduce64<OpSum>(q2) * inv_n + a.eps);
        forget_unpacked();
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) affine_put(i, rstd, mean, true);
    } else {                                              // FGE_NORM_RMSNORM (beta is not part of it)
        float q2 = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            float v[CW];
            Store<T>::unpack(raw[i], v);
#pragma unroll
            for (int e = 0; e < CW; ++e) q2 += v[e] * v[e];
        }
        const float rr = rsqrtf(allreduce64<OpSum>(q2) * inv_n + a.eps);
        forget_unpacked();
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) affine_put(i, rr, 0.0f, false);
    }
}

// K3 for rows wider than rownorm_kernel's registers hold: one workgroup of four waves per row,
// the row read once per pass (two passes for RMSNorm, three for the others) - from memory, where
// a row of this width sits in the L2 between the passes, or from LDS (CACHE) - 16 bytes per lane and step.  In place
// (in == out) is fine: a thread only ever rewrites the chunks it read itself.
// CACHE: the row (at most 64 KB) is kept in LDS as loaded, each thread parking the chunks it will
// need again, so memory is read once; two such workgroups fit a CU.
template <typename T, bool CACHE>
__global__ __launch_bounds__(256) void rownorm_wide_kernel(const RowArgs a) {
    constexpr int CW = Store<T>::CW;
    __shared__ float red[2][4];
    extern __shared__ __attribute__((aligned(16))) unsigned char rowbuf_raw[];
    uint4 *rowbuf = reinterpret_cast<uint4 *>(rowbuf_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t rowg = blockIdx.x;
    const int64_t off = (rowg / a.M) * a.bso + (rowg % a.M) * a.ldo;
    const T *in = reinterpret_cast<const T *>(a.in) + off;
    T *out = reinterpret_cast<T *>(a.out) + off;
    const int cpr = a.N / CW;
    const float inv_n = 1.0f / (float)a.N;
    int turn = 0;
    // reduction over the workgroup: waves first, then the four partial results through LDS
    // (two alternating slots, so one barrier per reduction is enough)
    auto block_reduce = [&]<typename Op>(Op, float v) __attribute__((always_inline)) {
        v = allreduce64<Op>(v);
        if (lane == 0) red[turn][wave] = v;
        __syncthreads();
        const float r = Op::f(Op::f(red[turn][0], red[turn][1]), Op::f(red[turn][2], red[turn][3]));
        turn ^= 1;
        return r;
    };
    // first touch of a chunk (from memory; parked in LDS when cached) and later touches
    auto load_first = [&](int q, float (&v)[CW]) __attribute__((always_inline)) {
        const uint4 u = *reinterpret_cast<const uint4 *>(in + (int64_t)q * CW);
        if constexpr (CACHE) rowbuf[q] = u;
        Store<T>::unpack(u, v);
    };
    auto load = [&](int q, float (&v)[CW]) __attribute__((always_inline)) {
        if constexpr (CACHE) Store<T>::unpack(rowbuf[q], v);
        else                 Store<T>::unpack(*reinterpret_cast<const uint4 *>(in + (int64_t)q * CW), v);
    };
    auto store = [&](int q, const float (&v)[CW]) __attribute__((always_inline)) {
        *reinterpret_cast<uint4 *>(out + (int64_t)q * CW) = Store<T>::pack(v);
    };

    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident();
#pragma unroll 4
        for (int q = tid; q < cpr; q += 256) {
            float v[CW];
            load_first(q, v);
#pragma unroll
            for (int e = 0; e < CW; ++e) m = max_nc(m, v[e]);
        }
        m = block_reduce(OpMax{}, m);
        const float c = -m * LOG2E;
        float s = 0.0f;
#pragma unroll 4
        for (int q = tid; q < cpr; q += 256) {
            float v[CW];
            load(q, v);
#pragma unroll
            for (int e = 0; e < CW; ++e) s += exp_rel(v[e], c);
        }
        s = block_reduce(OpSum{}, s);
        if (a.norm == FGE_NORM_LOGSUMEXP) {
            if (tid == 0) a.aux[rowg] = m + __logf(s);
            if (a.in != a.out)
                for (int q = tid; q < cpr; q += 256)
                    *reinterpret_cast<uint4 *>(out + (int64_t)q * CW) =
                        CACHE ? rowbuf[q] : *reinterpret_cast<const uint4 *>(in + (int64_t)q * CW);
            return;
        }
        const float inv = fast_rcp(s);
#pragma unroll 4
        for (int q = tid; q < cpr; q += 256) {
            float v[CW];
            load(q, v);
#pragma unroll
            for (int e = 0; e < CW; ++e) v[e] = exp_rel(v[e], c) * inv;
            store(q, v);
        }
        return;
    }
    float shift = 0.0f, scale;
    if (a.norm == FGE_NORM_LAYERNORM) {
        float sm = 0.0f;
#pragma unroll 4
        for (int q = tid; q < cpr; q += 256) {
            float v[CW];
            load_first(q, v);
#pragma unroll
            for (int e = 0; e < CW; ++e) sm += v[e];
        }
        shift = block_reduce(OpSum{}, sm) * inv_n;
        float q2 = 0.0f;
#pragma unroll 4
        for (int q = tid; q < cpr; q += 256) {
            float v[CW];
            load(q, v);
#pragma unroll
            for (int e = 0; e < CW; ++e) q2 += (v[e] - shift) * (v[e] - shift);
        }
        scale = rsqrtf(block_reduce(OpSum{}, q2) * inv_n + a.eps);
    } else {                                              // FGE_NORM_RMSNORM
        float q2 = 0.0f;
#pragma unroll 4
        for (int q = tid; q < cpr; q += 256) {
            float v[CW];
            load_first(q, v);
#pragma unroll
            for (int e = 0; e < CW; ++e) q2 += v[e] * v[e];
        }
        scale = rsqrtf(block_reduce(OpSum{}, q2) * inv_n + a.eps);
    }
    const bool use_beta = a.norm == FGE_NORM_LAYERNORM && a.beta != nullptr;
#pragma unroll 4
    for (int q = tid; q < cpr; q += 256) {
        float v[CW];
        load(q, v);
#pragma unroll
        for (int e4 = 0; e4 < CW; e4 += 4) {
            float4 g = make_float4(1.f, 1.f, 1.f, 1.f), b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (a.gamma) g = *reinterpret_cast<const float4 *>(a.gamma + q * CW + e4);
            if (use_beta) b = *reinterpret_cast<const float4 *>(a.beta + q * CW + e4);
            v[e4 + 0] = (v[e4 + 0] - shift) * scale * g.x + b.x;
            v[e4 + 1] = (v[e4 + 1] - shift) * scale * g.y + b.y;
            v[e4 + 2] = (v[e4 + 2] - shift) * scale * g.z + b.z;
            v[e4 + 3] = (v[e4 + 3] - shift) * scale * g.w + b.w;
        }
        store(q, v);
    }
}

// Row op over a K-split product for the few rows such problems have: one workgroup of four
// waves per row.  Every thread owns up to NCH chunks of four neighbouring columns (N <= 1024 * NCH),
// adds the S partial products of its chunks in slice order - the loads of a chunk's slices are
// independent of each other, so they are all in flight together: one memory round trip for the
// whole row, where a single wave walking the slices of a row paid one per slice -, applies scale,
// bias, activation (and the gate of the gated form), keeps the fp32 row in registers, reduces the
// row statistic over the workgroup and stores the finished row.  The result does not depend on
// the schedule (slice order, fixed reduction tree).
struct SplitRowArgs {
    const float *P, *P2;        // S dense fp32 rows x N partial products each, `slice` elements apart (P2: second product of the gated form, or null)
    const float *b, *b2, *gamma, *beta;
    void *out;
    float *aux;
    int M, N, S;                // rows per problem (row r of the partials is row r % M of problem r / M), columns, slices
    int64_t slice, ldo, bso;
    float scale, post, lo, hi, eps;
    int act, norm;
};
template <typename OutT, int NCH>
__global__ __launch_bounds__(256) void splitk_rows_kernel(const SplitRowArgs a) {
    __shared__ float red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t rowg = blockIdx.x;
    OutT *out = reinterpret_cast<OutT *>(a.out) + (rowg / a.M) * a.bso + (rowg % a.M) * a.ldo;
    const int n4 = a.N >> 2;
    const float inv_n = 1.0f / (float)a.N;
    int turn = 0;
    auto block_reduce = [&]<typename Op>(Op, float v) __attribute__((always_inline)) {
        v = allreduce64<Op>(v);
        if (lane == 0) red[turn][wave] = v;
        __syncthreads();
        const float r = Op::f(Op::f(red[turn][0], red[turn][1]), Op::f(red[turn][2], red[turn][3]));
        turn ^= 1;
        return r;
    };
    auto slices = [&](const float *q) __attribute__((always_inline)) {
        floatx4 acc = *reinterpret_cast<const floatx4 *>(q);
#pragma unroll 4
        for (int sl = 1; sl < a.S; ++sl) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(q + sl * a.slice);
            acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        return acc;
    };
    float v[NCH][4];
    bool ok[NCH];
    dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int q = tid + j * 256;
            ok[j] = q < n4;
            const int col = (ok[j] ? q : 0) << 2;
            const floatx4 acc = slices(a.P + rowg * a.N + col);
            floatx4 gate = {1.0f, 1.0f, 1.0f, 1.0f};
            if (a.P2 != nullptr) {
                const floatx4 u = slices(a.P2 + rowg * a.N + col);
#pragma unroll
                for (int e = 0; e < 4; ++e) gate[e] = a.scale * u[e] + (a.b2 != nullptr ? a.post * a.b2[col + e] : 0.0f);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float bias = a.b != nullptr ? a.post * a.b[col + e] : 0.0f;
                v[j][e] = activate<ACT>(a.scale * acc[e] + bias, a.lo, a.hi) * gate[e];
            }
        }
    });
    auto put = [&](int j, const float (&r)[4]) __attribute__((always_inline)) {
        if (!ok[j]) return;
        OutT *o = out + ((tid + j * 256) << 2);
        if constexpr (sizeof(OutT) == 4) {
            *reinterpret_cast<floatx4 *>(o) = floatx4{r[0], r[1], r[2], r[3]};
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) Store<OutT>::put(o + e, r[e]);
        }
    };
    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident();
#pragma unroll
        for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) if (ok[j]) m = max_nc(m, v[j][e]);
        m = block_reduce(OpMax{}, m);
        const float c = -m * LOG2E;
        float sum = 0.0f;
        float ex[NCH][4];
#pragma unroll
        for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) { ex[j][e] = ok[j] ? exp_rel(v[j][e], c) : 0.0f; sum += ex[j][e]; }
        sum = block_reduce(OpSum{}, sum);
        if (a.norm == FGE_NORM_LOGSUMEXP) {
            if (tid == 0) a.aux[rowg] = m + __logf(sum);
#pragma unroll
            for (int j = 0; j < NCH; ++j) put(j, v[j]);
            return;
        }
        const float inv = fast_rcp(sum);
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) ex[j][e] *= inv;
            put(j, ex[j]);
        }
        return;
    }
    float shift = 0.0f;
    if (a.norm == FGE_NORM_LAYERNORM) {
        float sm = 0.0f;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) if (ok[j]) sm += v[j][e];
        shift = block_reduce(OpSum{}, sm) * inv_n;
    }
    float q2 = 0.0f;
#pragma unroll
    for (int j = 0; j < NCH; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) if (ok[j]) q2 += (v[j][e] - shift) * (v[j][e] - shift);
    const float rstd = rsqrtf(block_reduce(OpSum{}, q2) * inv_n + a.eps);
    const bool use_beta = a.norm == FGE_NORM_LAYERNORM && a.beta != nullptr;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        if (!ok[j]) continue;
        const int col = (tid + j * 256) << 2;
        floatx4 g = {1.0f, 1.0f, 1.0f, 1.0f}, be = {0.0f, 0.0f, 0.0f, 0.0f};
        if (a.gamma != nullptr) g = *reinterpret_cast<const floatx4 *>(a.gamma + col);
        if (use_beta) be = *reinterpret_cast<const floatx4 *>(a.beta + col);
        float r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = (v[j][e] - shift) * rstd * g[e] + be[e];
        put(j, r);
    }
}
template <typename OutT> inline hipError_t launch_splitk_rows_t(const SplitRowArgs &a, int64_t rows, hipStream_t s) {
    const dim3 grid((unsigned)rows), block(256);
    const int nch = (a.N / 4 + 255) / 256;
    if (nch <= 1)      hipLaunchKernelGGL((splitk_rows_kernel<OutT, 1>), grid, block, 0, s, a);
    else if (nch <= 2) hipLaunchKernelGGL((splitk_rows_kernel<OutT, 2>), grid, block, 0, s, a);
    else if (nch <= 4) hipLaunchKernelGGL((splitk_rows_kernel<OutT, 4>), grid, block, 0, s, a);
    else if (nch <= 8) hipLaunchKernelGGL((splitk_rows_kernel<OutT, 8>), grid, block, 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// Second pass of the fused path for rows split over several column strips.  The tile kernel
// left one pair per (row, strip) in the workspace - `tiles_n` strips of `bn` columns per row -
// and the row itself parked in `out`; this kernel merges the pairs and finishes the row in
// place.  Merge rules:
//   softmax / logsumexp: m = max_t m_t, s = sum_t s_t exp(m_t - m); parked e_t * exp(m_t - m)/s
//   layernorm: mean = sum_t n_t mean_t / N, M2 = sum_t (M2_t + n_t (mean_t - mean)^2)
//   rmsnorm:   sum of the per-strip sums of squares
// WAVES = 1: one wavefront per row, four rows per workgroup.  WAVES = 4 (wide rows): the four
// waves of a workgroup share one row - each merges the pairs for itself (they are few), the
// elements are divided among all 256 threads.
template <typename T, int WAVES>
__global__ __launch_bounds__(256) void finish_kernel(const RowArgs a) {
    constexpr int CW = Store<T>::CW;
    constexpr int TEAM = 64 * WAVES;                      // threads per row
    const int lane = threadIdx.x & 63;
    const int member = WAVES == 1 ? lane : (int)threadIdx.x;
    const int64_t rowg = WAVES == 1 ? (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6) : (int64_t)blockIdx.x;
    if (rowg >= (int64_t)a.batch * a.M) return;           // wave-uniform
    T *out = reinterpret_cast<T *>(a.out) + (rowg / a.M) * a.bso + (rowg % a.M) * a.ldo;
    const int cpr = a.N / CW;
    const int S = a.tiles_n, SW = a.bn;
    const float2 *wr = a.ws + rowg * S;
    const float inv_n = 1.0f / (float)a.N;

    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident();
        for (int t = lane; t < S; t += 64) m = fmaxf(m, wr[t].x);
        m = allreduce64<OpMax>(m);
        float s = 0.0f;
        for (int t = lane; t < S; t += 64) s += wr[t].y * fast_exp(wr[t].x - m);
        s = allreduce64<OpSum>(s);
        if (a.norm == FGE_NORM_LOGSUMEXP) {
            if (member == 0) a.aux[rowg] = m + __logf(s);
            return;
        }
        const float inv = fast_rcp(s);
#pragma unroll 4
        for (int q = member; q < cpr; q += TEAM) {
            const float f = fast_exp(wr[(q * CW) / SW].x - m) * inv;
            float v[CW];
            Store<T>::unpack(*reinterpret_cast<const uint4 *>(out + (int64_t)q * CW), v);
#pragma unroll
            for (int e = 0; e < CW; ++e) v[e] *= f;
            *reinterpret_cast<uint4 *>(out + (int64_t)q * CW) = Store<T>::pack(v);
        }
        return;
    }
    float scale, shift;
    if (a.norm == FGE_NORM_LAYERNORM) {
        float sm = 0.0f;
        for (int t = lane; t < S; t += 64) sm += (float)max(0, min(SW, a.N - t * SW)) * wr[t].x;
        shift = allreduce64<OpSum>(sm) * inv_n;
        float m2 = 0.0f;
        for (int t = lane; t < S; t += 64) {
            const float d = wr[t].x - shift;
            m2 += wr[t].y + (float)max(0, min(SW, a.N - t * SW)) * d * d;
        }
        scale = rsqrtf(allreduce64<OpSum>(m2) * inv_n + a.eps);
    } else {
        float ss = 0.0f;
        for (int t = lane; t < S; t += 64) ss += wr[t].x;
        shift = 0.0f;
        scale = rsqrtf(allreduce64<OpSum>(ss) * inv_n + a.eps);
    }
    const bool use_beta = a.norm == FGE_NORM_LAYERNORM && a.beta != nullptr;
#pragma unroll 4
    for (int q = member; q < cpr; q += TEAM) {
        float v[CW];
        Store<T>::unpack(*reinterpret_cast<const uint4 *>(out + (int64_t)q * CW), v);
#pragma unroll
        for (int e4 = 0; e4 < CW; e4 += 4) {
            float4 g = make_float4(1.f, 1.f, 1.f, 1.f), b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (a.gamma) g = *reinterpret_cast<const float4 *>(a.gamma + q * CW + e4);
            if (use_beta) b = *reinterpret_cast<const float4 *>(a.beta + q * CW + e4);
            v[e4 + 0] = (v[e4 + 0] - shift) * scale * g.x + b.x;
            v[e4 + 1] = (v[e4 + 1] - shift) * scale * g.y + b.y;
            v[e4 + 2] = (v[e4 + 2] - shift) * scale * g.z + b.z;
            v[e4 + 3] = (v[e4 + 3] - shift) * scale * g.w + b.w;
        }
        *reinterpret_cast<uint4 *>(out + (int64_t)q * CW) = Store<T>::pack(v);
    }
}

}  // namespace fge
