// Row-wise and elementwise kernels: the unfused K2 (activation) and K3 (row operation), and
// the light second pass of the fused path that merges per-strip row statistics.
// One 64-lane wavefront owns one row; data moves in 16-byte chunks per lane.
#pragma once
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

// K3: out = rowop(A).  The row lives in registers: lane l holds chunks l, l+64, ... (CH of them).
template <typename T, int CH>
__global__ __launch_bounds__(256) void rownorm_kernel(const RowArgs a) {
    constexpr int CW = Store<T>::CW;
    const int lane = threadIdx.x & 63;
    const int64_t rowg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rowg >= (int64_t)a.batch * a.M) return;           // wave-uniform
    const int64_t off = (rowg / a.M) * a.bso + (rowg % a.M) * a.ldo;
    const T *in = reinterpret_cast<const T *>(a.in) + off;
    T *out = reinterpret_cast<T *>(a.out) + off;
    const int cpr = a.N / CW;

    float v[CH][CW];
    bool ok[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int q = lane + 64 * i;
        ok[i] = q < cpr;
        if (ok[i]) {
            Store<T>::unpack(*reinterpret_cast<const uint4 *>(in + (int64_t)q * CW), v[i]);
        } else {
#pragma unroll
            for (int e = 0; e < CW; ++e) v[i][e] = 0.0f;
        }
    }
    const float inv_n = 1.0f / (float)a.N;
    auto store_row = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) *reinterpret_cast<uint4 *>(out + (int64_t)(lane + 64 * i) * CW) = Store<T>::pack(v[i]);
    };

    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident();
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) {
#pragma unroll
                for (int e = 0; e < CW; ++e) m = fmaxf(m, v[i][e]);
            }
        m = allreduce64<OpMax>(m);
        float s = 0.0f;
        if (a.norm == FGE_NORM_SOFTMAX) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
#pragma unroll
                for (int e = 0; e < CW; ++e) {
                    v[i][e] = ok[i] ? fast_exp(v[i][e] - m) : 0.0f;
                    s += v[i][e];
                }
            s = allreduce64<OpSum>(s);
            const float inv = fast_rcp(s);
#pragma unroll
            for (int i = 0; i < CH; ++i)
#pragma unroll
                for (int e = 0; e < CW; ++e) v[i][e] *= inv;
            store_row();
        } else {
#pragma unroll
            for (int i = 0; i < CH; ++i)
#pragma unroll
                for (int e = 0; e < CW; ++e) s += ok[i] ? fast_exp(v[i][e] - m) : 0.0f;
            s = allreduce64<OpSum>(s);
            if (lane == 0) a.aux[rowg] = m + __logf(s);
            if (a.in != a.out) store_row();
        }
        return;
    }

    // gamma / beta for this lane's chunks are read when needed (fp32, 16 bytes at a time)
    auto affine = [&](int i, float scale, float shift) __attribute__((always_inline)) {
        const int col = (lane + 64 * i) * CW;
#pragma unroll
        for (int e4 = 0; e4 < CW; e4 += 4) {
            float4 g = make_float4(1.f, 1.f, 1.f, 1.f), b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (a.gamma) g = *reinterpret_cast<const float4 *>(a.gamma + col + e4);
            if (a.beta) b = *reinterpret_cast<const float4 *>(a.beta + col + e4);
            v[i][e4 + 0] = (v[i][e4 + 0] - shift) * scale * g.x + b.x;
            v[i][e4 + 1] = (v[i][e4 + 1] - shift) * scale * g.y + b.y;
            v[i][e4 + 2] = (v[i][e4 + 2] - shift) * scale * g.z + b.z;
            v[i][e4 + 3] = (v[i][e4 + 3] - shift) * scale * g.w + b.w;
        }
    };
    if (a.norm == FGE_NORM_LAYERNORM) {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int e = 0; e < CW; ++e) s += v[i][e];            // masked chunks hold zeros
        const float mean = allreduce64<OpSum>(s) * inv_n;
        float q2 = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int e = 0; e < CW; ++e) {
                const float d = v[i][e] - mean;
                q2 += ok[i] ? d * d : 0.0f;
            }
        const float rstd = rsqrtf(allreduce64<OpSum>(q2) * inv_n + a.eps);
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (ok[i]) affine(i, rstd, mean);
    } else {  // FGE_NORM_RMSNORM (beta is not part of it)
        float q2 = 0.0f;
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int e = 0; e < CW; ++e) q2 += v[i][e] * v[i][e];
        const float rr = rsqrtf(allreduce64<OpSum>(q2) * inv_n + a.eps);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (!ok[i]) continue;
            const int col = (lane + 64 * i) * CW;
#pragma unroll
            for (int e4 = 0; e4 < CW; e4 += 4) {
                float4 g = make_float4(1.f, 1.f, 1.f, 1.f);
                if (a.gamma) g = *reinterpret_cast<const float4 *>(a.gamma + col + e4);
                v[i][e4 + 0] *= rr * g.x; v[i][e4 + 1] *= rr * g.y;
                v[i][e4 + 2] *= rr * g.z; v[i][e4 + 3] *= rr * g.w;
            }
        }
    }
    store_row();
}

// Second pass of the fused path for rows split over several column strips.  The tile kernel
// left one pair per (row, strip) in the workspace - `tiles_n` strips of `bn` columns per row -
// and the row itself parked in `out`; this kernel merges the pairs and finishes the row in
// place.  One wavefront per row.  Merge rules:
//   softmax / logsumexp: m = max_t m_t, s = sum_t s_t exp(m_t - m); parked e_t * exp(m_t - m)/s
//   layernorm: mean = sum_t n_t mean_t / N, M2 = sum_t (M2_t + n_t (mean_t - mean)^2)
//   rmsnorm:   sum of the per-strip sums of squares
template <typename T>
__global__ __launch_bounds__(256) void finish_kernel(const RowArgs a) {
    constexpr int CW = Store<T>::CW;
    const int lane = threadIdx.x & 63;
    const int64_t rowg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
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
            if (lane == 0) a.aux[rowg] = m + __logf(s);
            return;
        }
        const float inv = fast_rcp(s);
        for (int q = lane; q < cpr; q += 64) {
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
    for (int q = lane; q < cpr; q += 64) {
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
