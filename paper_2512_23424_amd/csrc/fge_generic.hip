// Element-granular kernels for shapes the vectorised kernels do not take: extents or strides
// that are not multiples of 16 bytes, and row operations over rows wider than a wave's
// registers hold.  They make every valid shape computable; they are not tuned (plain fp32 FMA
// on the vector ALU, scalar loads and stores, rows re-read from memory per pass).
//
//   generic_gemm_kernel : dst = act(post*(alpha*X.W^T + b))   32x32 tile, LDS staged, fp32 FMA
//   generic_act_kernel  : dst = act(src) [* second operand]   elementwise
//   generic_row_kernel  : out = rowop(src)                    one wave per row, passes over src
//   splitk_sum_kernel   : dst = act(post*(alpha*sum_s P_s + b))  the slices of a K-split product, summed in slice order
//   pad_rows_kernel     : dense copy of a matrix with K padded by zeros to whole 16-byte chunks
//                         (and zero rows appended): what makes an operand with odd extents or
//                         strides fit the vectorised kernels, at one extra read and write of it
#include "fge_launch.h"

namespace fge {

namespace {

template <typename T> __device__ __forceinline__ const T *row_ptr(const void *base, int64_t rowg, int M,
                                                                 int64_t ld, int64_t bs) {
    return reinterpret_cast<const T *>(base) + (rowg / M) * bs + (rowg % M) * ld;
}

template <typename InT, typename DstT>
__global__ __launch_bounds__(256) void generic_gemm_kernel(const GenArgs a) {
    constexpr int T = 32;
    __shared__ float xs[T][T + 1], ws[T][T + 1];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 x 8 threads
    const int n0 = blockIdx.x * T, m0 = blockIdx.y * T, z = blockIdx.z;
    const InT *X = reinterpret_cast<const InT *>(a.X) + (int64_t)z * a.bsx;
    const InT *W = reinterpret_cast<const InT *>(a.W);
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int k0 = 0; k0 < a.K; k0 += T) {
        const int k = k0 + tx;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = ty + 8 * i;
            xs[r][tx] = (m0 + r < a.M && k < a.K) ? Store<InT>::get(X + (int64_t)(m0 + r) * a.ldx + k) : 0.0f;
            ws[r][tx] = (n0 + r < a.N && k < a.K) ? Store<InT>::get(W + (int64_t)(n0 + r) * a.ldw + k) : 0.0f;
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < T; ++kk) {
            const float w = ws[tx][kk];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = fmaf(xs[ty + 8 * i][kk], w, acc[i]);
        }
        __syncthreads();
    }
    const int col = n0 + tx;
    if (col >= a.N) return;
    const float scale = a.post * a.alpha;
    const float bias = a.b != nullptr ? a.post * a.b[col] : 0.0f;
    DstT *dst = reinterpret_cast<DstT *>(a.dst) + (int64_t)z * a.bsd;
    dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = m0 + ty + 8 * i;
            if (row < a.M)
                Store<DstT>::put(dst + (int64_t)row * a.ldd + col, activate<ACT>(scale * acc[i] + bias, a.lo, a.hi));
        }
    });
}

template <typename T>
__global__ __launch_bounds__(256) void generic_act_kernel(const GenArgs a) {
    const int64_t total = (int64_t)a.batch * a.M * a.N;
    dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
        for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
            const int64_t rowg = idx / a.N;
            const int c = (int)(idx - rowg * a.N);
            const int64_t off = (rowg / a.M) * a.bsd + (rowg % a.M) * a.ldd + c;
            float v = activate<ACT>(Store<T>::get(reinterpret_cast<const T *>(a.X) + off), a.lo, a.hi);
            if (a.W != nullptr) v *= Store<T>::get(reinterpret_cast<const T *>(a.W) + off);   // gate
            Store<T>::put(reinterpret_cast<T *>(a.dst) + off, v);
        }
    });
}

// src: rows x N of SrcT (row stride lds, batch stride bss); out: rows x N of OutT (ldd, bsd).
template <typename SrcT, typename OutT>
__global__ __launch_bounds__(256) void generic_row_kernel(const GenArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t rowg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rowg >= (int64_t)a.batch * a.M) return;                       // wave-uniform
    const SrcT *src = row_ptr<SrcT>(a.X, rowg, a.M, a.ldx, a.bsx);
    OutT *out = const_cast<OutT *>(row_ptr<OutT>(a.dst, rowg, a.M, a.ldd, a.bsd));
    const float inv_n = 1.0f / (float)a.N;
    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident();
        for (int j = lane; j < a.N; j += 64) m = max_nc(m, Store<SrcT>::get(src + j));
        m = allreduce64<OpMax>(m);
        float s = 0.0f;
        for (int j = lane; j < a.N; j += 64) s += fast_exp(Store<SrcT>::get(src + j) - m);
        s = allreduce64<OpSum>(s);
        if (a.norm == FGE_NORM_SOFTMAX) {
            const float inv = 1.0f / s;
            for (int j = lane; j < a.N; j += 64) Store<OutT>::put(out + j, fast_exp(Store<SrcT>::get(src + j) - m) * inv);
        } else {
            if (lane == 0) a.aux[rowg] = m + __logf(s);
            if (reinterpret_cast<const void *>(src) != reinterpret_cast<const void *>(out))
                for (int j = lane; j < a.N; j += 64) Store<OutT>::put(out + j, Store<SrcT>::get(src + j));
        }
    } else if (a.norm == FGE_NORM_LAYERNORM) {
        float s = 0.0f;
        for (int j = lane; j < a.N; j += 64) s += Store<SrcT>::get(src + j);
        const float mean = allreduce64<OpSum>(s) * inv_n;
        float d2 = 0.0f;
        for (int j = lane; j < a.N; j += 64) {
            const float d = Store<SrcT>::get(src + j) - mean;
            d2 += d * d;
        }
        const float rstd = rsqrtf(allreduce64<OpSum>(d2) * inv_n + a.eps);
        for (int j = lane; j < a.N; j += 64) {
            const float g = a.gamma != nullptr ? a.gamma[j] : 1.0f, b = a.beta != nullptr ? a.beta[j] : 0.0f;
            Store<OutT>::put(out + j, (Store<SrcT>::get(src + j) - mean) * rstd * g + b);
        }
    } else if (a.norm == FGE_NORM_RMSNORM) {
        float s = 0.0f;
        for (int j = lane; j < a.N; j += 64) {
            const float v = Store<SrcT>::get(src + j);
            s += v * v;
        }
        const float rr = rsqrtf(allreduce64<OpSum>(s) * inv_n + a.eps);
        for (int j = lane; j < a.N; j += 64) {
            const float g = a.gamma != nullptr ? a.gamma[j] : 1.0f;
            Store<OutT>::put(out + j, Store<SrcT>::get(src + j) * rr * g);
        }
    } else {
        if (reinterpret_cast<const void *>(src) != reinterpret_cast<const void *>(out))
            for (int j = lane; j < a.N; j += 64) Store<OutT>::put(out + j, Store<SrcT>::get(src + j));
    }
}

// The same row operation for fp32 source rows that start on 16-byte boundaries (the rows of padded
// width the repacked path produces; ldx and bsx multiples of 4) and a result of any width and
// stride: one workgroup of four waves per row.  The statistics passes read 16 bytes per lane, four
// loads in flight per thread; the last pass reads and writes one element per lane, so that a
// wave's stores are one contiguous run whatever the alignment of the result's rows.  CACHE: the
// row (at most 64 KB) is parked in LDS by the first pass and read from there afterwards; longer
// rows are read from memory by every pass, and softmax / logsumexp take their two statistics in
// one pass.
// (The wave-per-row kernel above walks a row with one load in flight per lane: 2048 rows of 50257
// columns took it 1.0 ms.)
template <typename OutT, bool CACHE>
__global__ __launch_bounds__(256) void aligned_src_row_kernel(const GenArgs a) {
    __shared__ float red[2][4];
    extern __shared__ __attribute__((aligned(16))) float rowbuf[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t rowg = blockIdx.x;
    const float *src = row_ptr<float>(a.X, rowg, a.M, a.ldx, a.bsx);
    OutT *out = const_cast<OutT *>(row_ptr<OutT>(a.dst, rowg, a.M, a.ldd, a.bsd));
    const int n4 = a.N >> 2;                                     // whole groups of four columns
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
    // first pass over the row: f(v) for every valid element, 16 bytes per lane (+ the ragged tail)
    auto sweep_first = [&](auto &&f) __attribute__((always_inline)) {
#pragma unroll 4
        for (int q = tid; q < n4; q += 256) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(src + 4 * q);
            if constexpr (CACHE) *reinterpret_cast<floatx4 *>(rowbuf + 4 * q) = v;
            f(v[0]); f(v[1]); f(v[2]); f(v[3]);
        }
        const int j = 4 * n4 + tid;
        if (j < a.N) {
            const float v = src[j];
            if constexpr (CACHE) rowbuf[j] = v;
            f(v);
        }
        if constexpr (CACHE) __syncthreads();
    };
    auto sweep = [&](auto &&f) __attribute__((always_inline)) {
        const float *r = CACHE ? rowbuf : src;
#pragma unroll 4
        for (int q = tid; q < n4; q += 256) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(r + 4 * q);
            f(v[0]); f(v[1]); f(v[2]); f(v[3]);
        }
        const int j = 4 * n4 + tid;
        if (j < a.N) f(r[j]);
    };
    // last pass: out[j] = g(j, v[j]), one element per lane and step
    auto emit = [&](auto &&g) __attribute__((always_inline)) {
        const float *r = CACHE ? rowbuf : src;
#pragma unroll 4
        for (int j = tid; j < a.N; j += 256) Store<OutT>::put(out + j, g(j, r[j]));
    };
    if (a.norm == FGE_NORM_SOFTMAX || a.norm == FGE_NORM_LOGSUMEXP) {
        float m = OpMax::ident(), s = 0.0f, c;
        if constexpr (CACHE) {
            sweep_first([&](float v) __attribute__((always_inline)) { m = max_nc(m, v); });
            m = block_reduce(OpMax{}, m);
            c = -m * LOG2E;
            sweep([&](float v) __attribute__((always_inline)) { s += exp_rel(v, c); });
            s = block_reduce(OpSum{}, s);
        } else {
            // a row that is read from memory every time: maximum and sum in one pass - every thread
            // keeps a running maximum and rescales its sum so far whenever the maximum rises
            // (a thread without elements ends with 0 * exp2(-inf) = 0)
#pragma unroll 4
            for (int q = tid; q < n4; q += 256) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(src + 4 * q);
                const float mn = max_nc(max_nc(max_nc(v[0], v[1]), max_nc(v[2], v[3])), m);
                const float cn = -mn * LOG2E;
                s = s * exp_rel(m, cn) + ((exp_rel(v[0], cn) + exp_rel(v[1], cn)) + (exp_rel(v[2], cn) + exp_rel(v[3], cn)));
                m = mn;
            }
            if (const int j = 4 * n4 + tid; j < a.N) {
                const float v = src[j], mn = max_nc(v, m), cn = -mn * LOG2E;
                s = s * exp_rel(m, cn) + exp_rel(v, cn);
                m = mn;
            }
            const float mt = m;
            m = block_reduce(OpMax{}, mt);
            c = -m * LOG2E;
            s = block_reduce(OpSum{}, s * exp_rel(mt, c));
        }
        if (a.norm == FGE_NORM_SOFTMAX) {
            const float inv = 1.0f / s;
            emit([&](int, float v) __attribute__((always_inline)) { return exp_rel(v, c) * inv; });
        } else {
            if (tid == 0) a.aux[rowg] = m + __logf(s);
            emit([&](int, float v) __attribute__((always_inline)) { return v; });
        }
    } else if (a.norm == FGE_NORM_LAYERNORM) {
        float s = 0.0f;
        sweep_first([&](float v) __attribute__((always_inline)) { s += v; });
        const float mean = block_reduce(OpSum{}, s) * inv_n;
        float d2 = 0.0f;
        sweep([&](float v) __attribute__((always_inline)) { d2 += (v - mean) * (v - mean); });
        const float rstd = rsqrtf(block_reduce(OpSum{}, d2) * inv_n + a.eps);
        emit([&](int j, float v) __attribute__((always_inline)) {
            return (v - mean) * rstd * (a.gamma != nullptr ? a.gamma[j] : 1.0f) + (a.beta != nullptr ? a.beta[j] : 0.0f);
        });
    } else if (a.norm == FGE_NORM_RMSNORM) {
        float s = 0.0f;
        sweep_first([&](float v) __attribute__((always_inline)) { s += v * v; });
        const float rr = rsqrtf(block_reduce(OpSum{}, s) * inv_n + a.eps);
        emit([&](int j, float v) __attribute__((always_inline)) { return v * rr * (a.gamma != nullptr ? a.gamma[j] : 1.0f); });
    } else {
        sweep_first([&](float) __attribute__((always_inline)) {});
        emit([&](int, float v) __attribute__((always_inline)) { return v; });
    }
}

// K-split product: X holds `K` dense fp32 slices of M x N partial sums, `bsx` elements apart; four
// neighbouring columns per thread (N is a multiple of 4).  The slices are added in slice order,
// so the result does not depend on how the launch was scheduled.
template <typename DstT>
__global__ __launch_bounds__(256) void splitk_sum_kernel(const GenArgs a) {
    const int n4 = a.N >> 2;
    const int64_t total = (int64_t)a.M * n4;
    const float *P = reinterpret_cast<const float *>(a.X);
    const float *P2 = reinterpret_cast<const float *>(a.W);     // gated form: the second product's slices
    const float scale = a.post * a.alpha;
    auto sum = [&](const float *q) __attribute__((always_inline)) {
        floatx4 acc = *reinterpret_cast<const floatx4 *>(q);
        for (int sl = 1; sl < a.K; ++sl) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(q + sl * a.bsx);
            acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        return acc;
    };
    dispatch_act(a.act, [&]<int ACT>() __attribute__((always_inline)) {
        for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
            const int64_t row = idx / n4;
            const int col = (int)(idx - row * n4) << 2;
            const floatx4 acc = sum(P + row * a.N + col);
            floatx4 gate = {1.0f, 1.0f, 1.0f, 1.0f};
            if (P2 != nullptr) {
                const floatx4 u = sum(P2 + row * a.N + col);
#pragma unroll
                for (int e = 0; e < 4; ++e) gate[e] = scale * u[e] + (a.b2 != nullptr ? a.post * a.b2[col + e] : 0.0f);
            }
            DstT *d = reinterpret_cast<DstT *>(a.dst) + row * a.ldd + col;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float bias = a.b != nullptr ? a.post * a.b[col + e] : 0.0f;
                Store<DstT>::put(d + e, activate<ACT>(scale * acc[e] + bias, a.lo, a.hi) * gate[e]);
            }
        }
    });
}

// dst: rows_dst x Kp dense (Kp a multiple of the 16-byte chunk); row r < batch * M is row r of the
// source (M rows per problem, strides ld / bs), zero filled from K on; rows beyond are zero.
// One thread per 16-byte chunk of dst: element-granular reads (the source rows need not be
// aligned), one 16-byte store.
template <typename T>
__global__ __launch_bounds__(256) void pad_rows_kernel(const PadArgs a) {
    constexpr int CW = 16 / (int)sizeof(T);
    const int cpr = a.Kp / CW;
    const int64_t total = a.rows_dst * cpr;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / cpr;
        const int k0 = (int)(idx - r * cpr) * CW;
        T v[CW];
        const bool live = r < (int64_t)a.batch * a.M;
        const T *src = live ? row_ptr<T>(a.src, r, a.M, a.ld, a.bs) : nullptr;
#pragma unroll
        for (int e = 0; e < CW; ++e) {
            T z{};
            v[e] = (live && k0 + e < a.K) ? src[k0 + e] : z;
        }
        *reinterpret_cast<uint4 *>(reinterpret_cast<T *>(a.dst) + r * a.Kp + k0) = *reinterpret_cast<const uint4 *>(v);
    }
}

// dst[0 .. np) = src[0 .. n), zero beyond
__global__ __launch_bounds__(256) void pad_vec_kernel(const float *src, float *dst, int n, int np) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < np) dst[i] = i < n ? src[i] : 0.0f;
}

}  // namespace

hipError_t launch_pad_rows(int dtype, hipStream_t s, const PadArgs &a) {
    const int cw = dtype == FGE_F32 ? 4 : dtype == FGE_F8E4M3 ? 16 : 8;
    const int64_t total = a.rows_dst * (a.Kp / cw);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;                           // grid-stride beyond that
    const dim3 grid((unsigned)(blocks > 0 ? blocks : 1)), block(256);
    if (dtype == FGE_F32)          hipLaunchKernelGGL((pad_rows_kernel<float>), grid, block, 0, s, a);
    else if (dtype == FGE_F8E4M3)  hipLaunchKernelGGL((pad_rows_kernel<f8_t>), grid, block, 0, s, a);
    else                           hipLaunchKernelGGL((pad_rows_kernel<bf16_t>), grid, block, 0, s, a);   // any 16-bit type: bits are copied
    return hipGetLastError();
}

hipError_t launch_pad_vec(const float *src, float *dst, int n, int np, hipStream_t s) {
    hipLaunchKernelGGL(pad_vec_kernel, dim3((unsigned)((np + 255) / 256)), dim3(256), 0, s, src, dst, n, np);
    return hipGetLastError();
}

hipError_t launch_splitk_sum(int dst_dtype, hipStream_t s, const GenArgs &a) {
    const int64_t total = (int64_t)a.M * (a.N >> 2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;                           // grid-stride beyond that
    const dim3 grid((unsigned)blocks), block(256);
    if (dst_dtype == FGE_BF16)     hipLaunchKernelGGL((splitk_sum_kernel<bf16_t>), grid, block, 0, s, a);
    else if (dst_dtype == FGE_F16) hipLaunchKernelGGL((splitk_sum_kernel<f16_t>), grid, block, 0, s, a);
    else                           hipLaunchKernelGGL((splitk_sum_kernel<float>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_generic_gemm(int in_dtype, int dst_dtype, hipStream_t s, const GenArgs &a) {
    const dim3 grid((unsigned)((a.N + 31) / 32), (unsigned)((a.M + 31) / 32), (unsigned)a.batch), block(256);
#define FGE_GG(InT, NarrowT)                                                                           \
    do {                                                                                               \
        if (dst_dtype != FGE_F32) hipLaunchKernelGGL((generic_gemm_kernel<InT, NarrowT>), grid, block, 0, s, a); \
        else                      hipLaunchKernelGGL((generic_gemm_kernel<InT, float>), grid, block, 0, s, a);   \
    } while (0)
    if (in_dtype == FGE_BF16)     FGE_GG(bf16_t, bf16_t);
    else if (in_dtype == FGE_F16) FGE_GG(f16_t, f16_t);
    else if (in_dtype == FGE_F8E4M3) FGE_GG(f8_t, bf16_t);
    else                          FGE_GG(float, bf16_t);
#undef FGE_GG
    return hipGetLastError();
}

hipError_t launch_generic_act(int dtype, hipStream_t s, const GenArgs &a) {
    const int64_t total = (int64_t)a.batch * a.M * a.N;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;                           // grid-stride beyond that
    const dim3 grid((unsigned)blocks), block(256);
    if (dtype == FGE_BF16)     hipLaunchKernelGGL((generic_act_kernel<bf16_t>), grid, block, 0, s, a);
    else if (dtype == FGE_F16) hipLaunchKernelGGL((generic_act_kernel<f16_t>), grid, block, 0, s, a);
    else                       hipLaunchKernelGGL((generic_act_kernel<float>), grid, block, 0, s, a);
    return hipGetLastError();
}

// src is fp32 (the fused intermediate) or of the output type (the unfused A)
hipError_t launch_generic_row(int src_dtype, int out_dtype, hipStream_t s, const GenArgs &a) {
    const int64_t rows = (int64_t)a.batch * a.M;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (src_dtype == FGE_F32 && a.X != a.dst && a.ldx % 4 == 0 && a.bsx % 4 == 0 && (reinterpret_cast<uintptr_t>(a.X) & 15) == 0 &&
        rows <= INT32_MAX) {
        // source rows on 16-byte boundaries: one workgroup per row; the row parked in LDS when it fits
        const dim3 g1((unsigned)rows);
        const size_t row_bytes = ((size_t)a.N * 4 + 15) / 16 * 16;
#define FGE_ROW(OT)                                                                                       \
        do {                                                                                               \
            if (row_bytes <= ((size_t)64 << 10) - 256)                                                     \
                hipLaunchKernelGGL((aligned_src_row_kernel<OT, true>), g1, block, row_bytes, s, a);        \
            else                                                                                           \
                hipLaunchKernelGGL((aligned_src_row_kernel<OT, false>), g1, block, 0, s, a);               \
        } while (0)
        if (out_dtype == FGE_BF16)     FGE_ROW(bf16_t);
        else if (out_dtype == FGE_F16) FGE_ROW(f16_t);
        else                           FGE_ROW(float);
#undef FGE_ROW
        return hipGetLastError();
    }
    if (src_dtype == FGE_F32) {
        if (out_dtype == FGE_BF16)     hipLaunchKernelGGL((generic_row_kernel<float, bf16_t>), grid, block, 0, s, a);
        else if (out_dtype == FGE_F16) hipLaunchKernelGGL((generic_row_kernel<float, f16_t>), grid, block, 0, s, a);
        else                           hipLaunchKernelGGL((generic_row_kernel<float, float>), grid, block, 0, s, a);
    } else if (src_dtype == out_dtype) {
        if (out_dtype == FGE_BF16) hipLaunchKernelGGL((generic_row_kernel<bf16_t, bf16_t>), grid, block, 0, s, a);
        else                       hipLaunchKernelGGL((generic_row_kernel<f16_t, f16_t>), grid, block, 0, s, a);
    } else {
        return hipErrorInvalidValue;                                     // never asked for
    }
    return hipGetLastError();
}

}  // namespace fge
