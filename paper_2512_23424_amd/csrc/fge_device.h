// Device-side building blocks shared by every kernel of the library (gfx950 only):
// storage-type conversion, the activations, and wavefront reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fge.h"

namespace fge {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

struct bf16_t { uint16_t bits; };   // storage only; arithmetic is always fp32
struct f16_t { uint16_t bits; };    // IEEE half, storage only
struct f8_t { uint8_t bits; };      // 8-bit E4M3 (bias 7, no infinities), operand storage only

__device__ __forceinline__ float as_f32(uint32_t v) { return __builtin_bit_cast(float, v); }
__device__ __forceinline__ uint32_t as_u32(float v) { return __builtin_bit_cast(uint32_t, v); }

// ---------------------------------------------------------------- asynchronous global -> LDS copy
// One 16-byte element per lane: lane l's data lands at lds_base + 16*l, lds_base being uniform
// over the wave.  Completion is tracked by the wave's vector-memory counter only; callers wait
// with lds_dma_wait() and then synchronise the workgroup before anyone reads the data.
// Written in assembly on purpose: for the builtin form the compiler assumes that every later
// LDS read may alias the copy and drains the vector-memory counter in front of it, which turns
// a prefetch into a synchronous load.  m0 is not used by any compiler-generated code of these
// kernels (no other LDS-direct, GWS or indexed-register instruction is emitted).  It cannot be
// declared as clobbered: the compiler treats m0 as a reserved register and rejects it on the
// clobber list with a warning that the entry has no effect.
// The global address is a wave-uniform 64-bit base (scalar registers) plus a 32-bit byte offset
// per lane, the LDS address a wave-uniform byte address: stepping along K and switching stage
// buffers is then scalar arithmetic only, and a lane keeps one register per copy instead of a
// 64-bit pointer.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    typedef __attribute__((address_space(3))) const void *lptr_t;
    return (uint32_t)(uintptr_t)(lptr_t)p;
}
// The instruction's immediate offset (here step * 1024, step = 0 .. 3) is added to the LDS address
// and to the global address alike (checked on the hardware), so up to four copies whose LDS
// destinations lie 1024 bytes apart share one value of the LDS base register: set_base says
// whether this copy writes it (the first copy of a run and of every group of four) or relies on
// the value the previous copy of its group left there.  Callers lower lane_off by step * 1024.
__device__ __forceinline__ void lds_dma16(const void *base, uint32_t lane_off, uint32_t lds_addr, int step, bool set_base) {
    if (set_base) asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" :: "s"(lds_addr) : "memory");
    switch (step) {
    case 0:  asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(lane_off), "s"(base) : "memory"); break;
    case 1:  asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" :: "v"(lane_off), "s"(base) : "memory"); break;
    case 2:  asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" :: "v"(lane_off), "s"(base) : "memory"); break;
    default: asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" :: "v"(lane_off), "s"(base) : "memory"); break;
    }
}
__device__ __forceinline__ void lds_dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---------------------------------------------------------------- storage conversion
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// fp32 -> bf16, round to nearest even (the hardware conversion of gfx950).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}
// two at once (one conversion instruction): lo in bits 0-15, hi in bits 16-31
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> struct Store;
template <> struct Store<float> {
    static constexpr int CW = 4;                       // elements per 16-byte chunk
    __device__ static __forceinline__ void put(float *p, float v) { *p = v; }
    __device__ static __forceinline__ float get(const float *p) { return *p; }
    // one 16-byte chunk <-> CW floats
    __device__ static __forceinline__ void unpack(const uint4 &u, float *v) {
        v[0] = as_f32(u.x); v[1] = as_f32(u.y); v[2] = as_f32(u.z); v[3] = as_f32(u.w);
    }
    __device__ static __forceinline__ uint4 pack(const float *v) {
        uint4 u;
        u.x = as_u32(v[0]); u.y = as_u32(v[1]); u.z = as_u32(v[2]); u.w = as_u32(v[3]);
        return u;
    }
};
template <> struct Store<bf16_t> {
    static constexpr int CW = 8;
    __device__ static __forceinline__ void put(bf16_t *p, float v) { p->bits = f32_to_bf16(v); }
    __device__ static __forceinline__ float get(const bf16_t *p) { return bf16_to_f32(p->bits); }
    __device__ static __forceinline__ void unpack(const uint4 &u, float *v) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i]     = as_f32(w[i] << 16);
            v[2 * i + 1] = as_f32(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ uint4 pack(const float *v) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

template <> struct Store<f16_t> {
    static constexpr int CW = 8;
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    // fp32 -> fp16 rounds to nearest even (the conversion instruction under the default mode)
    __device__ static __forceinline__ void put(f16_t *p, float v) {
        p->bits = __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));
    }
    __device__ static __forceinline__ float get(const f16_t *p) {
        return static_cast<float>(__builtin_bit_cast(_Float16, p->bits));
    }
    __device__ static __forceinline__ void unpack(const uint4 &u, float *v) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x2_t f = __builtin_convertvector(__builtin_bit_cast(f16x2_t, w[i]), f32x2_t);
            v[2 * i] = f[0];
            v[2 * i + 1] = f[1];
        }
    }
    __device__ static __forceinline__ uint4 pack(const float *v) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x2_t f = {v[2 * i], v[2 * i + 1]};
            w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2_t));
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// Operands only: nothing is ever stored in this type.
template <> struct Store<f8_t> {
    static constexpr int CW = 16;
    __device__ static __forceinline__ float get(const f8_t *p) {
        return __builtin_amdgcn_cvt_f32_fp8((int)p->bits, 0);
    }
};

// ---------------------------------------------------------------- activations (fp32)
// exp and reciprocal use the hardware transcendental units (about 1 ulp each); the forms
// below avoid cancellation so the relative error stays near 1e-6 for every input.
__device__ __forceinline__ float fast_exp(float x) { return __expf(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
constexpr float LOG2E = 1.4426950408889634f;
// exp(x - m) as one multiply-add and one exponential: c = -m * LOG2E is formed once per row
__device__ __forceinline__ float exp_rel(float x, float c) { return __builtin_amdgcn_exp2f(fmaf(x, LOG2E, c)); }
// max / clamp as single median-of-three instructions (the compiler wraps fmaxf / fminf of
// values it cannot prove canonical - anything that came through LDS or a select - in an extra
// canonicalising instruction each)
__device__ __forceinline__ float max_nc(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, __builtin_inff()); }
__device__ __forceinline__ float clamp_nc(float y, float lo, float hi) { return __builtin_amdgcn_fmed3f(y, lo, hi); }

template <int ACT> __device__ __forceinline__ float activate(float y, float lo, float hi) {
    if constexpr (ACT == FGE_ACT_RELU) {
        return fmaxf(y, 0.0f);
    } else if constexpr (ACT == FGE_ACT_GELU_TANH) {
        // 0.5 y (1 + tanh u) == y * sigmoid(2u),  u = sqrt(2/pi) (y + 0.044715 y^3)
        // (exp(-2u) as one exp2: the factor below is -2 sqrt(2/pi) log2(e))
        const float w = -2.302208198144325f * (y + 0.044715f * y * y * y);
        return y * fast_rcp(1.0f + __builtin_amdgcn_exp2f(w));
    } else if constexpr (ACT == FGE_ACT_GELU_ERF) {
        // 0.5 y (1 + erf(y/sqrt2)) = y * Phi(y).  erfc(|x|) by the rational approximation 7.1.26
        // of Abramowitz & Stegun (|error| <= 1.5e-7 on erf):  erfc(|x|) = poly(t) exp(-x^2),
        // t = 1/(1 + p|x|), x = y/sqrt2.  With h = 0.5 erfc(|x|):  Phi(y) = h for y < 0 and
        // 1 - h otherwise, so  y Phi(y) = max(y, 0) - |y| h  in both cases, the negative tail
        // without cancellation.  The constants carry the scalings: u = y sqrt(0.5 log2 e), so that
        // exp(-x^2) = exp2(-u^2) and p|x| = P|u|; the polynomial's coefficients are halved.
        const float u = 0.8493218002880191f * y;                          // sqrt(0.5 * log2(e)) * y
        const float t = fast_rcp(fmaf(0.2727374809f, fabsf(u), 1.0f));    // P = p / sqrt(log2(e))
        float q = 0.5307027145f;
        q = q * t - 0.7265760135f;
        q = q * t + 0.7107068705f;
        q = q * t - 0.142248368f;
        q = q * t + 0.127414796f;
        const float h = q * t * __builtin_amdgcn_exp2f(-u * u);
        return fmaf(-fabsf(y), h, fmaxf(y, 0.0f));
    } else if constexpr (ACT == FGE_ACT_SILU) {
        return y * fast_rcp(1.0f + fast_exp(-y));
    } else if constexpr (ACT == FGE_ACT_CLAMP) {
        return clamp_nc(y, lo, hi);                // the host passes lo <= hi
    } else {
        return y;
    }
}

// Calls f.template operator()<ACT>() with the runtime activation code turned into a constant,
// so the per-element loop inside f carries no branch.
template <typename F> __device__ __forceinline__ void dispatch_act(int act, F &&f) {
    switch (act) {
    case FGE_ACT_RELU:      f.template operator()<FGE_ACT_RELU>(); break;
    case FGE_ACT_GELU_TANH: f.template operator()<FGE_ACT_GELU_TANH>(); break;
    case FGE_ACT_GELU_ERF:  f.template operator()<FGE_ACT_GELU_ERF>(); break;
    case FGE_ACT_SILU:      f.template operator()<FGE_ACT_SILU>(); break;
    case FGE_ACT_CLAMP:     f.template operator()<FGE_ACT_CLAMP>(); break;
    default:                f.template operator()<FGE_ACT_NONE>(); break;
    }
}

// Compile-time loop: f.template operator()<I>() for I in [I0, N).  Used where an unrolled
// runtime loop would leave register arrays indexed by a variable.
template <int I0, int N, typename F> __device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I0 < N) {
        f.template operator()<I0>();
        static_for<I0 + 1, N>(f);
    }
}

// ---------------------------------------------------------------- wavefront reductions
struct OpSum { __device__ static __forceinline__ float f(float a, float b) { return a + b; }
               static constexpr float ident() { return 0.0f; } };
struct OpMax { __device__ static __forceinline__ float f(float a, float b) { return max_nc(a, b); }
               static constexpr float ident() { return -__builtin_inff(); } };

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// All-reduce over groups of G neighbouring lanes (G a power of two, groups aligned to G).
// Steps: quad swaps (xor 1, xor 2), mirror within 8, mirror within 16 - valid because after
// each step the value is uniform inside the smaller group -, a swizzle exchanging lanes i and
// i^16, and a shuffle across the two halves of the wave.
template <typename Op, int G> __device__ __forceinline__ float allreduce_lanes(float v) {
    if constexpr (G >= 2)  v = Op::f(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    if constexpr (G >= 4)  v = Op::f(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    if constexpr (G >= 8)  v = Op::f(v, dpp_mov<0x141>(v));   // row_half_mirror
    if constexpr (G >= 16) v = Op::f(v, dpp_mov<0x140>(v));   // row_mirror
    if constexpr (G >= 32) v = Op::f(v, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(
                                            __builtin_bit_cast(int, v), 0x401F)));   // and 0x1f, xor 0x10
    if constexpr (G >= 64) v = Op::f(v, __shfl_xor(v, 32, 64));
    return v;
}
template <typename Op> __device__ __forceinline__ float allreduce32(float v) { return allreduce_lanes<Op, 32>(v); }

// All-reduce over the whole 64-lane wavefront.
template <typename Op> __device__ __forceinline__ float allreduce64(float v) { return allreduce_lanes<Op, 64>(v); }

}  // namespace fge
