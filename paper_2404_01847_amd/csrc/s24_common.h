// Shared host/device helpers of the s24 library (argument checks, launch
// plumbing, bf16 / binary16 conversions, the activation arithmetic).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "s24.h"

#define S24_REQUIRE(cond, code) \
    do {                        \
        if (!(cond)) return (code); \
    } while (0)

static inline bool s24_aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline bool s24_valid_dtype(int dt) { return dt == S24_F32 || dt == S24_BF16 || dt == S24_F16; }
static inline bool s24_valid_gate(int g) { return g == S24_GATE_SILU || g == S24_GATE_GELU_ERF; }
static inline bool s24_valid_layout(int l) { return l == S24_ROW_MAJOR || l == S24_COL_MAJOR; }
static inline size_t s24_elem_size(int dt) { return dt == S24_F32 ? 4 : 2; }

// Call after a kernel launch: turns a refused launch into S24_ERR_LAUNCH.
static inline int s24_launch_status() { return hipGetLastError() == hipSuccess ? S24_OK : S24_ERR_LAUNCH; }

__device__ __forceinline__ float s24_bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Two fp32 values -> two bf16 in one dword (lo in bits 0..15), round to nearest even: gfx950's packed conversion,
// one instruction where the integer form (add the rounding bias, shift, merge) takes seven.  Written as the
// instruction itself so that every kernel rounds the same fp32 value to the same bits.
__device__ __forceinline__ uint32_t s24_pack_bf16x2(float lo, float hi)
{
    uint32_t d = 0;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(d) : "v"(lo), "v"(hi));
#endif
    return d;
}

// fp32 -> bf16 bits, round to nearest even.
__device__ __forceinline__ uint32_t s24_f32_to_bf16(float f) { return s24_pack_bf16x2(f, f) & 0xFFFFu; }

// Storage types of the kernels: uint16_t holds bf16 bits, s24_half is IEEE binary16, float is itself.
// s24_num<T> converts between 16-bit storage and the fp32 the arithmetic runs in: one value from its 16 bits,
// the low / high half of a dword, and back (round to nearest even; binary16 overflows to infinity).
typedef _Float16 s24_half;
template <typename T> struct s24_num;
template <> struct s24_num<uint16_t> {
    static __device__ __forceinline__ float widen(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
    static __device__ __forceinline__ float lo(uint32_t d) { return __uint_as_float(d << 16); }
    static __device__ __forceinline__ float hi(uint32_t d) { return __uint_as_float(d & 0xFFFF0000u); }
    static __device__ __forceinline__ uint32_t narrow(float f) { return s24_f32_to_bf16(f); }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) { return s24_pack_bf16x2(a, b); }
};
template <> struct s24_num<s24_half> {
    static __device__ __forceinline__ float widen(uint32_t bits16)
    {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
    }
    static __device__ __forceinline__ float lo(uint32_t d) { return widen(d & 0xFFFFu); }
    static __device__ __forceinline__ float hi(uint32_t d) { return widen(d >> 16); }
    // The conversion is pinned to the one instruction that rounds an fp32 value to binary16.  Written as a C++
    // cast the compiler merges it with the multiplication before it into a mixed-precision instruction in some
    // kernels and not in others, and the two do not always agree in the last bit; with the instruction fixed,
    // every kernel that forms the same fp32 value stores the same bits.
    static __device__ __forceinline__ uint32_t narrow(float f)
    {
        uint32_t h = 0;
#if defined(__HIP_DEVICE_COMPILE__)
        asm("v_cvt_f16_f32 %0, %1" : "=v"(h) : "v"(f));
#endif
        return h & 0xFFFFu;
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) { return narrow(a) | (narrow(b) << 16); }
};

// silu(g) * u in fp32, shared by the stand-alone SwiGLU kernel and the GEMM epilogue that applies it
// 1 / (1 + 2^(-x log2 e)) with the hardware exponential and reciprocal (about 2 ulp in fp32, far inside what the
// bf16 or fp32 outputs of the activation kernels need; saturates to 0 and 1 for large |x|)
__device__ __forceinline__ float s24_sigmoid(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * x));
}
__device__ __forceinline__ float s24_silu_mul(float g, float u) { return g * s24_sigmoid(g) * u; }

// backward of h = silu(g) * u for an incoming dh: dg = dh u s (1 + g (1 - s)), du = dh silu(g), s = sigmoid(g)
__device__ __forceinline__ void s24_swiglu_grad(float dh, float g, float u, float &dg, float &du)
{
    const float s = s24_sigmoid(g);
    const float gs = g * s;
    dg = dh * u * (s + gs * (1.0f - s));
    du = dh * gs;
}

// Normal CDF Phi(x) and e = exp(-x^2/2), for GELU(x) = x Phi(x) (the erf form: Phi(x) = (1 + erf(x / sqrt 2)) / 2) and
// its slope Phi(x) + x e / sqrt(2 pi).  The lower tail is Phi(-s) = e * Q(t), t = 1 / (1 + 0.375 s), with Q(t) = t * (a
// degree-8 polynomial) fitted to the exact function (tests/fit_normal_cdf.py derives the constants, and
// tests/test_gelu_constants.py checks the ones below against math.erf on the CPU): one hardware exp2, one hardware
// reciprocal and nine fused multiply-adds, no branch, shared by the value and the slope.  In fp32: |error| < 4e-7 for
// Phi and GELU', < 4e-7 max(1, |x|) for GELU, and the lower tail keeps a relative accuracy of a few 1e-6 because the
// exponential is a factor, not a term.  The library routines (erff plus expf, both with range
// reduction and two code paths that a wave walks one after the other) cost about three times as much, which
// matters where this runs in a GEMM epilogue with nothing to hide behind.
__device__ __forceinline__ void s24_normal(float x, float &cdf, float &e)
{
    const float t = __builtin_amdgcn_rcpf(fmaf(0.375f, fabsf(x), 1.0f));
    float q = -3.291070461e-02f;
    q = fmaf(q, t, 1.368783563e-01f);
    q = fmaf(q, t, -1.865182221e-01f);
    q = fmaf(q, t, 5.062932521e-02f);
    q = fmaf(q, t, 1.562976278e-02f);
    q = fmaf(q, t, 8.863758296e-02f);
    q = fmaf(q, t, 1.284458190e-01f);
    q = fmaf(q, t, 1.496045738e-01f);
    q = fmaf(q, t, 1.496033818e-01f);
    e = __builtin_amdgcn_exp2f(-0.72134752f * x * x);
    const float tail = e * (q * t);
    cdf = x < 0.0f ? tail : 1.0f - tail;
}
// shared by the ungated activation kernels, the gated stand-alone kernels and the GEMM epilogues
__device__ __forceinline__ float s24_gelu(float x)
{
    float cdf, e;
    s24_normal(x, cdf, e);
    return x * cdf;
}
__device__ __forceinline__ float s24_gelu_slope(float x)
{
    float cdf, e;
    s24_normal(x, cdf, e);
    return fmaf(x, e * 0.3989422804f, cdf);
}

// Gated activation h = act(g) * u with act chosen at compile time (GATE: 0 = SiLU, 1 = GELU), and its backward
template <int GATE> __device__ __forceinline__ float s24_glu(float g, float u)
{
    if (GATE == S24_GATE_SILU) return s24_silu_mul(g, u);
    return s24_gelu(g) * u;
}
template <int GATE> __device__ __forceinline__ void s24_glu_grad(float dh, float g, float u, float &dg, float &du)
{
    if (GATE == S24_GATE_SILU) {
        s24_swiglu_grad(dh, g, u, dg, du);
    } else {
        float cdf, e;
        s24_normal(g, cdf, e);
        dg = dh * u * fmaf(g, e * 0.3989422804f, cdf);
        du = dh * (g * cdf);
    }
}
