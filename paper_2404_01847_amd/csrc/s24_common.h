// Shared host/device helpers of the s24 library (argument checks, launch
// plumbing, bf16 conversions).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "s24.h"

#define S24_REQUIRE(cond, code) \
    do {                        \
        if (!(cond)) return (code); \
    } while (0)

static inline bool s24_aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline bool s24_valid_dtype(int dt) { return dt == S24_F32 || dt == S24_BF16; }
static inline size_t s24_elem_size(int dt) { return dt == S24_F32 ? 4 : 2; }

// Call after a kernel launch: turns a refused launch into S24_ERR_LAUNCH.
static inline int s24_launch_status() { return hipGetLastError() == hipSuccess ? S24_OK : S24_ERR_LAUNCH; }

__device__ __forceinline__ float s24_bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// fp32 -> bf16, round to nearest even (inputs are finite).
__device__ __forceinline__ uint32_t s24_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ uint32_t s24_pack_bf16x2(float lo, float hi)
{
    return s24_f32_to_bf16(lo) | (s24_f32_to_bf16(hi) << 16);
}

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
