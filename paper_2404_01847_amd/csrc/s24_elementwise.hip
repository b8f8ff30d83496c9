// HBM-bound elementwise kernels: masked decay on gradients (Eq. 10), the gated
// activation SwiGLU forward/backward (Sec. 5.2) and the ungated ReLU / GELU.
// Every lane moves eight consecutive elements per tensor with 16-byte
// accesses; arithmetic is fp32, storage bf16 or fp32.
#include "s24_common.h"

namespace {

constexpr int kThreads = 256;

template <typename T> struct Vec8;

template <> struct Vec8<uint16_t> {  // bf16
    static __device__ __forceinline__ void load(const uint16_t *p, float (&x)[8])
    {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[2 * k] = __uint_as_float(d[k] << 16);
            x[2 * k + 1] = __uint_as_float(d[k] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void store(uint16_t *p, const float (&x)[8])
    {
        uint4 v;
        v.x = s24_pack_bf16x2(x[0], x[1]);
        v.y = s24_pack_bf16x2(x[2], x[3]);
        v.z = s24_pack_bf16x2(x[4], x[5]);
        v.w = s24_pack_bf16x2(x[6], x[7]);
        *reinterpret_cast<uint4 *>(p) = v;
    }
};

template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float *p, float (&x)[8])
    {
        const float4 a = reinterpret_cast<const float4 *>(p)[0], b = reinterpret_cast<const float4 *>(p)[1];
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&x)[8])
    {
        reinterpret_cast<float4 *>(p)[0] = make_float4(x[0], x[1], x[2], x[3]);
        reinterpret_cast<float4 *>(p)[1] = make_float4(x[4], x[5], x[6], x[7]);
    }
};


// ---- masked decay: G += lambda * W where the mask prunes -------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void masked_decay_kernel(float *__restrict__ G, const T *__restrict__ W,
                                                                const uint16_t *__restrict__ mask, float lambda,
                                                                int64_t n8, int q8, int bq)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    const int64_t row = idx / q8;
    const int c8 = (int)(idx - row * q8);
    float g[8], w[8];
    Vec8<float>::load(G + idx * 8, g);
    Vec8<T>::load(W + idx * 8, w);
    // two neighbouring block masks; this row's four bits of each
    const uint32_t mm = *reinterpret_cast<const uint32_t *>(mask + (row >> 2) * bq + 2 * c8);
    const int sh = 4 * (int)(row & 3);
    const uint32_t bits = ((mm >> sh) & 0xFu) | (((mm >> (16 + sh)) & 0xFu) << 4);
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (!((bits >> k) & 1u)) g[k] = fmaf(lambda, w[k], g[k]);
    Vec8<float>::store(G + idx * 8, g);
}

// ---- SwiGLU ------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void swiglu_fwd_kernel(const T *__restrict__ G, const T *__restrict__ U,
                                                              T *__restrict__ H, int64_t n8, int f8, int64_t ld)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    const int64_t row = idx / f8;
    const int64_t in_off = row * ld + (idx - row * f8) * 8;
    float g[8], u[8], h[8];
    Vec8<T>::load(G + in_off, g);
    Vec8<T>::load(U + in_off, u);
#pragma unroll
    for (int k = 0; k < 8; ++k) h[k] = s24_silu_mul(g[k], u[k]);
    Vec8<T>::store(H + idx * 8, h);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void swiglu_bwd_kernel(const T *__restrict__ dH, const T *__restrict__ G,
                                                              const T *__restrict__ U, T *__restrict__ dG,
                                                              T *__restrict__ dU, int64_t n8, int f8, int64_t ld)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    const int64_t row = idx / f8;
    const int64_t off = row * ld + (idx - row * f8) * 8;
    float d[8], g[8], u[8], dg[8], du[8];
    Vec8<T>::load(dH + idx * 8, d);
    Vec8<T>::load(G + off, g);
    Vec8<T>::load(U + off, u);
#pragma unroll
    for (int k = 0; k < 8; ++k) s24_swiglu_grad(d[k], g[k], u[k], dg[k], du[k]);
    Vec8<T>::store(dG + off, dg);
    Vec8<T>::store(dU + off, du);
}

// ---- ReLU / GELU(erf) ----------------------------------------------------------
template <typename T, int ACT>
__global__ __launch_bounds__(kThreads) void act_fwd_kernel(const T *__restrict__ Z, T *__restrict__ H, int64_t n8)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    float z[8], h[8];
    Vec8<T>::load(Z + idx * 8, z);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (ACT == S24_ACT_RELU) h[k] = z[k] > 0.0f ? z[k] : 0.0f;
        else h[k] = 0.5f * z[k] * (1.0f + erff(z[k] * 0.70710678118654752f));
    }
    Vec8<T>::store(H + idx * 8, h);
}

template <typename T, int ACT>
__global__ __launch_bounds__(kThreads) void act_bwd_kernel(const T *__restrict__ dH, const T *__restrict__ Z,
                                                           T *__restrict__ dZ, int64_t n8)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    float d[8], z[8], o[8];
    Vec8<T>::load(dH + idx * 8, d);
    Vec8<T>::load(Z + idx * 8, z);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float dz;
        if (ACT == S24_ACT_RELU) dz = z[k] > 0.0f ? 1.0f : 0.0f;
        else
            dz = 0.5f * (1.0f + erff(z[k] * 0.70710678118654752f)) +
                 z[k] * 0.39894228040143268f * expf(-0.5f * z[k] * z[k]);
        o[k] = d[k] * dz;
    }
    Vec8<T>::store(dZ + idx * 8, o);
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }
constexpr int64_t kMaxThreads = (int64_t)0x7FFFFFFF * kThreads;

}  // namespace

extern "C" int s24_masked_decay_grad(float *G, const void *W, s24_dtype wdt, const uint16_t *mask, float lambda,
                                     int64_t r, int64_t q, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(wdt), S24_ERR_DTYPE);
    S24_REQUIRE(r >= 0 && q >= 0 && r % 4 == 0 && q % 16 == 0, S24_ERR_SHAPE);
    if (r == 0 || q == 0) return S24_OK;
    S24_REQUIRE(G && W && mask, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(G, 16) && s24_aligned(W, 16) && s24_aligned(mask, 4), S24_ERR_ALIGN);
    const int64_t n8 = r * q / 8;
    S24_REQUIRE(n8 <= kMaxThreads && q / 8 < (1ll << 31), S24_ERR_SHAPE);
    if (n8 == 0) return S24_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (wdt == S24_BF16)
        hipLaunchKernelGGL(masked_decay_kernel<uint16_t>, dim3(blocks_for(n8)), dim3(kThreads), 0, st, G,
                           static_cast<const uint16_t *>(W), mask, lambda, n8, (int)(q / 8), (int)(q / 4));
    else
        hipLaunchKernelGGL(masked_decay_kernel<float>, dim3(blocks_for(n8)), dim3(kThreads), 0, st, G,
                           static_cast<const float *>(W), mask, lambda, n8, (int)(q / 8), (int)(q / 4));
    return s24_launch_status();
}

static int check_gated(const void *a, const void *b, const void *c, int64_t p, int64_t f, int64_t ld, int dt)
{
    S24_REQUIRE(s24_valid_dtype(dt), S24_ERR_DTYPE);
    S24_REQUIRE(p >= 0 && f >= 0 && f % 8 == 0 && ld % 8 == 0 && ld >= f, S24_ERR_SHAPE);
    S24_REQUIRE(p * f / 8 <= kMaxThreads && f / 8 < (1ll << 31), S24_ERR_SHAPE);
    if (p * f == 0) return S24_OK;
    S24_REQUIRE(a && b && c, S24_ERR_NULL);
    return S24_OK;
}

extern "C" int s24_swiglu_fwd(const void *G, const void *U, void *H, int64_t p, int64_t f, int64_t ld_gu, s24_dtype dt,
                              void *stream)
{
    const int rc = check_gated(G, U, H, p, f, ld_gu, dt);
    if (rc != S24_OK || p * f == 0) return rc;
    S24_REQUIRE(s24_aligned(G, 16) && s24_aligned(U, 16) && s24_aligned(H, 16), S24_ERR_ALIGN);
    const int64_t n8 = p * f / 8;
    if (n8 == 0) return S24_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == S24_BF16)
        hipLaunchKernelGGL(swiglu_fwd_kernel<uint16_t>, dim3(blocks_for(n8)), dim3(kThreads), 0, st,
                           static_cast<const uint16_t *>(G), static_cast<const uint16_t *>(U), static_cast<uint16_t *>(H),
                           n8, (int)(f / 8), ld_gu);
    else
        hipLaunchKernelGGL(swiglu_fwd_kernel<float>, dim3(blocks_for(n8)), dim3(kThreads), 0, st,
                           static_cast<const float *>(G), static_cast<const float *>(U), static_cast<float *>(H), n8,
                           (int)(f / 8), ld_gu);
    return s24_launch_status();
}

extern "C" int s24_swiglu_bwd(const void *dH, const void *G, const void *U, void *dG, void *dU, int64_t p, int64_t f,
                              int64_t ld_gu, s24_dtype dt, void *stream)
{
    const int rc = check_gated(dH, G, U, p, f, ld_gu, dt);
    if (rc != S24_OK || p * f == 0) return rc;
    S24_REQUIRE(dG && dU, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dH, 16) && s24_aligned(G, 16) && s24_aligned(U, 16) && s24_aligned(dG, 16) &&
                    s24_aligned(dU, 16),
                S24_ERR_ALIGN);
    const int64_t n8 = p * f / 8;
    if (n8 == 0) return S24_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == S24_BF16)
        hipLaunchKernelGGL(swiglu_bwd_kernel<uint16_t>, dim3(blocks_for(n8)), dim3(kThreads), 0, st,
                           static_cast<const uint16_t *>(dH), static_cast<const uint16_t *>(G),
                           static_cast<const uint16_t *>(U), static_cast<uint16_t *>(dG), static_cast<uint16_t *>(dU), n8,
                           (int)(f / 8), ld_gu);
    else
        hipLaunchKernelGGL(swiglu_bwd_kernel<float>, dim3(blocks_for(n8)), dim3(kThreads), 0, st,
                           static_cast<const float *>(dH), static_cast<const float *>(G), static_cast<const float *>(U),
                           static_cast<float *>(dG), static_cast<float *>(dU), n8, (int)(f / 8), ld_gu);
    return s24_launch_status();
}

template <typename T>
static int launch_act(const void *a, const void *b, void *c, int64_t n8, int act, bool bwd, hipStream_t st)
{
    const dim3 grid(blocks_for(n8)), block(kThreads);
    const T *pa = static_cast<const T *>(a), *pb = static_cast<const T *>(b);
    T *pc = static_cast<T *>(c);
    if (!bwd) {
        if (act == S24_ACT_RELU) hipLaunchKernelGGL((act_fwd_kernel<T, S24_ACT_RELU>), grid, block, 0, st, pa, pc, n8);
        else hipLaunchKernelGGL((act_fwd_kernel<T, S24_ACT_GELU_ERF>), grid, block, 0, st, pa, pc, n8);
    } else {
        if (act == S24_ACT_RELU) hipLaunchKernelGGL((act_bwd_kernel<T, S24_ACT_RELU>), grid, block, 0, st, pa, pb, pc, n8);
        else hipLaunchKernelGGL((act_bwd_kernel<T, S24_ACT_GELU_ERF>), grid, block, 0, st, pa, pb, pc, n8);
    }
    return s24_launch_status();
}

extern "C" int s24_act_fwd(const void *Z, void *H, int64_t n, s24_act act, s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(dt) && (act == S24_ACT_RELU || act == S24_ACT_GELU_ERF), S24_ERR_DTYPE);
    S24_REQUIRE(n >= 0 && n % 8 == 0 && n / 8 <= kMaxThreads, S24_ERR_SHAPE);
    if (n == 0) return S24_OK;
    S24_REQUIRE(Z && H, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(Z, 16) && s24_aligned(H, 16), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dt == S24_BF16 ? launch_act<uint16_t>(Z, nullptr, H, n / 8, act, false, st)
                          : launch_act<float>(Z, nullptr, H, n / 8, act, false, st);
}

extern "C" int s24_act_bwd(const void *dH, const void *Z, void *dZ, int64_t n, s24_act act, s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(dt) && (act == S24_ACT_RELU || act == S24_ACT_GELU_ERF), S24_ERR_DTYPE);
    S24_REQUIRE(n >= 0 && n % 8 == 0 && n / 8 <= kMaxThreads, S24_ERR_SHAPE);
    if (n == 0) return S24_OK;
    S24_REQUIRE(dH && Z && dZ, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dH, 16) && s24_aligned(Z, 16) && s24_aligned(dZ, 16), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dt == S24_BF16 ? launch_act<uint16_t>(dH, Z, dZ, n / 8, act, true, st)
                          : launch_act<float>(dH, Z, dZ, n / 8, act, true, st);
}
