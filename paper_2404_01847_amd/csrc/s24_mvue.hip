// Unbiased 2:4 pruning of the output gradient for a sparse weight-gradient GEMM
// (Eq. 4: grad W = S_z(grad Z^T) X with S_z the minimum-variance unbiased estimator, Eq. 6).
//
// The paper names the estimator without spelling it out.  Built here from its definition: of every four
// consecutive tokens of one feature two are kept, element j with probability pi_j and stored as a_j / pi_j
// (unbiased); sum_j a_j^2 / pi_j under sum pi = 2, pi <= 1 is least for pi_j proportional to |a_j|, capped
// at one.  Without a cap (2 max|a| <= S = sum |a|) a kept element becomes sign(a_j) S / 2; with a cap the
// largest element is always kept as it is and one of the others, with probability |a_j| / R (R = S - max|a|,
// their sum), becomes sign(a_j) R.  The pair is drawn by systematic sampling with one uniform number u per group, taken
// from a counter-based integer hash of (seed, feature, token group).  Every decision is an fp32 operation
// written with explicit round-to-nearest intrinsics in a fixed order, so the result is a pure function of the
// inputs and the seed, reproducible bit for bit by any implementation that follows the same order.
#include "s24_common.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

struct Kept { int i0, i1; float v0, v1; };

__device__ __forceinline__ Kept mvue_group(const float (&a)[4], uint32_t bits)
{
    float m[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) m[i] = fabsf(a[i]);
    const float S = __fadd_rn(__fadd_rn(m[0], m[1]), __fadd_rn(m[2], m[3]));
    const float mx = fmaxf(fmaxf(m[0], m[1]), fmaxf(m[2], m[3]));
    const bool capped = __fmul_rn(2.0f, mx) > S;   // then mx exceeds the other three together: it is unique
    const float R = __fsub_rn(S, mx);              // the others' sum, as fp32 gives it
    const float D = capped ? R : S, scale = capped ? 1.0f : 2.0f;
    const float inv = D > 0.0f ? __fdiv_rn(1.0f, D) : 0.0f;
    const float common = capped ? R : __fmul_rn(0.5f, S);
    float pi[4], val[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool top = capped && m[i] == mx;
        pi[i] = top ? 1.0f : fminf(__fmul_rn(__fmul_rn(scale, m[i]), inv), 1.0f);
        val[i] = m[i] == 0.0f ? 0.0f : copysignf(top ? m[i] : common, a[i]);
    }
    const float c1 = pi[0], c2 = __fadd_rn(c1, pi[1]), c3 = __fadd_rn(c2, pi[2]);
    const float u = __fmul_rn((float)bits, 0x1p-23f), v = __fadd_rn(u, 1.0f);
    int i0 = (u >= c1) + (u >= c2) + (u >= c3);
    int i1 = (v >= c1) + (v >= c2) + (v >= c3);
    if (i1 == i0) {   // only on rounding knife edges and in groups with fewer than two non-zeros
        if (i0 < 3) i1 = i0 + 1;
        else { i0 = 2; i1 = 3; }
    }
    auto pick = [&](int j) { return j == 0 ? val[0] : (j == 1 ? val[1] : (j == 2 ? val[2] : val[3])); };
    return {i0, i1, pick(i0), pick(i1)};
}

template <typename T> struct Elem;
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t *p) { return s24_bf16_to_f32(*p); }
};
template <> struct Elem<s24_half> {
    static __device__ __forceinline__ float load(const s24_half *p) { return (float)*p; }
};
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
};

// One lane = one feature of one 64-token chunk: 16 groups, 32 kept values (64 or 128 bytes, contiguous in
// the chunk-major operand) and four metadata words.  Lanes of a wave are consecutive features, so every row
// read and every store is one contiguous run; the four waves of a workgroup take four consecutive chunks.
template <typename T>
__global__ __launch_bounds__(kThreads) void mvue24_kernel(const T *__restrict__ dY, int64_t ld, int r, int chunks,
                                                          uint32_t seed, T *__restrict__ vals, uint16_t *__restrict__ meta)
{
    const int lane = threadIdx.x & 63;
    const int f = (int)blockIdx.x * 64 + lane;
    const int c = (int)blockIdx.y * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    if (c >= chunks) return;
    // wave-uniform row pointers plus the lane's column: no per-load address arithmetic; lanes past the last
    // feature re-read the last one and store nothing
    const T *src = dY + (int64_t)c * 64 * ld + (int)blockIdx.x * 64;
    const uint32_t row_bytes = (uint32_t)ld * (uint32_t)sizeof(T);   // 63 rows stay below 4 GB (checked on the host)
    const uint32_t col_bytes = (uint32_t)min(lane, r - 1 - (int)blockIdx.x * 64) * (uint32_t)sizeof(T);
    float out[32];
    uint32_t words[2] = {0u, 0u};
    // counter-based draw: the seed is hashed alone, then with the feature (the lane's key), then with the token
    // group, so that consecutive seeds -- one per step and operand -- give unrelated streams
    const uint32_t key = mix32(mix32(seed) + (uint32_t)f * 0x9E3779B9U);
#pragma unroll
    for (int g = 0; g < 16; ++g) {
        float a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = Elem<T>::load(reinterpret_cast<const T *>(reinterpret_cast<const char *>(src) + (col_bytes + (uint32_t)(4 * g + i) * row_bytes)));
        const uint32_t bits = mix32(key + (uint32_t)(16 * c + g) * 0x85EBCA6BU) >> 9;
        const Kept k = mvue_group(a, bits);
        out[2 * g] = k.v0;
        out[2 * g + 1] = k.v1;
        words[g >> 3] |= (uint32_t)(k.i0 | (k.i1 << 2)) << (4 * (g & 7));
    }
    if (f >= r) return;
    const int64_t o = (int64_t)c * r + f;
    if constexpr (sizeof(T) == 2) {
        uint4 *dst = reinterpret_cast<uint4 *>(vals + o * 32);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            dst[k] = make_uint4(s24_num<T>::pack2(out[8 * k], out[8 * k + 1]), s24_num<T>::pack2(out[8 * k + 2], out[8 * k + 3]),
                                s24_num<T>::pack2(out[8 * k + 4], out[8 * k + 5]), s24_num<T>::pack2(out[8 * k + 6], out[8 * k + 7]));
    } else {
        float4 *dst = reinterpret_cast<float4 *>(vals + o * 32);
#pragma unroll
        for (int k = 0; k < 8; ++k) dst[k] = make_float4(out[4 * k], out[4 * k + 1], out[4 * k + 2], out[4 * k + 3]);
    }
    *reinterpret_cast<uint2 *>(meta + o * 4) = make_uint2(words[0], words[1]);
}

}  // namespace

extern "C" int s24_mvue24(const void *dY, s24_dtype dt, int64_t p, int64_t r, int64_t ld, uint32_t seed, void *vals,
                          uint16_t *meta, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(dt), S24_ERR_DTYPE);
    S24_REQUIRE(p >= 0 && r >= 0 && p % 64 == 0 && ld >= r, S24_ERR_SHAPE);
    S24_REQUIRE(p < (1ll << 31) && r < (1ll << 31) && p / 256 + 1 <= 65535 && ld < (1ll << 24), S24_ERR_SHAPE);
    if (p == 0 || r == 0) return S24_OK;
    S24_REQUIRE(dY && vals && meta, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dY, s24_elem_size(dt)) && s24_aligned(vals, 16) && s24_aligned(meta, 8), S24_ERR_ALIGN);
    const int chunks = (int)(p / 64);
    const dim3 grid((unsigned)((r + 63) / 64), (unsigned)((chunks + 3) / 4)), block(kThreads);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == S24_BF16)
        hipLaunchKernelGGL(mvue24_kernel<uint16_t>, grid, block, 0, st, static_cast<const uint16_t *>(dY), ld, (int)r, chunks,
                           seed, static_cast<uint16_t *>(vals), meta);
    else if (dt == S24_F16)
        hipLaunchKernelGGL(mvue24_kernel<s24_half>, grid, block, 0, st, static_cast<const s24_half *>(dY), ld, (int)r, chunks,
                           seed, static_cast<s24_half *>(vals), meta);
    else
        hipLaunchKernelGGL(mvue24_kernel<float>, grid, block, 0, st, static_cast<const float *>(dY), ld, (int)r, chunks, seed,
                           static_cast<float *>(vals), meta);
    return s24_launch_status();
}
