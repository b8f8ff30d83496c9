// HBM-bound elementwise kernels: masked decay on gradients (Eq. 10), the gated
// activations SwiGLU / GEGLU forward and backward on row- or column-major
// operands (Sec. 5.2 step 3), the bias gradient of step 2, and the ungated
// ReLU / GELU.  Every lane moves eight consecutive elements per tensor with
// 16-byte accesses; arithmetic is fp32, storage bf16, binary16 or fp32.
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

template <> struct Vec8<s24_half> {
    static __device__ __forceinline__ void load(const s24_half *p, float (&x)[8])
    {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[2 * k] = s24_num<s24_half>::lo(d[k]);
            x[2 * k + 1] = s24_num<s24_half>::hi(d[k]);
        }
    }
    static __device__ __forceinline__ void store(s24_half *p, const float (&x)[8])
    {
        uint4 v;
        v.x = s24_num<s24_half>::pack2(x[0], x[1]);
        v.y = s24_num<s24_half>::pack2(x[2], x[3]);
        v.z = s24_num<s24_half>::pack2(x[4], x[5]);
        v.w = s24_num<s24_half>::pack2(x[6], x[7]);
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

// ---- gated activation, operands and result in the same layout -------------------------------------------
// G, U (row stride ld_in) and H (row stride ld_out) are rows x cols with cols contiguous: tokens x features for
// row-major operands, features x tokens for column-major ones (then G and U are the two halves of Z one after
// the other).  Eight consecutive elements per lane.
template <typename T, int GATE>
__global__ __launch_bounds__(kThreads) void glu_fwd_kernel(const T *__restrict__ G, const T *__restrict__ U,
                                                           T *__restrict__ H, int64_t n8, int c8, int64_t ld_in,
                                                           int64_t ld_out)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    const int64_t row = idx / c8, col = (idx - row * c8) * 8;
    float g[8], u[8], h[8];
    Vec8<T>::load(G + row * ld_in + col, g);
    Vec8<T>::load(U + row * ld_in + col, u);
#pragma unroll
    for (int k = 0; k < 8; ++k) h[k] = s24_glu<GATE>(g[k], u[k]);
    Vec8<T>::store(H + row * ld_out + col, h);
}

template <typename T, int GATE>
__global__ __launch_bounds__(kThreads) void glu_bwd_kernel(const T *__restrict__ dH, const T *__restrict__ G,
                                                           const T *__restrict__ U, T *__restrict__ dG,
                                                           T *__restrict__ dU, int64_t n8, int c8, int64_t ld_h,
                                                           int64_t ld_z)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n8) return;
    const int64_t row = idx / c8, col = (idx - row * c8) * 8;
    const int64_t off = row * ld_z + col;
    float d[8], g[8], u[8], dg[8], du[8];
    Vec8<T>::load(dH + row * ld_h + col, d);
    Vec8<T>::load(G + off, g);
    Vec8<T>::load(U + off, u);
#pragma unroll
    for (int k = 0; k < 8; ++k) s24_glu_grad<GATE>(d[k], g[k], u[k], dg[k], du[k]);
    Vec8<T>::store(dG + off, dg);
    Vec8<T>::store(dU + off, du);
}

// ---- gated activation across layouts: a 64 x 64 tile goes through LDS ---------------------------------------
// The tile is read along the contiguous axis of its source (eight elements per lane), and written along the
// contiguous axis of its destination, which is the other one.  LDS holds it as fp32, 64 rows of 65 words: the
// transposed reads of a wave (32 or 64 different rows, one column) then fall on distinct banks.
constexpr int kTT = 64, kTPitch = kTT + 1;

// Reads the tile [r0, r0+64) x [c0, c0+64) of a rows x cols matrix (cols contiguous) into lds[r][c]; cells past the
// edge become zero.  256 lanes, two passes of 32 rows.
template <typename T>
__device__ __forceinline__ void tile_in(const T *__restrict__ src, int64_t ld, int64_t rows, int64_t cols, int64_t r0,
                                        int64_t c0, float *lds, int tid)
{
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = 32 * pass + (tid >> 3), c = 8 * (tid & 7);
        float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (r0 + r < rows && c0 + c < cols) Vec8<T>::load(src + (r0 + r) * ld + c0 + c, x);   // cols is a multiple of 8
#pragma unroll
        for (int k = 0; k < 8; ++k) lds[r * kTPitch + c + k] = x[k];
    }
}

// H[c][r] = act(G[r][c]) * U[r][c]: source rows x cols (cols contiguous), destination cols x rows (rows contiguous)
template <typename T, int GATE>
__global__ __launch_bounds__(kThreads) void glu_fwd_transpose_kernel(const T *__restrict__ G, const T *__restrict__ U,
                                                                     T *__restrict__ H, int64_t rows, int64_t cols,
                                                                     int64_t ld_in, int64_t ld_out)
{
    __shared__ float s_h[kTT * kTPitch];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * kTT, c0 = (int64_t)blockIdx.x * kTT;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = 32 * pass + (tid >> 3), c = 8 * (tid & 7);
        float g[8], u[8];
        if (r0 + r < rows && c0 + c < cols) {
            Vec8<T>::load(G + (r0 + r) * ld_in + c0 + c, g);
            Vec8<T>::load(U + (r0 + r) * ld_in + c0 + c, u);
#pragma unroll
            for (int k = 0; k < 8; ++k) s_h[r * kTPitch + c + k] = s24_glu<GATE>(g[k], u[k]);
        }
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int c = 32 * pass + (tid >> 3), r = 8 * (tid & 7);
        if (c0 + c < cols && r0 + r < rows) {   // rows is a multiple of 8: eight cells are all in or all out
            float h[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) h[k] = s_h[(r + k) * kTPitch + c];
            Vec8<T>::store(H + (c0 + c) * ld_out + r0 + r, h);
        }
    }
}

// Backward with dH in the other layout than Z: G, U, dG, dU are rows x cols (cols contiguous, row stride ld_z),
// dH is cols x rows (rows contiguous, row stride ld_h) and crosses through LDS.
template <typename T, int GATE>
__global__ __launch_bounds__(kThreads) void glu_bwd_transpose_kernel(const T *__restrict__ dH, const T *__restrict__ G,
                                                                     const T *__restrict__ U, T *__restrict__ dG,
                                                                     T *__restrict__ dU, int64_t rows, int64_t cols,
                                                                     int64_t ld_h, int64_t ld_z)
{
    __shared__ float s_d[kTT * kTPitch];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * kTT, c0 = (int64_t)blockIdx.x * kTT;
    tile_in<T>(dH, ld_h, cols, rows, c0, r0, s_d, tid);   // s_d[c][r]
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = 32 * pass + (tid >> 3), c = 8 * (tid & 7);
        if (r0 + r < rows && c0 + c < cols) {
            const int64_t off = (r0 + r) * ld_z + c0 + c;
            float g[8], u[8], dg[8], du[8];
            Vec8<T>::load(G + off, g);
            Vec8<T>::load(U + off, u);
#pragma unroll
            for (int k = 0; k < 8; ++k) s24_glu_grad<GATE>(s_d[(c + k) * kTPitch + r], g[k], u[k], dg[k], du[k]);
            Vec8<T>::store(dG + off, dg);
            Vec8<T>::store(dU + off, du);
        }
    }
}

// ---- bias gradient (Sec. 5.2 step 2: d of Z = X W^T + d): sums over tokens --------------------------------------
// Row-major dZ[p][n]: a workgroup of 16 waves owns 64 columns.  A lane reads 16 bytes (eight 16-bit or four fp32
// columns), so one wave-wide load covers the 64-column segments of 8 (4) consecutive rows, the 16 waves walk the
// rows 128 (64) at a time, four loads in flight per wave.  Lanes that hold the same columns are summed by a
// butterfly, the waves' partial sums meet in LDS in a fixed order: the result does not depend on scheduling.
constexpr int kBiasThreads = 1024;
template <typename T>
__global__ __launch_bounds__(kBiasThreads) void bias_grad_rows_kernel(const T *__restrict__ dZ, int64_t ld, int64_t p,
                                                                      int64_t n, float *__restrict__ db, float beta)
{
    constexpr int VEC = 16 / (int)sizeof(T), LPR = 64 / VEC, RPW = 64 / LPR;   // columns per lane, lanes per row, rows per load
    constexpr int64_t STEP = (kBiasThreads / 64) * RPW;
    __shared__ float s_part[kBiasThreads / 64][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cl = VEC * (lane % LPR);
    const int64_t c = (int64_t)blockIdx.x * 64 + cl;
    float acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
    auto add_row = [&](const uint4 &v) {
        if constexpr (sizeof(T) == 2) {
            const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                acc[2 * k] += s24_num<T>::lo(d[k]);
                acc[2 * k + 1] += s24_num<T>::hi(d[k]);
            }
        } else {
            acc[0] += __uint_as_float(v.x);
            acc[1] += __uint_as_float(v.y);
            acc[2] += __uint_as_float(v.z);
            acc[3] += __uint_as_float(v.w);
        }
    };
    if (c < n) {   // n is a multiple of 8: a lane's columns are all in or all out
        const T *src = dZ + c;
        int64_t t = wave * RPW + lane / LPR;
        for (; t + 3 * STEP < p; t += 4 * STEP) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const uint4 *>(src + (t + u * STEP) * ld);
#pragma unroll
            for (int u = 0; u < 4; ++u) add_row(v[u]);
        }
        for (; t < p; t += STEP) add_row(*reinterpret_cast<const uint4 *>(src + t * ld));
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] += __shfl_xor(acc[k], off, 64);
    if (lane < LPR) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) s_part[wave][cl + k] = acc[k];
    }
    __syncthreads();
    if (tid < 64 && (int64_t)blockIdx.x * 64 + tid < n) {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < kBiasThreads / 64; ++k) sum += s_part[k][tid];
        float *o = db + (int64_t)blockIdx.x * 64 + tid;
        *o = beta != 0.0f ? *o + sum : sum;
    }
}

// Column-major dZ (n rows of p contiguous tokens): one wave per feature, eight tokens per lane and step
template <typename T>
__global__ __launch_bounds__(kThreads) void bias_grad_cols_kernel(const T *__restrict__ dZ, int64_t ld, int64_t p,
                                                                  int64_t n, float *__restrict__ db, float beta)
{
    const int lane = threadIdx.x & 63;
    const int64_t c = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (c >= n) return;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t t = 8 * lane; t < p; t += 8 * 64) {   // p is a multiple of 8
        float x[8];
        Vec8<T>::load(dZ + c * ld + t, x);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] += x[k];
    }
    float sum = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
    if (lane == 0) db[c] = beta != 0.0f ? db[c] + sum : sum;
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
        else h[k] = s24_gelu(z[k]);
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
        else dz = s24_gelu_slope(z[k]);
        o[k] = d[k] * dz;
    }
    Vec8<T>::store(dZ + idx * 8, o);
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }
constexpr int64_t kMaxThreads = (int64_t)0x7FFFFFFF * kThreads;

}  // namespace

// Runs `...` with T bound to the storage type of dtype dt.
#define S24_WITH_TYPE(dt, ...)            \
    do {                                  \
        if ((dt) == S24_BF16) {           \
            using T = uint16_t;           \
            __VA_ARGS__;                  \
        } else if ((dt) == S24_F16) {     \
            using T = s24_half;           \
            __VA_ARGS__;                  \
        } else {                          \
            using T = float;              \
            __VA_ARGS__;                  \
        }                                 \
    } while (0)

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
    S24_WITH_TYPE(wdt, hipLaunchKernelGGL(masked_decay_kernel<T>, dim3(blocks_for(n8)), dim3(kThreads), 0, st, G,
                                          static_cast<const T *>(W), mask, lambda, n8, (int)(q / 8), (int)(q / 4)));
    return s24_launch_status();
}

namespace {
// G, U: rows x cols (cols contiguous, stride ld_in); H the same shape with stride ld_out
template <typename T>
int launch_glu_fwd(const void *G, const void *U, void *H, int64_t rows, int64_t cols, int64_t ld_in, int64_t ld_out, int gate,
                   hipStream_t st)
{
    const int64_t n8 = rows * cols / 8;
    const dim3 grid(blocks_for(n8)), block(kThreads);
    auto *g = static_cast<const T *>(G), *u = static_cast<const T *>(U);
    auto *h = static_cast<T *>(H);
    if (gate == S24_GATE_SILU)
        hipLaunchKernelGGL((glu_fwd_kernel<T, S24_GATE_SILU>), grid, block, 0, st, g, u, h, n8, (int)(cols / 8), ld_in, ld_out);
    else
        hipLaunchKernelGGL((glu_fwd_kernel<T, S24_GATE_GELU_ERF>), grid, block, 0, st, g, u, h, n8, (int)(cols / 8), ld_in, ld_out);
    return s24_launch_status();
}
template <typename T>
int launch_glu_bwd(const void *dH, const void *G, const void *U, void *dG, void *dU, int64_t rows, int64_t cols, int64_t ld_h,
                   int64_t ld_z, int gate, hipStream_t st)
{
    const int64_t n8 = rows * cols / 8;
    const dim3 grid(blocks_for(n8)), block(kThreads);
    auto *d = static_cast<const T *>(dH), *g = static_cast<const T *>(G), *u = static_cast<const T *>(U);
    auto *dg = static_cast<T *>(dG), *du = static_cast<T *>(dU);
    if (gate == S24_GATE_SILU)
        hipLaunchKernelGGL((glu_bwd_kernel<T, S24_GATE_SILU>), grid, block, 0, st, d, g, u, dg, du, n8, (int)(cols / 8), ld_h, ld_z);
    else
        hipLaunchKernelGGL((glu_bwd_kernel<T, S24_GATE_GELU_ERF>), grid, block, 0, st, d, g, u, dg, du, n8, (int)(cols / 8), ld_h, ld_z);
    return s24_launch_status();
}
// the transposing kernels: source rows x cols (cols contiguous)
template <typename T>
int launch_glu_fwd_t(const void *G, const void *U, void *H, int64_t rows, int64_t cols, int64_t ld_in, int64_t ld_out, int gate,
                     hipStream_t st)
{
    const dim3 grid((unsigned)((cols + kTT - 1) / kTT), (unsigned)((rows + kTT - 1) / kTT)), block(kThreads);
    S24_REQUIRE(grid.y <= 65535, S24_ERR_SHAPE);   // 4 M rows of the source: beyond any token count of one GPU
    auto *g = static_cast<const T *>(G), *u = static_cast<const T *>(U);
    auto *h = static_cast<T *>(H);
    if (gate == S24_GATE_SILU)
        hipLaunchKernelGGL((glu_fwd_transpose_kernel<T, S24_GATE_SILU>), grid, block, 0, st, g, u, h, rows, cols, ld_in, ld_out);
    else
        hipLaunchKernelGGL((glu_fwd_transpose_kernel<T, S24_GATE_GELU_ERF>), grid, block, 0, st, g, u, h, rows, cols, ld_in, ld_out);
    return s24_launch_status();
}
template <typename T>
int launch_glu_bwd_t(const void *dH, const void *G, const void *U, void *dG, void *dU, int64_t rows, int64_t cols, int64_t ld_h,
                     int64_t ld_z, int gate, hipStream_t st)
{
    const dim3 grid((unsigned)((cols + kTT - 1) / kTT), (unsigned)((rows + kTT - 1) / kTT)), block(kThreads);
    S24_REQUIRE(grid.y <= 65535, S24_ERR_SHAPE);   // 4 M rows of the source: beyond any token count of one GPU
    auto *d = static_cast<const T *>(dH), *g = static_cast<const T *>(G), *u = static_cast<const T *>(U);
    auto *dg = static_cast<T *>(dG), *du = static_cast<T *>(dU);
    if (gate == S24_GATE_SILU)
        hipLaunchKernelGGL((glu_bwd_transpose_kernel<T, S24_GATE_SILU>), grid, block, 0, st, d, g, u, dg, du, rows, cols, ld_h, ld_z);
    else
        hipLaunchKernelGGL((glu_bwd_transpose_kernel<T, S24_GATE_GELU_ERF>), grid, block, 0, st, d, g, u, dg, du, rows, cols, ld_h, ld_z);
    return s24_launch_status();
}

// Shape rules shared by the gated entry points: p tokens, f gated features, every leading dimension a multiple of 8
// elements and at least the extent it strides over.
int check_glu(int64_t p, int64_t f, int dt, int gate)
{
    S24_REQUIRE(s24_valid_dtype(dt) && s24_valid_gate(gate), S24_ERR_DTYPE);
    S24_REQUIRE(p >= 0 && f >= 0 && f % 8 == 0, S24_ERR_SHAPE);
    S24_REQUIRE(p * f / 8 <= kMaxThreads && f / 8 < (1ll << 31) && p < (1ll << 31), S24_ERR_SHAPE);
    return S24_OK;
}
bool ld_ok(int layout, int64_t ld, int64_t p, int64_t n) { return ld % 8 == 0 && ld >= (layout == S24_COL_MAJOR ? p : n); }
}  // namespace

extern "C" int s24_glu_fwd(const void *Z, s24_layout lz, int64_t ldz, void *H, s24_layout lh, int64_t ldh, int64_t p,
                           int64_t f, s24_gate gate, s24_dtype dt, void *stream)
{
    const int rc = check_glu(p, f, dt, gate);
    if (rc != S24_OK) return rc;
    S24_REQUIRE(s24_valid_layout(lz) && s24_valid_layout(lh), S24_ERR_DTYPE);
    S24_REQUIRE(ld_ok(lz, ldz, p, 2 * f) && ld_ok(lh, ldh, p, f), S24_ERR_SHAPE);
    S24_REQUIRE((lz == S24_ROW_MAJOR && lh == S24_ROW_MAJOR) || p % 8 == 0, S24_ERR_SHAPE);   // tokens contiguous somewhere
    if (p * f == 0) return S24_OK;
    S24_REQUIRE(Z && H, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(Z, 16) && s24_aligned(H, 16), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t es = s24_elem_size(dt);
    // the up half Z_2: f columns further in a row-major Z, f rows further in a column-major one
    const void *U = static_cast<const char *>(Z) + (lz == S24_ROW_MAJOR ? f : f * ldz) * es;
    int out = S24_OK;
    if (lz == S24_ROW_MAJOR && lh == S24_ROW_MAJOR) S24_WITH_TYPE(dt, out = launch_glu_fwd<T>(Z, U, H, p, f, ldz, ldh, gate, st));
    else if (lz == S24_COL_MAJOR && lh == S24_COL_MAJOR) S24_WITH_TYPE(dt, out = launch_glu_fwd<T>(Z, U, H, f, p, ldz, ldh, gate, st));
    else if (lz == S24_COL_MAJOR) S24_WITH_TYPE(dt, out = launch_glu_fwd_t<T>(Z, U, H, f, p, ldz, ldh, gate, st));
    else S24_WITH_TYPE(dt, out = launch_glu_fwd_t<T>(Z, U, H, p, f, ldz, ldh, gate, st));
    return out;
}

extern "C" int s24_glu_bwd(const void *dH, s24_layout lh, int64_t ldh, const void *Z, s24_layout lz, int64_t ldz, void *dZ,
                           int64_t p, int64_t f, s24_gate gate, s24_dtype dt, void *stream)
{
    const int rc = check_glu(p, f, dt, gate);
    if (rc != S24_OK) return rc;
    S24_REQUIRE(s24_valid_layout(lz) && s24_valid_layout(lh), S24_ERR_DTYPE);
    S24_REQUIRE(ld_ok(lz, ldz, p, 2 * f) && ld_ok(lh, ldh, p, f), S24_ERR_SHAPE);
    S24_REQUIRE((lz == S24_ROW_MAJOR && lh == S24_ROW_MAJOR) || p % 8 == 0, S24_ERR_SHAPE);
    if (p * f == 0) return S24_OK;
    S24_REQUIRE(dH && Z && dZ, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dH, 16) && s24_aligned(Z, 16) && s24_aligned(dZ, 16), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t half = (size_t)(lz == S24_ROW_MAJOR ? f : f * ldz) * s24_elem_size(dt);
    const void *U = static_cast<const char *>(Z) + half;
    void *dU = static_cast<char *>(dZ) + half;
    int out = S24_OK;
    if (lz == S24_ROW_MAJOR && lh == S24_ROW_MAJOR) S24_WITH_TYPE(dt, out = launch_glu_bwd<T>(dH, Z, U, dZ, dU, p, f, ldh, ldz, gate, st));
    else if (lz == S24_COL_MAJOR && lh == S24_COL_MAJOR) S24_WITH_TYPE(dt, out = launch_glu_bwd<T>(dH, Z, U, dZ, dU, f, p, ldh, ldz, gate, st));
    else if (lz == S24_COL_MAJOR) S24_WITH_TYPE(dt, out = launch_glu_bwd_t<T>(dH, Z, U, dZ, dU, f, p, ldh, ldz, gate, st));
    else S24_WITH_TYPE(dt, out = launch_glu_bwd_t<T>(dH, Z, U, dZ, dU, p, f, ldh, ldz, gate, st));
    return out;
}

// SwiGLU on separately addressed halves: the row-major gated kernels with the SiLU gate
extern "C" int s24_swiglu_fwd(const void *G, const void *U, void *H, int64_t p, int64_t f, int64_t ld_gu, s24_dtype dt,
                              void *stream)
{
    const int rc = check_glu(p, f, dt, S24_GATE_SILU);
    if (rc != S24_OK) return rc;
    S24_REQUIRE(ld_gu % 8 == 0 && ld_gu >= f, S24_ERR_SHAPE);
    if (p * f == 0) return S24_OK;
    S24_REQUIRE(G && U && H, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(G, 16) && s24_aligned(U, 16) && s24_aligned(H, 16), S24_ERR_ALIGN);
    int out = S24_OK;
    S24_WITH_TYPE(dt, out = launch_glu_fwd<T>(G, U, H, p, f, ld_gu, f, S24_GATE_SILU, static_cast<hipStream_t>(stream)));
    return out;
}

extern "C" int s24_swiglu_bwd(const void *dH, const void *G, const void *U, void *dG, void *dU, int64_t p, int64_t f,
                              int64_t ld_gu, s24_dtype dt, void *stream)
{
    const int rc = check_glu(p, f, dt, S24_GATE_SILU);
    if (rc != S24_OK) return rc;
    S24_REQUIRE(ld_gu % 8 == 0 && ld_gu >= f, S24_ERR_SHAPE);
    if (p * f == 0) return S24_OK;
    S24_REQUIRE(dH && G && U && dG && dU, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dH, 16) && s24_aligned(G, 16) && s24_aligned(U, 16) && s24_aligned(dG, 16) && s24_aligned(dU, 16),
                S24_ERR_ALIGN);
    int out = S24_OK;
    S24_WITH_TYPE(dt, out = launch_glu_bwd<T>(dH, G, U, dG, dU, p, f, f, ld_gu, S24_GATE_SILU, static_cast<hipStream_t>(stream)));
    return out;
}

extern "C" int s24_bias_grad(const void *dZ, s24_layout layout, int64_t ld, int64_t p, int64_t n, float *db, float beta,
                             s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(dt) && s24_valid_layout(layout), S24_ERR_DTYPE);
    S24_REQUIRE(p >= 0 && n >= 0 && n % 8 == 0 && ld_ok(layout, ld, p, n) && p < (1ll << 31) && n < (1ll << 31), S24_ERR_SHAPE);
    S24_REQUIRE(layout == S24_ROW_MAJOR || p % 8 == 0, S24_ERR_SHAPE);
    S24_REQUIRE(beta == 0.0f || beta == 1.0f, S24_ERR_UNSUPPORTED);
    if (n == 0) return S24_OK;
    S24_REQUIRE(db != nullptr && (p == 0 || dZ != nullptr), S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dZ, 16) && s24_aligned(db, 4), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (layout == S24_ROW_MAJOR)
        S24_WITH_TYPE(dt, hipLaunchKernelGGL(bias_grad_rows_kernel<T>, dim3((unsigned)((n + 63) / 64)), dim3(kBiasThreads), 0, st,
                                             static_cast<const T *>(dZ), ld, p, n, db, beta));
    else
        S24_WITH_TYPE(dt, hipLaunchKernelGGL(bias_grad_cols_kernel<T>, dim3((unsigned)((n + 3) / 4)), dim3(kThreads), 0, st,
                                             static_cast<const T *>(dZ), ld, p, n, db, beta));
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
    int out = S24_OK;
    S24_WITH_TYPE(dt, out = launch_act<T>(Z, nullptr, H, n / 8, act, false, static_cast<hipStream_t>(stream)));
    return out;
}

extern "C" int s24_act_bwd(const void *dH, const void *Z, void *dZ, int64_t n, s24_act act, s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(dt) && (act == S24_ACT_RELU || act == S24_ACT_GELU_ERF), S24_ERR_DTYPE);
    S24_REQUIRE(n >= 0 && n % 8 == 0 && n / 8 <= kMaxThreads, S24_ERR_SHAPE);
    if (n == 0) return S24_OK;
    S24_REQUIRE(dH && Z && dZ, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(dH, 16) && s24_aligned(Z, 16) && s24_aligned(dZ, 16), S24_ERR_ALIGN);
    int out = S24_OK;
    S24_WITH_TYPE(dt, out = launch_act<T>(dH, Z, dZ, n / 8, act, true, static_cast<hipStream_t>(stream)));
    return out;
}
