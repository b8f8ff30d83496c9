// Instrumentation, not part of the method: the two ceilings a roofline for this library is read against, measured on
// the device the library runs on instead of taken from a data sheet.
//   s24_probe_matrix_rate  a register-only loop of matrix-core instructions (no LDS, no memory): the rate at which
//                          the chip issues v_mfma_f32_32x32x16_bf16 (dense) or v_smfmac_f32_32x32x32_bf16 (2:4
//                          sparse) when nothing else competes, at the clock it holds under that load
//   s24_probe_copy         a plain device-to-device copy in 16-byte accesses: what HBM delivers to a kernel that
//                          does nothing but move bytes
// The caller times the launches (events on the stream) and divides.
#include "s24_common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kProbeThreads = 512;   // eight waves, two per SIMD, as in the large-tile GEMMs
constexpr int kChains = 4;           // independent accumulators per wave: covers the instruction's own latency

__device__ __forceinline__ float probe_value(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return (float)((int)(x & 0xFFFF) - 32768) * (1.0f / 65536.0f);   // in [-0.5, 0.5): operands with every bit in use
}

// KIND 0: dense 32x32x16, 2*32*32*16 FLOP per instruction; KIND 1: sparse 32x32x32, 2*32*32*32 dense-equivalent FLOP
template <int KIND> __global__ __launch_bounds__(kProbeThreads) void matrix_rate_kernel(int iters, float *sink)
{
    const uint32_t id = blockIdx.x * kProbeThreads + threadIdx.x;
    bf16x8 a[kChains];
    bf16x16 b[kChains];
    f32x16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
#pragma unroll
        for (int j = 0; j < 8; ++j) a[c][j] = (__bf16)probe_value(id * 131u + c * 17u + j);
#pragma unroll
        for (int j = 0; j < 16; ++j) b[c][j] = (__bf16)probe_value(id * 257u + c * 29u + j + 1000u);
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[c][j] = 0.0f;
    }
    const int idx = 0x4E4E4E4E;   // index nibbles i0 | i1 << 2 of kept positions {2,3} and {0,1} in turn: legal pairs
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) {
            if constexpr (KIND == 0) {
                bf16x8 bb;
#pragma unroll
                for (int j = 0; j < 8; ++j) bb[j] = b[c][j];
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], bb, acc[c], 0, 0, 0);
            } else {
                acc[c] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[c], b[c], acc[c], idx, 0, 0);
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[c][j];
    sink[id] = s;
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// One 16-byte access per lane and a workgroup per 4 KB: measured the fastest shape on MI355X (6.5 TB/s read + written;
// two, four and eight accesses per lane gave 6.1, 6.2 and 4.4), ahead of the runtime's own device copy (5.0).
__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

extern "C" int s24_probe_matrix_rate(int sparse, int workgroups, int iters, float *sink, void *stream)
{
    S24_REQUIRE(workgroups >= 0 && workgroups <= (1 << 20) && iters >= 0, S24_ERR_SHAPE);
    if (workgroups == 0) return S24_OK;
    S24_REQUIRE(sink != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(sink, 4), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (sparse)
        hipLaunchKernelGGL(matrix_rate_kernel<1>, dim3(workgroups), dim3(kProbeThreads), 0, st, iters, sink);
    else
        hipLaunchKernelGGL(matrix_rate_kernel<0>, dim3(workgroups), dim3(kProbeThreads), 0, st, iters, sink);
    return s24_launch_status();
}

extern "C" int s24_probe_copy(const void *src, void *dst, int64_t bytes, void *stream)
{
    S24_REQUIRE(bytes >= 0 && bytes % 16 == 0, S24_ERR_SHAPE);
    if (bytes == 0) return S24_OK;
    S24_REQUIRE(src && dst, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(src, 16) && s24_aligned(dst, 16), S24_ERR_ALIGN);
    const int64_t n16 = bytes / 16;
    const int64_t grid = (n16 + 255) / 256;
    S24_REQUIRE(grid < (1ll << 31), S24_ERR_SHAPE);
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), n16);
    return s24_launch_status();
}
