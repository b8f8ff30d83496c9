// GEMMs of the 2:4-sparse FFN step on gfx950 matrix cores, for bf16 and IEEE binary16 operands alike (fp32
// accumulation; the element type only selects the instruction and the epilogue conversions).
//
//   sparse NT  out[n][m] = sum_k B[n][k] * A[m][k], A 2:4-compressed along k
//              (Eq. 2 with A = W, Eq. 3 with A = W^T): v_smfmac_f32_32x32x32_{bf16,f16},
//              with the activation forward / backward (Sec. 5.2) and the bias as optional epilogues
//   sparse TN  dW = S_z(dY^T) X (Eq. 4): the same instruction, the dense operand read through transposing LDS reads
//   dense  NT  Y = X W^T (Eq. 1, first GEMM; the comparison kernel): v_mfma_f32_32x32x16_{bf16,f16}
//   dense  TN  dW = dY^T X (Eq. 1, third GEMM): both operands copied as they lie in memory, k-contiguous
//              fragments by ds_read_b64_tr_b16; masked decay (Eq. 10) as an optional epilogue
//   fp32       one-thread-per-output kernels for the small checking workload (no fp32 sparse instruction exists)
//
// Register layout of the sparse instruction (one 32x32 tile, 32 of k):
// lane l holds for A row l%32 the eight kept values of k in [16*(l/32),
// 16*(l/32)+16) in order, with their 2-bit positions in bits [2j+1:2j] of the
// index register half chosen by ABID; for B column l%32, element j holds
// k = 16*(j/8) + 8*(l/32) + j%8; accumulator i holds row 8*(i/4)+4*(l/32)+i%4
// of column l%32.  One metadata word (a uint16 per 16 of k) is exactly one
// lane's index half, and the chunk-major storage of the compressed operand
// (vals[K/64][M][32], meta[K/64][M][4]) makes the 64-byte value run and the
// four index words of one row and chunk contiguous, rows back to back.
#include "s24_common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) _Float16 f16x16;

// The 16-bit kernels move operands as raw bits (fragments are typed bf16x8 / bf16x16 whatever they hold); the
// element type T (uint16_t = bf16 bits, s24_half = IEEE binary16) only selects the matrix instruction and the
// conversions of the epilogues.
template <typename T> struct Mma;
template <> struct Mma<uint16_t> {
    static __device__ __forceinline__ f32x16 dense(bf16x8 a, bf16x8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    template <int ABID> static __device__ __forceinline__ f32x16 sparse(bf16x8 a, bf16x16 b, f32x16 c, int idx)
    {
        return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, b, c, idx, 0, ABID);
    }
};
template <> struct Mma<s24_half> {
    static __device__ __forceinline__ f32x16 dense(bf16x8 a, bf16x8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    template <int ABID> static __device__ __forceinline__ f32x16 sparse(bf16x8 a, bf16x16 b, f32x16 c, int idx)
    {
        return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x16, b), c, idx, 0, ABID);
    }
};

constexpr int BM = 128, BN = 128, BK = 64;  // workgroup tile; BK in elements of k
constexpr int kThreads = 256;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ bf16x16 as_bf16x16(uint4 lo, uint4 hi)
{
    struct { uint4 a, b; } t{lo, hi};
    return __builtin_bit_cast(bf16x16, t);
}

// LDS tile of a k-contiguous operand: rows of 64 bf16 (128 bytes = 8 chunks of
// 16 bytes); chunk c of row r sits at chunk position c ^ ((r ^ r>>3) & 7), which
// keeps 16-byte accesses to one chunk column free of bank conflicts both over
// consecutive rows (MFMA operand reads) and over rows 8 apart (transposed stores).
__device__ __forceinline__ int lds_off(int row, int chunk)
{
    return row * 128 + ((chunk ^ ((row ^ (row >> 3)) & 7)) << 4);
}
__device__ __forceinline__ uint4 lds_read(const unsigned char *buf, int row, int chunk)
{
    return *reinterpret_cast<const uint4 *>(buf + lds_off(row, chunk));
}

// Copy a [rows x 64] bf16 tile (row stride ld elements) from global memory into
// registers: 1024 chunks of 16 bytes, four per thread.  Rows >= nrows read as zero.
struct TileRegs { uint4 v[4]; };
__device__ __forceinline__ void tile_load(TileRegs &t, const uint16_t *g, int64_t ld, int row0, int nrows, int k0, int tid)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + kThreads * i, row = id >> 3, c = id & 7;
        if (row0 + row < nrows) t.v[i] = *reinterpret_cast<const uint4 *>(g + (int64_t)(row0 + row) * ld + k0 + 8 * c);
        else t.v[i] = make_uint4(0, 0, 0, 0);
    }
}
__device__ __forceinline__ void tile_store(const TileRegs &t, unsigned char *buf, int tid)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + kThreads * i, row = id >> 3, c = id & 7;
        *reinterpret_cast<uint4 *>(buf + lds_off(row, c)) = t.v[i];
    }
}

// ------------------------------------------------------------------ sparse NT
// Large tile: workgroup tile 256 (m) x 256 (n) x 64 (k), eight waves as 2 (m) x 4 (n), each
// wave 128 x 64 = 4 x 2 accumulator tiles.  Both operands are copied from
// global memory straight into LDS (no register staging) through a ring of
// three 50 KB stages; the copies of chunk kc+3 go out while the second half of chunk kc is
// multiplied, and the one barrier of a chunk sits between its two halves, where the matrix unit
// still has the second half's operands in registers (see the main loop).  LDS layouts: dense operand rows of 128 bytes with the
// 16-byte chunk c of row r at slot c ^ ((r ^ r>>3) & 7); compressed operand
// rows of 64 bytes with chunk c at slot c ^ ((r>>2) & 3).  Both keep any 16
// consecutive lanes of an operand read on distinct 16-byte slots modulo 256
// bytes, which is what a full-rate 128-bit LDS read needs on this chip.
namespace big {
constexpr int BM = 256, BN = 256, THREADS = 512;
constexpr int B_STAGE = BN * 128, A_STAGE = BM * 64, M_STAGE = BM * 8, STAGE = B_STAGE + A_STAGE + M_STAGE;
typedef __attribute__((address_space(3))) void *lds_ptr;
typedef const __attribute__((address_space(1))) void *glb_ptr;

__device__ __forceinline__ int b_slot(int row, int c) { return row * 128 + ((c ^ ((row ^ (row >> 3)) & 7)) << 4); }
__device__ __forceinline__ int a_slot(int row, int c) { return row * 64 + ((c ^ ((row >> 2) & 3)) << 4); }

// Buffer descriptor for direct-to-LDS copies: base address in scalar registers, raw (unstructured) addressing, no
// bounds clamp that the kernels rely on (every offset they form is inside the operand and below 4 GB, which the host
// checks; the descriptor declares the full 4 GB of records).
// (The host pass of the compiler does not know these builtins: it sees empty bodies.)
#if defined(__HIP_DEVICE_COMPILE__)
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t buffer_of(const void *base)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0xFFFFFFFFu, 0x27000);
}
// BYTES (16 or 4) per lane from byte offset `voff` of the buffer to lds + 64 * BYTES * (lane's index in the wave)
template <int BYTES> __device__ __forceinline__ void buffer_to_lds(rsrc_t buf, lds_ptr lds, uint32_t voff)
{
    static_assert(BYTES == 16 || BYTES == 4, "copy width");
    if constexpr (BYTES == 16) __builtin_amdgcn_raw_ptr_buffer_load_lds(buf, lds, 16, voff, 0, 0, 0);
    else __builtin_amdgcn_raw_ptr_buffer_load_lds(buf, lds, 4, voff, 0, 0, 0);
}
// 8 bytes / 2 bytes into registers from byte offset voff (per lane) + soff (wave-uniform, a scalar register): a load
// whose address costs one vector register however many of them a wave issues in a row
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 buffer_load_8(rsrc_t buf, uint32_t voff, uint32_t soff)
{
    const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(buf, (int)voff, (int)soff, 0);
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint32_t buffer_load_2(rsrc_t buf, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b16(buf, (int)voff, (int)soff, 0);
}
#else
typedef const void *rsrc_t;
__device__ __forceinline__ rsrc_t buffer_of(const void *base) { return base; }
template <int BYTES> __device__ __forceinline__ void buffer_to_lds(rsrc_t, lds_ptr, uint32_t) {}
__device__ __forceinline__ uint2 buffer_load_8(rsrc_t, uint32_t, uint32_t) { return make_uint2(0, 0); }
__device__ __forceinline__ uint32_t buffer_load_2(rsrc_t, uint32_t, uint32_t) { return 0; }
#endif

// s_waitcnt immediate: vmcnt(n), lgkmcnt(0), expcnt unconstrained
__host__ __device__ constexpr int wait_vm_lgkm0(int n) { return (n & 15) | (7 << 4) | ((n >> 4) << 14); }

// Workgroup barrier that leaves up to VM vector-memory operations (direct-to-LDS copies of later
// chunks) in flight.  The raw wait and barrier instructions carry no memory semantics for the
// compiler, so they are fenced on both sides against reordering of LDS accesses, in the
// optimiser (empty asm with a memory clobber) and in the instruction scheduler.
template <int VM>
__device__ __forceinline__ void wait_and_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(VM));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// Clock probe (instrumentation, off unless a buffer is registered): workgroup 0 of a large-tile kernel
// reports how many core-clock cycles and how many ticks of the fixed 100 MHz reference passed between its
// first and its last instruction.  Their ratio is the core clock the chip sustained under this kernel.
struct ClockStamp { unsigned long long cycles, ticks; };
__device__ __forceinline__ ClockStamp clock_now()
{
    return {__builtin_readcyclecounter(), __builtin_amdgcn_s_memrealtime()};
}
__device__ __forceinline__ void clock_report(unsigned long long *probe, const ClockStamp &t0)
{
    if (probe != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
        const ClockStamp t1 = clock_now();
        probe[0] = t1.cycles - t0.cycles;
        probe[1] = t1.ticks - t0.ticks;
    }
}

// Output of one wave's 64 (n) x 128 (m) accumulator tile as bf16.  The wave parks the tile in LDS as
// 64 rows of 256 bytes and streams it out 16 bytes per lane, 16 lanes covering one 256-byte row
// segment of the output.  Inside a row the 8-byte unit u is stored at u ^ (row & 31), so the
// accumulator writes of 32 consecutive rows (same u) fall on distinct banks; a 16-byte read gets
// units 2c and 2c+1 from one aligned slot, in swapped order on odd rows.
// `estage` is EWAVE bytes of LDS private to the wave and no longer used for anything else.
// A wave tile has MI accumulator blocks along m (4: 128 features, rows of 256 bytes; 2: 64 features, rows of 128
// bytes whose units are swizzled with row & 15).
constexpr int EWAVE = 64 * 256;
template <typename T, int MI>
__device__ __forceinline__ void stage_tile(const f32x16 (&acc)[MI][2], unsigned char *estage, int lane)
{
    constexpr int RB = 64 * MI, UMASK = 8 * MI - 1;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int nl = 32 * ni + (lane & 31), u = 8 * mi + 2 * g4 + (lane >> 5);
                *reinterpret_cast<uint2 *>(estage + nl * RB + ((u ^ (nl & UMASK)) << 3)) =
                    make_uint2(s24_num<T>::pack2(acc[mi][ni][4 * g4], acc[mi][ni][4 * g4 + 1]),
                               s24_num<T>::pack2(acc[mi][ni][4 * g4 + 2], acc[mi][ni][4 * g4 + 3]));
            }
}
// Z = X W^T + d (Sec. 5.2 step 2): adds the bias of output feature m to the wave's 128 (m) x 64 (n) accumulator
// tile before it is rounded.  `bias` points at the entry of the tile's first feature; features at or past `limit`
// (edge tiles; never stored) read the last four valid entries instead.
template <typename T, int MI>
__device__ __forceinline__ void add_bias(f32x16 (&acc)[MI][2], const uint16_t *__restrict__ bias, int limit, int lane)
{
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int m = min(32 * mi + 8 * g4 + 4 * (lane >> 5), limit - 4);
            const uint2 b = *reinterpret_cast<const uint2 *>(bias + m);
            const float b4[4] = {s24_num<T>::lo(b.x), s24_num<T>::hi(b.x), s24_num<T>::lo(b.y), s24_num<T>::hi(b.y)};
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[mi][ni][4 * g4 + e] += b4[e];
        }
        // four loads in flight at a time: all sixteen at once would not fit beside the 128 accumulators
        __builtin_amdgcn_sched_barrier(0);
    }
}
// 16-byte chunk c (eight bf16, columns 8c .. 8c+7) of row nl of a staged tile
template <int MI = 4> __device__ __forceinline__ uint4 staged_chunk(const unsigned char *estage, int nl, int c)
{
    const int x = nl & (8 * MI - 1);
    const uint4 v = *reinterpret_cast<const uint4 *>(estage + nl * (64 * MI) + ((((2 * c) ^ x) & ~1) << 3));
    return (x & 1) ? make_uint4(v.z, v.w, v.x, v.y) : v;
}
template <typename T, int MI>
__device__ __forceinline__ void staged_store(const f32x16 (&acc)[MI][2], unsigned char *estage, uint16_t *__restrict__ Out,
                                             int N, int M, int n_base, int m_base, int lane)
{
    stage_tile<T, MI>(acc, estage, lane);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(0));   // the wave reads back only what it wrote itself
    asm volatile("" ::: "memory");
    constexpr int LPR = 4 * MI;   // lanes per row of the tile (16-byte pieces)
#pragma unroll 4
    for (int j = 0; j < LPR; ++j) {
        const int nl = (64 / LPR) * j + lane / LPR, c = lane % LPR;
        const int n = n_base + nl, m = m_base + 8 * c;
        if (n >= N || m >= M) continue;   // M is a multiple of 16 (and of 8): a chunk is all in or all out
        *reinterpret_cast<uint4 *>(Out + (int64_t)n * M + m) = staged_chunk<MI>(estage, nl, c);
    }
}

// Ungated activation and its slope, chosen at compile time (the same arithmetic as the stand-alone kernels)
template <int ACT> __device__ __forceinline__ float act_value(float z)
{
    if (ACT == S24_ACT_RELU) return z > 0.0f ? z : 0.0f;
    return s24_gelu(z);
}
template <int ACT> __device__ __forceinline__ float act_slope(float z)
{
    if (ACT == S24_ACT_RELU) return z > 0.0f ? 1.0f : 0.0f;
    return s24_gelu_slope(z);
}

// ACT_MODE 1 (forward of an ungated layer): the rounded tile Z is written to Out and H = act(Z) beside it, as the
// stand-alone activation kernel would form it from the stored Z.  ACT_MODE 2 (input gradient of the second
// projection): the rounded tile of dH is not written but multiplied by act'(Z), Z read from `GU`, into Out = dZ.
// SWIGLU (forward of a gated layer, Sec. 5.2): the compressed operand holds the gate rows [0, F) and the up rows
// [F, 2F) of one stacked weight (M = 2F).  A workgroup tile then takes 128 gate features and the 128 up features
// of the same indices, its epilogue pairs them and writes G and U (the halves of Out, row stride M) and
// H = act(G) * U (row stride F, act = SiLU or GELU by GATE), G and U rounded to the storage type before H is formed,
// as the stand-alone kernel sees them.  A bias d[2F] (Sec. 5.2 step 2), if given, is added before that rounding.
// GATE_BWD (input gradient of the down projection of a gated layer): the tile of dH = dY (M.*W_down) is not
// written; its rounding to the storage type goes straight into the backward of the activation, dG = dH U act'(G),
// dU = dH act(G), with G and U read from, and dG and dU written to, the halves of [N][2M] buffers.
// T is the storage type of every 16-bit buffer (bf16 bits or binary16).
// BIAS compiles the bias add into the plain forward kernel (the gated forward tests the pointer at run time; the
// plain kernel without a bias keeps its register budget, which the extra loads would push into scratch).
template <typename T, bool ACCUM, bool SWIGLU = false, bool GATE_BWD = false, int GATE = S24_GATE_SILU, bool BIAS = false,
          int ACT_MODE = 0, int ACT = S24_ACT_RELU, int MI = 4>
__global__ __launch_bounds__(128 * MI) void spmm_nt_big_kernel(const uint16_t *__restrict__ B,
                                                              const uint16_t *__restrict__ Av,
                                                              const uint16_t *__restrict__ Am,
                                                              uint16_t *__restrict__ Out, int N, int K, int M,
                                                              int tiles_m, int tiles_n, unsigned long long *probe,
                                                              uint16_t *__restrict__ H = nullptr, int F = 0,
                                                              const uint16_t *__restrict__ GU = nullptr,
                                                              const uint16_t *__restrict__ bias = nullptr)
{
    static_assert(!(ACCUM && (SWIGLU || GATE_BWD)) && !(SWIGLU && GATE_BWD), "the gated epilogues overwrite");
    static_assert(ACT_MODE == 0 || !(ACCUM || SWIGLU || GATE_BWD), "one epilogue at a time");
    // MI = accumulator blocks per wave along m.  4: the 256 x 256 tile of eight waves (2 x 4, 128 x 64 each).
    // 2: a 128 x 128 tile of four waves (2 x 2, 64 x 64 each) on 25 KB stages, two workgroups per compute unit,
    // for outputs with too few large tiles to fill the chip; every epilogue but the gated ones.  A lane
    // issues the same seven copies per chunk either way (the stage is half as tall and there are half as many lanes).
    static_assert(MI == 4 || (MI == 2 && !SWIGLU && !GATE_BWD), "the small tile has no gated epilogue");
    constexpr int BM = 64 * MI, BN = 64 * MI, WM = 32 * MI;   // workgroup tile, wave tile along m
    constexpr int B_STAGE = BN * 128, A_STAGE = BM * 64, M_STAGE = BM * 8, STAGE = B_STAGE + A_STAGE + M_STAGE;
    const ClockStamp t_start = clock_now();
    // One array per ring stage: the compiler then knows which stage a direct-to-LDS
    // copy writes and does not make reads of the other stages wait for it.
    __shared__ __attribute__((aligned(16))) unsigned char s0[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s1[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s2[STAGE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int wm = wave & 1, wn = wave >> 1;
    // Workgroups are dealt round-robin to the eight XCDs; give each XCD one contiguous
    // slab of the tile grid and walk it in groups of eight n-tiles so that the
    // workgroups resident on one XCD share operand rows in its L2.
    const int total = tiles_m * tiles_n, per_xcd = (total + 7) / 8;
    const int t = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (t >= total) return;
    constexpr int GROUP = 4;   // 4 token tiles x 8 feature tiles resident per XCD: least unique bytes per round
    const int group_sz = GROUP * tiles_m, grp = t / group_sz, in_grp = t - grp * group_sz;
    const int gw = min(GROUP, tiles_n - grp * GROUP);
    const int tm = in_grp / gw, tn = grp * GROUP + in_grp % gw;
    const int m0 = SWIGLU ? tm * 128 : tm * BM, n0 = tn * BN;   // SWIGLU: m0 = first feature of the tile
    const int nk = K / 64;
    // row of the compressed operand behind tile row i (clamped at the edge; such rows are never stored)
    auto a_row = [&](int i) {
        if (SWIGLU) return (i < 128 ? 0 : F) + min(m0 + (i & 127), F - 1);
        return min(m0 + i, M - 1);
    };

    // Sources of the direct-to-LDS copies: a wave-uniform base per operand (advanced by one chunk per stage, in
    // scalar registers: the base of a buffer descriptor) plus a fixed 32-bit byte offset per lane, so that seven
    // copies cost seven address registers and no vector arithmetic
    const char *baseB = reinterpret_cast<const char *>(B + (int64_t)n0 * K);
    const char *baseV = reinterpret_cast<const char *>(Av), *baseM = reinterpret_cast<const char *>(Am);
    uint32_t ob[4], oa[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 32 * wave + 8 * i + (lane >> 3);
        const int c = (lane & 7) ^ ((row ^ (row >> 3)) & 7);
        ob[i] = ((uint32_t)(min(n0 + row, N - 1) - n0) * (uint32_t)K + 8u * c) * 2u;   // a tile's rows span < 4 GB (host check)
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = 32 * wave + 16 * i + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        oa[i] = ((uint32_t)a_row(row) * 32u + 8u * c) * 2u;
    }
    // index words: one 4-byte direct-to-LDS copy per lane and chunk (row 32*wave + lane/2, dword lane%2)
    const uint32_t om = ((uint32_t)a_row(32 * wave + (lane >> 1)) * 4u + 2u * (lane & 1)) * 2u;
    // Every call issues exactly seven copies per lane (four of the dense operand, two of the
    // values, one of the index words), so the wait counts below are constants; past the last
    // chunk it re-reads the last one into a stage nobody will read again.
    auto issue = [&](unsigned char *st, int kc) {
        kc = min(kc, nk - 1);
        const rsrc_t pb = buffer_of(baseB + (int64_t)kc * 128), pv = buffer_of(baseV + (int64_t)kc * M * 64);
        const rsrc_t pm = buffer_of(baseM + (int64_t)kc * M * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) buffer_to_lds<16>(pb, (lds_ptr)(st + (32 * wave + 8 * i) * 128), ob[i]);
#pragma unroll
        for (int i = 0; i < 2; ++i) buffer_to_lds<16>(pv, (lds_ptr)(st + B_STAGE + (32 * wave + 16 * i) * 64), oa[i]);
        buffer_to_lds<4>(pm, (lds_ptr)(st + B_STAGE + A_STAGE + 32 * wave * 8), om);
    };

    f32x16 acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = f32x16{};

    // Fragments of one half (h = 0, 1: the two sparse instructions per accumulator tile and 64-chunk) of a stage
    const int g = lane >> 5;
    auto load_frags = [&](const unsigned char *st, int h, bf16x16 (&b)[2], bf16x8 (&a)[MI]) {
        const unsigned char *sb = st, *sa = st + B_STAGE;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int row = 64 * wn + 32 * ni + (lane & 31);
            b[ni] = as_bf16x16(*reinterpret_cast<const uint4 *>(sb + b_slot(row, 2 * h + g)),
                               *reinterpret_cast<const uint4 *>(sb + b_slot(row, 4 + 2 * h + g)));
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = WM * wm + 32 * mi + (lane & 31);
            a[mi] = as_bf16x8(*reinterpret_cast<const uint4 *>(sa + a_slot(row, 2 * g + h)));
        }
    };
    auto load_index = [&](const unsigned char *st, uint32_t (&x)[MI]) {
        const unsigned char *sm = st + B_STAGE + A_STAGE;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
            x[mi] = *reinterpret_cast<const uint32_t *>(sm + (WM * wm + 32 * mi + (lane & 31)) * 8 + 4 * g);
    };

    // keep the program order of these groups: the constant wait counts rely on it
    issue(s0, 0);
    __builtin_amdgcn_sched_barrier(0);
    issue(s1, 1);
    __builtin_amdgcn_sched_barrier(0);
    issue(s2, 2);
    __builtin_amdgcn_sched_barrier(0);
    wait_and_barrier<14>();   // chunk 0 has landed for everybody
    bf16x16 fb0[2];           // first-half fragments and index words of the chunk about to be multiplied
    bf16x8 fa0[MI];
    uint32_t ix[MI];
    load_index(s0, ix);
    load_frags(s0, 0, fb0, fa0);

    // One chunk, software-pipelined across the workgroup barrier.  On entry the first-half fragments of chunk kc
    // are in registers.  Phase A: their eight matrix instructions, with the eight LDS reads of the second half
    // dealt out between them.  Then the one barrier of the chunk: every wave has read all it needs of chunk
    // kc's stage, and chunk kc+1 (copied two chunks ago) has landed for everybody.  Phase B: the second half's
    // eight matrix instructions, whose operands are already in registers -- so the matrix unit has work while
    // the first-half fragments of chunk kc+1 come in from LDS and the seven copies of chunk kc+3 go out into the
    // stage chunk kc just vacated (one per matrix instruction: a wave that issues its copies in one burst sits in
    // the memory pipeline's queue while the matrix unit idles).  A barrier at the top of the chunk instead, with
    // nothing in registers, exposed the LDS latency of twelve reads per wave once per chunk.
    auto chunk = [&](unsigned char *cur, const unsigned char *nxt, int kc) {
        bf16x16 fb1[2];
        bf16x8 fa1[MI];
        load_frags(cur, 1, fb1, fa1);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Mma<T>::template sparse<0>(fa0[mi], fb0[ni], acc[mi][ni], (int)ix[mi]);
        // second-half reads: four of the dense operand and MI of the compressed one
        // (the large tile issues them two per matrix instruction in the first half of the phase, so that the last one
        // has returned before the barrier)
#pragma unroll
        for (int i = 0; i < 2 * MI; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (MI == 4 ? i < 4 : i < 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            else if (MI == 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        // all but the seven most recent copies (chunk kc+2) are complete: this lane's part of chunk kc+1 is in LDS,
        // and its own LDS reads of chunk kc are done
        wait_and_barrier<7>();
        issue(cur, kc + 3);
        uint32_t ixn[MI];
        load_index(nxt, ixn);
        load_frags(nxt, 0, fb0, fa0);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Mma<T>::template sparse<1>(fa1[mi], fb1[ni], acc[mi][ni], (int)ix[mi]);
        if constexpr (MI == 4) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i < 6) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                if (i < 7) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
        } else {   // four matrix instructions: 4 + 2 + 2 reads and 7 copies between them
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i == 0) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
                else if (i < 3) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                if (i < 3) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
                else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) ix[mi] = ixn[mi];
    };
    // past the last chunk the prefetched fragments come from a stage that holds a re-read of the last chunk (or
    // is being refilled with one); they are never multiplied
    int kc = 0;
    for (; kc + 3 <= nk; kc += 3) {
        chunk(s0, s1, kc);
        chunk(s1, s2, kc + 1);
        chunk(s2, s0, kc + 2);
    }
    if (kc < nk) chunk(s0, s1, kc);
    if (kc + 1 < nk) chunk(s1, s2, kc + 1);
    // drain the copies still in flight, then reuse the ring as a staging area for the output tile
    wait_and_barrier<0>();
    clock_report(probe, t_start);
    if constexpr (ACCUM) {
        // beta = 1: add the old output in fp32 straight from the accumulators (a single rounding)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int n = n0 + 64 * wn + 32 * ni + (lane & 31);
            if (n >= N) continue;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int m = m0 + WM * wm + 32 * mi + 8 * g4 + 4 * (lane >> 5);
                    if (m >= M) continue;
                    uint2 *dst = reinterpret_cast<uint2 *>(Out + (int64_t)n * M + m);
                    const uint2 old = *dst;
                    *dst = make_uint2(s24_num<T>::pack2(acc[mi][ni][4 * g4] + s24_num<T>::lo(old.x),
                                                        acc[mi][ni][4 * g4 + 1] + s24_num<T>::hi(old.x)),
                                      s24_num<T>::pack2(acc[mi][ni][4 * g4 + 2] + s24_num<T>::lo(old.y),
                                                        acc[mi][ni][4 * g4 + 3] + s24_num<T>::hi(old.y)));
                }
        }
        return;
    }
    // a wave's parking area for its output tile (64 rows of 64 MI bytes) in the drained ring
    static_assert(MI == 4 ? 3 * EWAVE <= STAGE : 2 * (EWAVE / 2) <= STAGE, "wave tiles must fit the ring stages");
    auto region = [&](int w) {
        if constexpr (MI == 4) return (w < 3 ? s0 : (w < 6 ? s1 : s2)) + (w % 3) * EWAVE;
        else return (w < 2 ? s0 : s1) + (w & 1) * (EWAVE / 2);
    };
    if constexpr (SWIGLU) {
        if (bias != nullptr) add_bias<T, MI>(acc, bias + (wm ? F : 0) + m0, F - m0, lane);   // wave-uniform
    } else if constexpr (BIAS) {
        add_bias<T, MI>(acc, bias + m0 + WM * wm, M - (m0 + WM * wm), lane);   // launched only with a bias
    }
    if constexpr (GATE_BWD) {
        unsigned char *est = region(wave);
        stage_tile<T, 4>(acc, est, lane);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(0));   // the wave reads back only what it wrote itself
        asm volatile("" ::: "memory");
        const int n_base = n0 + 64 * wn, m_base = m0 + 128 * wm;
        // the accumulators are dead now: all 32 loads of G and U go out before anything is computed
        const int c = lane & 15, m = min(m_base + 8 * c, M - 8);
        uint4 g[16], u[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t o = (int64_t)min(n_base + 4 * j + (lane >> 4), N - 1) * 2 * M + m;
            g[j] = *reinterpret_cast<const uint4 *>(GU + o);
            u[j] = *reinterpret_cast<const uint4 *>(GU + o + M);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int nl = 4 * j + (lane >> 4), n = n_base + nl;
            const uint4 dh = staged_chunk(est, nl, c);
            const uint32_t dw[4] = {dh.x, dh.y, dh.z, dh.w}, gw[4] = {g[j].x, g[j].y, g[j].z, g[j].w};
            const uint32_t uw[4] = {u[j].x, u[j].y, u[j].z, u[j].w};
            uint32_t dgw[4], duw[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float dg0, du0, dg1, du1;
                s24_glu_grad<GATE>(s24_num<T>::lo(dw[k]), s24_num<T>::lo(gw[k]), s24_num<T>::lo(uw[k]), dg0, du0);
                s24_glu_grad<GATE>(s24_num<T>::hi(dw[k]), s24_num<T>::hi(gw[k]), s24_num<T>::hi(uw[k]), dg1, du1);
                dgw[k] = s24_num<T>::pack2(dg0, dg1);
                duw[k] = s24_num<T>::pack2(du0, du1);
            }
            if (n < N && m_base + 8 * c < M) {   // M is a multiple of 16: a chunk is all in or all out
                const int64_t o = (int64_t)n * 2 * M + m;
                *reinterpret_cast<uint4 *>(Out + o) = make_uint4(dgw[0], dgw[1], dgw[2], dgw[3]);
                *reinterpret_cast<uint4 *>(Out + o + M) = make_uint4(duw[0], duw[1], duw[2], duw[3]);
            }
        }
    } else if constexpr (ACT_MODE == 2) {
        unsigned char *est = region(wave);
        stage_tile<T, MI>(acc, est, lane);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(0));   // the wave reads back only what it wrote itself
        asm volatile("" ::: "memory");
        constexpr int LPR = 4 * MI, RPP = 64 / LPR;   // lanes per tile row (16-byte pieces), rows per pass
        const int n_base = n0 + 64 * wn, m_base = m0 + WM * wm;
        const int c = lane % LPR, m = min(m_base + 8 * c, M - 8);
        uint4 z[LPR];   // the accumulators are dead: all loads of Z go out before anything is computed
#pragma unroll
        for (int j = 0; j < LPR; ++j)
            z[j] = *reinterpret_cast<const uint4 *>(GU + (int64_t)min(n_base + RPP * j + lane / LPR, N - 1) * M + m);
#pragma unroll
        for (int j = 0; j < LPR; ++j) {
            const int nl = RPP * j + lane / LPR, n = n_base + nl;
            const uint4 dh = staged_chunk<MI>(est, nl, c);
            const uint32_t dw[4] = {dh.x, dh.y, dh.z, dh.w}, zw[4] = {z[j].x, z[j].y, z[j].z, z[j].w};
            uint32_t o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                o[k] = s24_num<T>::pack2(s24_num<T>::lo(dw[k]) * act_slope<ACT>(s24_num<T>::lo(zw[k])),
                                         s24_num<T>::hi(dw[k]) * act_slope<ACT>(s24_num<T>::hi(zw[k])));
            if (n < N && m_base + 8 * c < M)   // M is a multiple of 16: a chunk is all in or all out
                *reinterpret_cast<uint4 *>(Out + (int64_t)n * M + m) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    } else if constexpr (ACT_MODE == 1) {
        unsigned char *est = region(wave);
        stage_tile<T, MI>(acc, est, lane);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(wait_vm_lgkm0(0));
        asm volatile("" ::: "memory");
        constexpr int LPR = 4 * MI, RPP = 64 / LPR;
        const int n_base = n0 + 64 * wn, m_base = m0 + WM * wm;
#pragma unroll 4
        for (int j = 0; j < LPR; ++j) {
            const int nl = RPP * j + lane / LPR, c = lane % LPR;
            const int n = n_base + nl, m = m_base + 8 * c;
            if (n >= N || m >= M) continue;
            const uint4 zc = staged_chunk<MI>(est, nl, c);
            const uint32_t zw[4] = {zc.x, zc.y, zc.z, zc.w};
            uint32_t h[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                h[k] = s24_num<T>::pack2(act_value<ACT>(s24_num<T>::lo(zw[k])), act_value<ACT>(s24_num<T>::hi(zw[k])));
            *reinterpret_cast<uint4 *>(Out + (int64_t)n * M + m) = zc;
            *reinterpret_cast<uint4 *>(H + (int64_t)n * M + m) = make_uint4(h[0], h[1], h[2], h[3]);
        }
    } else if constexpr (!SWIGLU) {
        staged_store<T, MI>(acc, region(wave), Out, N, M, n0 + 64 * wn, m0 + WM * wm, lane);
    } else {
        // waves (0, wn) and (1, wn) hold the gate and the up tile of the same 64 tokens x 128 features: both park
        // their bf16 tiles, then each takes 32 of the 64 token rows and writes G, U and H in 16-byte pieces
        stage_tile<T, 4>(acc, region(wave), lane);
        wait_and_barrier<0>();
        const unsigned char *sg = region(2 * wn), *su = region(2 * wn + 1);
#pragma unroll 2
        for (int j = 0; j < 8; ++j) {
            const int idx = j * 64 + lane, nl = 32 * wm + (idx >> 4), c = idx & 15;
            const int n = n0 + 64 * wn + nl, f = m0 + 8 * c;
            if (n >= N || f >= F) continue;   // F is a multiple of 8: a chunk is all in or all out
            const uint4 g = staged_chunk(sg, nl, c), u = staged_chunk(su, nl, c);
            const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w};
            uint32_t hw[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                hw[k] = s24_num<T>::pack2(s24_glu<GATE>(s24_num<T>::lo(gw[k]), s24_num<T>::lo(uw[k])),
                                          s24_glu<GATE>(s24_num<T>::hi(gw[k]), s24_num<T>::hi(uw[k])));
            *reinterpret_cast<uint4 *>(Out + (int64_t)n * M + f) = g;
            *reinterpret_cast<uint4 *>(Out + (int64_t)n * M + F + f) = u;
            *reinterpret_cast<uint4 *>(H + (int64_t)n * F + f) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
        }
    }
}
}  // namespace big

// ------------------------------------------------------------------ dense MFMA core
// Both operands in LDS as k-contiguous swizzled tiles.  MFMA step i of a lane
// with k-group g = lane/32 uses chunk 4*g + i of its row, i.e. k in
// [32*g + 8*i, 32*g + 8*i + 8) of the 64-wide chunk, for A and B alike.
template <typename T>
__device__ __forceinline__ void dense_chunk(f32x16 (&acc)[2][2], const unsigned char *sa, const unsigned char *sb, int wm,
                                            int wn, int lane)
{
    const int g = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16x8 a[2], b[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) a[mi] = as_bf16x8(lds_read(sa, 64 * wm + 32 * mi + (lane & 31), 4 * g + i));
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) b[ni] = as_bf16x8(lds_read(sb, 64 * wn + 32 * ni + (lane & 31), 4 * g + i));
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                acc[mi][ni] = Mma<T>::dense(a[mi], b[ni], acc[mi][ni]);
    }
}

// Y[n][m] = sum_k X[n][k] W[m][k]  (n tokens, m out-features)
template <typename T>
__global__ __launch_bounds__(kThreads) void dense_nt_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W,
                                                            uint16_t *__restrict__ Y, int N, int K, int M)
{
    __shared__ __attribute__((aligned(16))) unsigned char s_a[2][BM * 128];
    __shared__ __attribute__((aligned(16))) unsigned char s_b[2][BN * 128];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int nk = K / BK;
    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = f32x16{};
    TileRegs ra, rb;
    tile_load(ra, W, K, m0, M, 0, tid);
    tile_load(rb, X, K, n0, N, 0, tid);
    tile_store(ra, s_a[0], tid);
    tile_store(rb, s_b[0], tid);
    __syncthreads();
    for (int kc = 0; kc < nk; ++kc) {
        const bool more = kc + 1 < nk;
        if (more) {
            tile_load(ra, W, K, m0, M, (kc + 1) * BK, tid);
            tile_load(rb, X, K, n0, N, (kc + 1) * BK, tid);
        }
        dense_chunk<T>(acc, s_a[kc & 1], s_b[kc & 1], wm, wn, lane);
        if (more) {
            tile_store(ra, s_a[(kc + 1) & 1], tid);
            tile_store(rb, s_b[(kc + 1) & 1], tid);
        }
        __syncthreads();
    }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int n = n0 + 64 * wn + 32 * ni + (lane & 31);
        if (n >= N) continue;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = m0 + 64 * wm + 32 * mi + 8 * g + 4 * (lane >> 5);
                if (m >= M) continue;
                *reinterpret_cast<uint2 *>(Y + (int64_t)n * M + m) =
                    make_uint2(s24_num<T>::pack2(acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1]),
                               s24_num<T>::pack2(acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]));
            }
    }
}

// ------------------------------------------------------------------ dense NT, large tile
// The dense comparison GEMM in the same tiling family as the sparse kernel:
// 256 x 256 x 64 workgroup tiles, eight waves of 128 x 64, both operands copied
// straight into LDS.  A dense operand tile is twice the compressed one, so the
// ring has two 64 KB stages: the copies of chunk kc+1 fly during the math of kc.
namespace bignt {
// Dense NT GEMM, 256 x 256 tiles, eight waves of 128 x 64: the comparison kernel beside the sparse one, on the
// same schedule.  32 of k per ring stage (two 16 KB operand tiles, 64-byte rows), four stages, three chunks in
// flight; a chunk is two 16-wide steps of eight matrix instructions, the first running from registers while the
// second's fragments come in, the one barrier of the chunk between them, and after it the next chunk's first-step
// fragments and the four copies of chunk kc+4 dealt out between the second step's matrix instructions.
constexpr int BM = 256, BN = 256, THREADS = 512, OPERAND = 256 * 64, STAGE = 2 * OPERAND;
using big::a_slot;
using big::glb_ptr;
using big::lds_ptr;
using big::wait_vm_lgkm0;

template <typename T>
__global__ __launch_bounds__(THREADS) void dense_nt_big_kernel(const uint16_t *__restrict__ X,
                                                               const uint16_t *__restrict__ W, uint16_t *__restrict__ Y,
                                                               int N, int K, int M, int tiles_m, int tiles_n, unsigned long long *probe)
{
    const big::ClockStamp t_start = big::clock_now();
    __shared__ __attribute__((aligned(16))) unsigned char s0[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s1[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s2[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s3[STAGE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int total = tiles_m * tiles_n, per_xcd = (total + 7) / 8;
    const int t = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (t >= total) return;
    constexpr int GROUP = 8;
    const int group_sz = GROUP * tiles_m, grp = t / group_sz, in_grp = t - grp * group_sz;
    const int gw = min(GROUP, tiles_n - grp * GROUP);
    const int tm = in_grp / gw, tn = grp * GROUP + in_grp % gw;
    const int m0 = tm * BM, n0 = tn * BN;
    const int nk = K / 32;

    // copies: two per operand, lane and chunk; copy i of a wave fills rows 128 i + 16 wave .. +15 (four 16-byte
    // slots each); slot c of row r holds source chunk c ^ ((r >> 2) & 3).  Wave-uniform bases (one per operand,
    // advanced by 64 bytes per chunk) and fixed 32-bit lane offsets: 256 rows of K elements span < 4 GB (host check).
    const char *baseX = reinterpret_cast<const char *>(X + (int64_t)n0 * K), *baseW = reinterpret_cast<const char *>(W + (int64_t)m0 * K);
    uint32_t ox[2], ow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = 128 * i + 16 * wave + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        ox[i] = ((uint32_t)(min(n0 + row, N - 1) - n0) * (uint32_t)K + 8u * c) * 2u;
        ow[i] = ((uint32_t)(min(m0 + row, M - 1) - m0) * (uint32_t)K + 8u * c) * 2u;
    }
    // exactly four copies per lane and call; past the last chunk it re-reads the last one into a stage nobody reads
    auto issue = [&](unsigned char *st, int kc) {
        kc = min(kc, nk - 1);
        const big::rsrc_t px = big::buffer_of(baseX + (int64_t)kc * 64), pw = big::buffer_of(baseW + (int64_t)kc * 64);
#pragma unroll
        for (int i = 0; i < 2; ++i) big::buffer_to_lds<16>(px, (lds_ptr)(st + (128 * i + 16 * wave) * 64), ox[i]);
#pragma unroll
        for (int i = 0; i < 2; ++i) big::buffer_to_lds<16>(pw, (lds_ptr)(st + OPERAND + (128 * i + 16 * wave) * 64), ow[i]);
    };
    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = f32x16{};
    // fragments of 16-wide step i of a stage: lane group g = lane / 32 takes source chunk 2 g + i of both operands
    const int g = lane >> 5;
    auto load_frags = [&](const unsigned char *st, int i, bf16x8 (&b)[2], bf16x8 (&a)[4]) {
        const unsigned char *sb = st, *sa = st + OPERAND;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
            b[ni] = as_bf16x8(*reinterpret_cast<const uint4 *>(sb + a_slot(64 * wn + 32 * ni + (lane & 31), 2 * g + i)));
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
            a[mi] = as_bf16x8(*reinterpret_cast<const uint4 *>(sa + a_slot(128 * wm + 32 * mi + (lane & 31), 2 * g + i)));
    };
    // keep the program order of these groups: the constant wait counts rely on it
    issue(s0, 0);
    __builtin_amdgcn_sched_barrier(0);
    issue(s1, 1);
    __builtin_amdgcn_sched_barrier(0);
    issue(s2, 2);
    __builtin_amdgcn_sched_barrier(0);
    issue(s3, 3);
    __builtin_amdgcn_sched_barrier(0);
    big::wait_and_barrier<12>();   // chunk 0 has landed for everybody
    bf16x8 fb0[2], fa0[4];
    load_frags(s0, 0, fb0, fa0);
    auto chunk = [&](unsigned char *cur, const unsigned char *nxt, int kc) {
        bf16x8 fb1[2], fa1[4];
        load_frags(cur, 1, fb1, fa1);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Mma<T>::dense(fa0[mi], fb0[ni], acc[mi][ni]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {   // six reads, two per matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < 3) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        // all but the eight most recent copies (chunks kc+2, kc+3) are complete: this lane's part of chunk kc+1 is
        // in LDS, and its own reads of chunk kc are done
        big::wait_and_barrier<8>();
        issue(cur, kc + 4);
        load_frags(nxt, 0, fb0, fa0);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Mma<T>::dense(fa1[mi], fb1[ni], acc[mi][ni]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {   // six reads and four copies
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < 3) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            if (i & 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // past the last chunk the prefetched fragments come from a stage that holds a re-read of the last chunk (or is
    // being refilled with one); they are never multiplied
    int kc = 0;
    for (; kc + 4 <= nk; kc += 4) {
        chunk(s0, s1, kc);
        chunk(s1, s2, kc + 1);
        chunk(s2, s3, kc + 2);
        chunk(s3, s0, kc + 3);
    }
    if (kc < nk) chunk(s0, s1, kc);
    if (kc + 1 < nk) chunk(s1, s2, kc + 1);
    if (kc + 2 < nk) chunk(s2, s3, kc + 2);
    big::wait_and_barrier<0>();   // last (redundant) copies drained, nobody reads the ring any more: reuse it
    big::clock_report(probe, t_start);
    static_assert(2 * big::EWAVE <= STAGE, "two waves' output tiles per ring stage");
    unsigned char *est = (wave < 2 ? s0 : (wave < 4 ? s1 : (wave < 6 ? s2 : s3))) + (wave & 1) * big::EWAVE;
    big::staged_store<T, 4>(acc, est, Y, N, M, n0 + 64 * wn, m0 + 128 * wm, lane);
}
}  // namespace bignt

// ------------------------------------------------------------------ dense TN (dW), large tile
// dW[m][n] = sum_t dY[t][m] X[t][n] with 256 x 256 workgroup tiles.  Both operands are token-major, so a
// tile chunk (32 tokens x 256 columns) is copied into LDS as it lies in memory, rows of 512 bytes, and the
// matrix-core fragments (8 consecutive t per lane) are gathered with the transposing LDS read.
// ds_read_b64_tr_b16: in a group of 16 lanes, lane i points at row i/4, columns 4*(i%4)..+3 of a
// 4 (t) x 16 (columns) patch and receives, for column i, the four consecutive t (measured on the device
// with an index-filled tile); two such reads give one lane its eight k values.
// LDS swizzle: 16-byte chunk c of row t sits at slot c ^ (4*(t&3)), which keeps the eight 32-byte row
// segments touched by 32 lanes in one cycle on distinct banks.
// Four waves, one per SIMD, each a 128 x 128 tile of 4 x 4 accumulator blocks (256 accumulator registers):
// against eight waves of 128 x 64 this reads a third less LDS per matrix instruction, which matters
// because the chip sheds clock under the combined matrix + LDS + copy load.  The token axis moves through
// a ring of four 32 KB stages.  A chunk is waited for one iteration before it is used, so the first
// fragments of chunk kc+1 are fetched during the last matrix instructions of chunk kc and the barrier
// finds the matrix unit busy; the copies of chunk kc+3 are dealt out between the matrix instructions
// rather than issued in one burst.
namespace dmatn {
constexpr int THREADS = 256;
// WT = 32 x 32 accumulator blocks per wave and axis: 4 -> 256 x 256 workgroup tiles; 2 -> 128 x 128 tiles for
// outputs with too few large tiles to fill the chip.  BT = tokens per ring stage: 32 for the large tile (128 KB
// of LDS); for the small tile 32 (64 KB, two workgroups per CU) when there are more tiles than CUs, else 64 (a
// small tile has a quarter of the matrix work per token, so the barrier is paid half as often).
template <int WT, int BT_> struct Cfg {
    static constexpr int BM = 64 * WT, BN = 64 * WT, BT = BT_;
    static constexpr int ROWB = BM * 2, OPERAND = BT * ROWB, STAGE = 2 * OPERAND, CPR = ROWB / 16;
    static constexpr int NIO = OPERAND / 1024 / 4, NI = 2 * NIO;   // copies per wave, chunk and operand / in total
};
using big::glb_ptr;
using big::lds_ptr;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 *lds_v4i16;

template <int ROWB>
__device__ __forceinline__ int tr_off(int row, int col)
{
    return row * ROWB + ((((col >> 3) ^ ((row & 3) << 2))) << 4) + ((col & 7) << 1);
}
template <int ROWB>
__device__ __forceinline__ bf16x8 tr_frag(const unsigned char *p)
{
    // token rows t..t+3 and t+4..t+7 of this lane group's patch
    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16)(p));
    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16)(p + 4 * ROWB));
    struct { v4i16 a, b; } t{lo, hi};
    return __builtin_bit_cast(bf16x8, t);
}

// DECAY: the masked decay term is added in the epilogue: dW[m][n] += lambda * Wt[m][n] where bit
// 4*(m%4) + n%4 of mask[m/4][n/4] is clear, with the same single fused multiply-add the stand-alone
// decay kernel applies to the stored gradient, so both routes give the same bits.
// One launch covers up to four weight gradients (DwBatch): their tiles share one grid, so that the compute units
// left idle by the last, partial round of one problem take tiles of the next.  The operands of a problem may be
// windows of larger matrices: M and N are the extents of the window's output, ldy, ldx and ldw the row strides
// (elements) of dY, of X and of dW / Wt (the mask's row stride is ldw / 4; a window starts at a multiple of four
// rows and columns).
struct DwWindow {
    const uint16_t *dY, *X, *Wt, *mask;
    float *dW;
    int T, M, N, ldy, ldx, ldw, tiles_m, tiles_n;
    float lambda;
};
constexpr int kMaxBatch = 4;
// Workgroups are dealt round-robin to the eight XCDs.  Each XCD takes, of every problem in turn, one contiguous
// eighth of its tile list: first_slot[i] .. first_slot[i+1]-1 are the positions in an XCD's own list that belong to
// problem i (unused entries repeat the total), so every problem is spread over all XCDs exactly as a launch of its
// own would spread it, and the workgroups resident on one XCD share operand rows in its L2.
struct DwBatch {
    DwWindow w[kMaxBatch];
    int first_slot[kMaxBatch + 1];
};

template <typename ET, int WT, int BT_, bool ACCUM, bool DECAY>
__global__ __launch_bounds__(THREADS) void dense_tn_dma_kernel(const DwBatch batch, unsigned long long *probe)
{
    using C = Cfg<WT, BT_>;
    constexpr int BM = C::BM, BN = C::BN, BT = C::BT, ROWB = C::ROWB, OPERAND = C::OPERAND, STAGE = C::STAGE, CPR = C::CPR;
    constexpr int NIO = C::NIO, NI = C::NI;
    constexpr int KS = BT / 16, CPS = NI / KS;   // 16-token steps per chunk, copies issued per step
    static_assert(KS % 2 == 0 && CPS * KS == NI, "steps alternate between two fragment sets");
    const big::ClockStamp t_start = big::clock_now();
    __shared__ __attribute__((aligned(16))) unsigned char s0[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s1[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s2[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s3[STAGE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int slot = (int)(blockIdx.x >> 3);
    int which = 0;   // wave-uniform: the problem this workgroup's tile belongs to
#pragma unroll
    for (int i = 1; i < kMaxBatch; ++i)
        if (slot >= batch.first_slot[i]) which = i;
    const DwWindow &win = batch.w[which];
    const int per_xcd = batch.first_slot[which + 1] - batch.first_slot[which];
    const int t = (int)(blockIdx.x & 7) * per_xcd + (slot - batch.first_slot[which]);
    if (t >= win.tiles_m * win.tiles_n) return;
    const uint16_t *__restrict__ dY = win.dY, *__restrict__ X = win.X, *__restrict__ Wt = win.Wt, *__restrict__ mask = win.mask;
    float *__restrict__ dW = win.dW;
    const int T = win.T, M = win.M, N = win.N, ldy = win.ldy, ldx = win.ldx, ldw = win.ldw;
    const int tiles_m = win.tiles_m, tiles_n = win.tiles_n;
    const float lambda = win.lambda;
    constexpr int GROUP = 8;
    const int group_sz = GROUP * tiles_m, grp = t / group_sz, in_grp = t - grp * group_sz;
    const int gw = min(GROUP, tiles_n - grp * GROUP);
    const int tm = in_grp / gw, tn = grp * GROUP + in_grp % gw;
    const int m0 = tm * BM, n0 = tn * BN;
    const int nk = (T + BT - 1) / BT;

    // Copies: instruction g of an operand fills the 16-byte slots 64g .. 64g+63 of its stage region, slot ->
    // (row = slot / CPR, chunk = slot % CPR); the source chunk is chunk ^ (4 * (row & 3)).  Columns past the
    // matrix edge are clamped to its last 16-byte chunk.  A lane's byte offsets from the first token row of a
    // chunk are fixed for the whole kernel; only the (wave-uniform) row base moves, so a copy costs no vector
    // arithmetic.  A chunk always starts at a row that leaves BT rows below it: the last chunk of a token count
    // that is not a multiple of BT starts at T - BT and overlaps its predecessor (clear_tail drops the overlap);
    // with fewer than BT tokens in all there is one chunk, rows past T - 1 re-read row T - 1.
    uint32_t voffA[NIO], voffB[NIO];
    const int lastA = (min(M - m0, BM) >> 3) - 1, lastB = (min(N - n0, BN) >> 3) - 1;
#pragma unroll
    for (int j = 0; j < NIO; ++j) {
        const int slot = (wave * NIO + j) * 64 + lane, row = min(slot / CPR, T - 1), c = (slot % CPR) ^ (((slot / CPR) & 3) << 2);
        voffA[j] = (uint32_t)(row * ldy + m0 + 8 * min(c, lastA)) * 2u;
        voffB[j] = (uint32_t)(row * ldx + n0 + 8 * min(c, lastB)) * 2u;
    }
    auto first_row = [&](int kc) { return max(min(kc * BT, T - BT), 0); };
    // Copies first .. first+count-1 of a chunk's list (the dY tile's NIO, then the X tile's NIO).
    // The copies are buffer loads into LDS: a descriptor (scalar registers) whose base is the chunk's first token
    // row, and the lane's fixed 32-bit offset; nothing of a copy's address is computed on the vector unit.
    auto issue = [&](unsigned char *st, int kc, int first, int count) {
        const int row0 = first_row(kc);
        const big::rsrc_t ya = big::buffer_of(dY + (int64_t)row0 * ldy), xb = big::buffer_of(X + (int64_t)row0 * ldx);
#pragma unroll
        for (int c = first; c < first + count; ++c) {
            const int j = c < NIO ? c : c - NIO;
            if (c < NIO)
                big::buffer_to_lds<16>(ya, (lds_ptr)(st + (wave * NIO + j) * 1024), voffA[j]);
            else
                big::buffer_to_lds<16>(xb, (lds_ptr)(st + OPERAND + (wave * NIO + j) * 1024), voffB[j]);
        }
    };
    f32x16 acc[WT][WT];
#pragma unroll
    for (int mi = 0; mi < WT; ++mi)
#pragma unroll
        for (int ni = 0; ni < WT; ++ni) acc[mi][ni] = f32x16{};

    // fragment addressing of this lane: group G = lane/16 -> k half G/2, column half G%2
    const int gi = lane & 15, G = lane >> 4;
    const int frow = 8 * (G >> 1) + (gi >> 2), fcol = 16 * (G & 1) + 4 * (gi & 3);
    int offA[WT], offB[WT];
#pragma unroll
    for (int i = 0; i < WT; ++i) {
        offA[i] = tr_off<ROWB>(frow, 32 * WT * wm + 32 * i + fcol);
        offB[i] = OPERAND + tr_off<ROWB>(frow, 32 * WT * wn + 32 * i + fcol);
    }
    auto load_frags = [&](const unsigned char *st, int ks, bf16x8 (&a)[WT], bf16x8 (&b)[WT]) {
#pragma unroll
        for (int ni = 0; ni < WT; ++ni) b[ni] = tr_frag<ROWB>(st + offB[ni] + 16 * ks * ROWB);
#pragma unroll
        for (int mi = 0; mi < WT; ++mi) a[mi] = tr_frag<ROWB>(st + offA[mi] + 16 * ks * ROWB);
    };
    auto mma = [&](const bf16x8 (&a)[WT], const bf16x8 (&b)[WT]) {
#pragma unroll
        for (int mi = 0; mi < WT; ++mi)
#pragma unroll
            for (int ni = 0; ni < WT; ++ni)
                acc[mi][ni] = Mma<ET>::dense(a[mi], b[ni], acc[mi][ni]);
    };
    // Issue order of one 16-token step: a matrix instruction, then 4/WT LDS reads of the next step's fragments
    // (4*WT reads against WT*WT matrix instructions), and after every other matrix instruction one copy.
    // The reads go out in the first half of the step (two per matrix instruction for the large tile), so that the
    // last fragment has arrived well before the step ends: with one wave per SIMD nobody else covers a wait.
    auto interleave = [&]() {
        constexpr int RPM = 4 / WT, EARLY = WT == 4 ? 2 : 1;
        static_assert(RPM * WT * WT == 4 * WT && 2 * CPS <= WT * WT, "reads and copies fit between the matrix instructions");
#pragma unroll
        for (int i = 0; i < WT * WT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < WT * WT / EARLY) __builtin_amdgcn_sched_group_barrier(0x100, RPM * EARLY, 0);
            if ((i & 1) && (i >> 1) < CPS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // The last chunk of a token count that is not a multiple of BT holds BT - rem rows that must not contribute:
    // the leading rows that its predecessor already covered (the chunk starts at T - BT), or, when there are
    // fewer than BT tokens in all, the trailing rows past T.  They are cleared in the dY tile.
    auto clear_tail = [&](unsigned char *st, int kc) {
        const int rem = T - kc * BT, skip = T >= BT ? 0 : rem;
        for (int idx = tid; idx < (BT - rem) * CPR; idx += THREADS)
            *reinterpret_cast<uint4 *>(st + (skip + idx / CPR) * ROWB + ((idx % CPR) << 4)) = make_uint4(0, 0, 0, 0);
        __syncthreads();
    };
    const bool partial = (T % BT) != 0;

    // prologue: chunks 0..2 in flight, chunk 0 landed, its first fragments in registers
    issue(s0, 0, 0, NI);
    __builtin_amdgcn_sched_barrier(0);
    issue(s1, 1, 0, NI);
    __builtin_amdgcn_sched_barrier(0);
    issue(s2, 2, 0, NI);
    __builtin_amdgcn_sched_barrier(0);
    big::wait_and_barrier<2 * NI>();
    if (partial && nk == 1) clear_tail(s0, 0);
    bf16x8 fa[2][WT], fb[2][WT];   // fragments of the current and of the next 16-token step
    load_frags(s0, 0, fa[0], fb[0]);

    // Iteration kc: all but the NI most recent copies (chunk kc+2) are complete, so chunk kc+1 is in LDS for
    // every wave after the barrier, and nobody reads the stage of chunk kc-1 any more: it takes chunk kc+3.
    auto chunk = [&](const unsigned char *cur, unsigned char *nxt, unsigned char *refill, int kc) {
        big::wait_and_barrier<NI>();
        if (partial && kc + 2 == nk) clear_tail(nxt, kc + 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            issue(refill, kc + 3, ks * CPS, CPS);
            // past the last chunk the final prefetch reads a stage nobody uses; the result is dropped
            if (ks + 1 < KS) load_frags(cur, ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
            else load_frags(nxt, 0, fa[0], fb[0]);
            mma(fa[ks & 1], fb[ks & 1]);
            interleave();
        }
    };
    int kc = 0;
    for (; kc + 4 <= nk; kc += 4) {
        chunk(s0, s1, s3, kc);
        chunk(s1, s2, s0, kc + 1);
        chunk(s2, s3, s1, kc + 2);
        chunk(s3, s0, s2, kc + 3);
    }
    if (kc < nk) chunk(s0, s1, s3, kc);
    if (kc + 1 < nk) chunk(s1, s2, s0, kc + 1);
    if (kc + 2 < nk) chunk(s2, s3, s1, kc + 2);
    // Epilogue through LDS, so that global memory sees 16-byte accesses along rows: each wave parks 64 columns
    // of its tile at a time (32*WT rows of fp32, 256-byte rows) in its own ring stage, then lane l of pass j
    // owns row (64j + l) / 16, columns 4 * (l % 16) .. +3: one LDS read, one 16-byte store, and for the
    // optional terms one 16-byte load of the old gradient, one 8-byte load of W and one mask word.
    // The W and mask loads of a whole 64-column slice are issued in one go, well before they are needed: those of
    // the first slice ahead of the wait that drains the ring, those of the second before it is parked in LDS.
    // Loaded pass by pass where they are used, their latency was exposed eight times per tile with only four
    // waves on the compute unit to hide it (c5: 0.45 ms per step).
    // They are buffer loads: pass j reads four rows further down than pass j - 1, which is a wave-uniform step (a
    // scalar register), so the 64 loads of a slice share two address registers.  M is a multiple of 16 and a wave's
    // rows start at a multiple of 64: the four rows of a pass are all inside the matrix or all outside, and passes
    // past the edge re-read the last pass inside (a wave with no row inside re-reads the tile's first rows).
    constexpr int NP = 8 * WT;   // passes per slice
    uint2 wv[DECAY ? NP : 1];
    uint32_t keep[DECAY ? NP : 1];
    const int wave_rows = min(M - m0 - 32 * WT * wm, 32 * WT);   // rows of this wave's sub-tile inside the matrix
    const int wave_row0 = wave_rows > 0 ? 32 * WT * wm : 0, last_pass = wave_rows > 0 ? (wave_rows >> 2) - 1 : 0;
    auto decay_loads = [&](int h2) {
        if constexpr (DECAY) {
            const int nc = min(n0 + 32 * WT * wn + 64 * h2 + 4 * (lane & 15), N - 4);
            const big::rsrc_t wbuf = big::buffer_of(Wt + (int64_t)(m0 + wave_row0) * ldw);
            const big::rsrc_t mbuf = big::buffer_of(mask + (int64_t)((m0 + wave_row0) >> 2) * (ldw >> 2));
            const uint32_t voff_w = ((uint32_t)(lane >> 4) * (uint32_t)ldw + (uint32_t)nc) * 2u, voff_m = (uint32_t)(nc >> 2) * 2u;
            const uint32_t shift = 4 * (lane >> 4);   // row of the 4 x 4 block: the tile starts at a multiple of four
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const uint32_t jc = (uint32_t)min(j, last_pass);
                wv[j] = big::buffer_load_8(wbuf, voff_w, jc * 8u * (uint32_t)ldw);
                keep[j] = big::buffer_load_2(mbuf, voff_m, jc * 2u * (uint32_t)(ldw >> 2)) >> shift;
            }
        }
    };
    decay_loads(0);
    big::wait_and_barrier<0>();   // last (redundant) copies drained, nobody reads the ring any more: reuse it
    big::clock_report(probe, t_start);
    static_assert(32 * WT * 256 <= STAGE, "a wave's 64-column slice fits one stage");
    unsigned char *est = wave == 0 ? s0 : (wave == 1 ? s1 : (wave == 2 ? s2 : s3));
#pragma unroll
    for (int h2 = 0; h2 < WT / 2; ++h2) {
        if (h2 > 0) decay_loads(h2);
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int mi = 0; mi < WT; ++mi)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = 32 * mi + 8 * (e / 4) + 4 * (lane >> 5) + (e & 3), col = 32 * nj + (lane & 31);
                    *reinterpret_cast<float *>(est + row * 256 + col * 4) = acc[mi][2 * h2 + nj][e];
                }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(big::wait_vm_lgkm0(63));   // LDS only: the wave reads back only what it wrote itself
        asm volatile("" ::: "memory");
        constexpr int BATCH = 8;
#pragma unroll
        for (int j0 = 0; j0 < NP; j0 += BATCH) {
            float4 v[BATCH], old[BATCH];
            bool live[BATCH];
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const int idx = (j0 + b) * 64 + lane, row = idx >> 4, c4 = idx & 15;
                const int m = m0 + 32 * WT * wm + row, n = n0 + 32 * WT * wn + 64 * h2 + 4 * c4;
                live[b] = m < M && n < N;   // N is a multiple of 16: the four columns are all in or all out
                const int mc = min(m, M - 1), nc = min(n, N - 4);
                v[b] = *reinterpret_cast<const float4 *>(est + row * 256 + c4 * 16);
                if (ACCUM) old[b] = *reinterpret_cast<const float4 *>(dW + (int64_t)mc * ldw + nc);
            }
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const int idx = (j0 + b) * 64 + lane, row = idx >> 4, c4 = idx & 15;
                const int m = m0 + 32 * WT * wm + row, n = n0 + 32 * WT * wn + 64 * h2 + 4 * c4;
                float4 o = v[b];
                if (ACCUM) { o.x = old[b].x + o.x; o.y = old[b].y + o.y; o.z = old[b].z + o.z; o.w = old[b].w + o.w; }
                if constexpr (DECAY) {
                    const uint2 w2 = wv[j0 + b];
                    const uint32_t kp = keep[j0 + b];
                    if (!(kp & 1u)) o.x = fmaf(lambda, s24_num<ET>::lo(w2.x), o.x);
                    if (!(kp & 2u)) o.y = fmaf(lambda, s24_num<ET>::hi(w2.x), o.y);
                    if (!(kp & 4u)) o.z = fmaf(lambda, s24_num<ET>::lo(w2.y), o.z);
                    if (!(kp & 8u)) o.w = fmaf(lambda, s24_num<ET>::hi(w2.y), o.w);
                }
                if (live[b]) *reinterpret_cast<float4 *>(dW + (int64_t)m * ldw + n) = o;
            }
            __builtin_amdgcn_sched_barrier(0);   // one batch at a time: hoisting the next batches' reads costs registers
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(big::wait_vm_lgkm0(63));   // LDS reads done before the other half overwrites
        asm volatile("" ::: "memory");
    }
}
}  // namespace dmatn

// ------------------------------------------------------------------ sparse TN (weight gradient from a pruned dY)
// dW[m][n] = sum_t A[m][t] X[t][n] with A = S_z(dY^T) compressed along the tokens (Eq. 4).  The compressed
// operand takes the sparse NT kernel's path (chunk-major values and index words copied into the same LDS
// layout, one 128-bit read per fragment), the token-major X tile takes the dense TN kernel's (rows of 512 bytes
// copied as they lie, fragments gathered with the transposing LDS read).  One sparse instruction covers the
// tokens {16h .. 16h+15} and {32+16h .. 32+16h+15} of a 64-token chunk (h = 0, 1), which is how the index
// words split over a lane pair; its dense fragment is therefore two 8-token runs 32 tokens apart.
// 256 x 256 tiles, eight waves of 128 (m) x 64 (n), ring of three 50 KB stages, fp32 output through LDS.
namespace sptn {
constexpr int BM = 256, BN = 256, THREADS = 512, ROWB = BN * 2, CPR = ROWB / 16;
constexpr int B_STAGE = 64 * ROWB, A_STAGE = BM * 64, M_STAGE = BM * 8, STAGE = B_STAGE + A_STAGE + M_STAGE;
using big::a_slot;
using big::glb_ptr;
using big::lds_ptr;

template <typename ET, bool ACCUM, bool DECAY>
__global__ __launch_bounds__(THREADS) void spmm_tn_big_kernel(const uint16_t *__restrict__ Av,
                                                              const uint16_t *__restrict__ Am,
                                                              const uint16_t *__restrict__ X, float *__restrict__ dW,
                                                              int T, int M, int N, int tiles_m, int tiles_n,
                                                              unsigned long long *probe, const uint16_t *__restrict__ Wt,
                                                              const uint16_t *__restrict__ mask, float lambda)
{
    const big::ClockStamp t_start = big::clock_now();
    __shared__ __attribute__((aligned(16))) unsigned char s0[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s1[STAGE];
    __shared__ __attribute__((aligned(16))) unsigned char s2[STAGE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int total = tiles_m * tiles_n, per_xcd = (total + 7) / 8;
    const int t = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (t >= total) return;
    constexpr int GROUP = 8;
    const int group_sz = GROUP * tiles_m, grp = t / group_sz, in_grp = t - grp * group_sz;
    const int gw = min(GROUP, tiles_n - grp * GROUP);
    const int tm = in_grp / gw, tn = grp * GROUP + in_grp % gw;
    const int m0 = tm * BM, n0 = tn * BN;
    const int nk = T / 64;

    // Copies per lane and chunk: four of the X tile (rows 8*wave .. 8*wave+7), two of the values, one index dword;
    // buffer loads into LDS with a wave-uniform base per operand and chunk and a fixed 32-bit byte offset per lane
    // (64 token rows of X and one chunk of the compressed operand span less than 4 GB: host check).
    const char *baseX = reinterpret_cast<const char *>(X), *baseV = reinterpret_cast<const char *>(Av);
    const char *baseM = reinterpret_cast<const char *>(Am);
    uint32_t ob[4], oa[2];
    const int lastB = (min(N - n0, BN) >> 3) - 1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int slot = (wave * 4 + j) * 64 + lane, row = slot / CPR, c = (slot % CPR) ^ ((row & 3) << 2);
        ob[j] = ((uint32_t)row * (uint32_t)N + (uint32_t)(n0 + 8 * min(c, lastB))) * 2u;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = 32 * wave + 16 * i + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        oa[i] = ((uint32_t)min(m0 + row, M - 1) * 32u + 8u * c) * 2u;
    }
    const uint32_t om = ((uint32_t)min(m0 + 32 * wave + (lane >> 1), M - 1) * 4u + 2u * (lane & 1)) * 2u;
    // exactly seven copies per lane and call; past the last chunk it re-reads the last one into a stage nobody
    // will read again, so that the wait counts below are constants
    auto issue = [&](unsigned char *st, int kc) {
        kc = min(kc, nk - 1);
        const big::rsrc_t px = big::buffer_of(baseX + (int64_t)kc * 128 * N), pv = big::buffer_of(baseV + (int64_t)kc * M * 64);
        const big::rsrc_t pm = big::buffer_of(baseM + (int64_t)kc * M * 8);
#pragma unroll
        for (int j = 0; j < 4; ++j) big::buffer_to_lds<16>(px, (lds_ptr)(st + (wave * 4 + j) * 1024), ob[j]);
#pragma unroll
        for (int i = 0; i < 2; ++i) big::buffer_to_lds<16>(pv, (lds_ptr)(st + B_STAGE + (32 * wave + 16 * i) * 64), oa[i]);
        big::buffer_to_lds<4>(pm, (lds_ptr)(st + B_STAGE + A_STAGE + 32 * wave * 8), om);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = f32x16{};

    // X fragment addressing: lane group G = lane/16 -> 8-token half G/2, column half G%2
    const int gi = lane & 15, G = lane >> 4, g = lane >> 5;
    const int frow = 8 * (G >> 1) + (gi >> 2), fcol = 16 * (G & 1) + 4 * (gi & 3);
    int offB[2];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) offB[ni] = dmatn::tr_off<ROWB>(frow, 64 * wn + 32 * ni + fcol);
    // Fragments of half h of a stage (the tokens {16h..16h+15} and {32+16h..} of the chunk): eight transposing
    // reads of the X tile and four 128-bit reads of the values
    auto load_frags = [&](const unsigned char *st, int h, bf16x16 (&b)[2], bf16x8 (&a)[4]) {
        const unsigned char *sb = st, *sa = st + B_STAGE;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            struct { bf16x8 lo, hi; } pair{dmatn::tr_frag<ROWB>(sb + offB[ni] + 16 * h * ROWB),
                                           dmatn::tr_frag<ROWB>(sb + offB[ni] + (32 + 16 * h) * ROWB)};
            b[ni] = __builtin_bit_cast(bf16x16, pair);
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
            a[mi] = as_bf16x8(*reinterpret_cast<const uint4 *>(sa + a_slot(128 * wm + 32 * mi + (lane & 31), 2 * g + h)));
    };
    auto load_index = [&](const unsigned char *st, uint32_t (&x)[4]) {
        const unsigned char *sm = st + B_STAGE + A_STAGE;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
            x[mi] = *reinterpret_cast<const uint32_t *>(sm + (128 * wm + 32 * mi + (lane & 31)) * 8 + 4 * g);
    };

    // keep the program order of these groups: the constant wait counts rely on it
    issue(s0, 0);
    __builtin_amdgcn_sched_barrier(0);
    issue(s1, 1);
    __builtin_amdgcn_sched_barrier(0);
    issue(s2, 2);
    __builtin_amdgcn_sched_barrier(0);
    big::wait_and_barrier<14>();   // chunk 0 has landed for everybody
    bf16x16 fb0[2];
    bf16x8 fa0[4];
    uint32_t ix[4];
    load_index(s0, ix);
    load_frags(s0, 0, fb0, fa0);

    // One chunk, pipelined across the workgroup barrier exactly as in the NT kernel: the first half's matrix
    // instructions run from registers while the second half's fragments come in; after the one barrier of the chunk
    // the second half's matrix instructions cover the next chunk's index words and first-half fragments and the
    // seven copies of chunk kc+3 into the stage just vacated.
    auto chunk = [&](unsigned char *cur, const unsigned char *nxt, int kc) {
        bf16x16 fb1[2];
        bf16x8 fa1[4];
        load_frags(cur, 1, fb1, fa1);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Mma<ET>::template sparse<0>(fa0[mi], fb0[ni], acc[mi][ni], (int)ix[mi]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {   // twelve reads, two per matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < 6) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        big::wait_and_barrier<7>();   // this lane's part of chunk kc+1 is in LDS, its own reads of chunk kc are done
        issue(cur, kc + 3);
        uint32_t ixn[4];
        load_index(nxt, ixn);
        load_frags(nxt, 0, fb0, fa0);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Mma<ET>::template sparse<1>(fa1[mi], fb1[ni], acc[mi][ni], (int)ix[mi]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {   // sixteen reads and seven copies
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            if (i < 7) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) ix[mi] = ixn[mi];
    };
    // past the last chunk the prefetched fragments come from a stage that holds a re-read of the last chunk (or is
    // being refilled with one); they are never multiplied
    int kc = 0;
    for (; kc + 3 <= nk; kc += 3) {
        chunk(s0, s1, kc);
        chunk(s1, s2, kc + 1);
        chunk(s2, s0, kc + 2);
    }
    if (kc < nk) chunk(s0, s1, kc);
    if (kc + 1 < nk) chunk(s1, s2, kc + 1);
    big::wait_and_barrier<0>();   // copies drained, nobody reads the ring any more: reuse it
    big::clock_report(probe, t_start);
    // fp32 output through LDS in 16-byte row segments: a wave parks 64 rows x 64 columns (two of its four row
    // blocks) at a time in 16 KB of the ring, lane l of pass j owns row (64j + l) / 16, columns 4 * (l % 16) .. +3
    static_assert(3 * 16384 <= STAGE, "three waves' staging areas per ring stage");
    unsigned char *est = (wave < 3 ? s0 : (wave < 6 ? s1 : s2)) + (wave % 3) * 16384;
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int mj = 0; mj < 2; ++mj)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = 32 * mj + 8 * (e / 4) + 4 * (lane >> 5) + (e & 3), col = 32 * ni + (lane & 31);
                    *reinterpret_cast<float *>(est + row * 256 + col * 4) = acc[2 * h2 + mj][ni][e];
                }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(big::wait_vm_lgkm0(0));   // the wave reads back only what it wrote itself
        asm volatile("" ::: "memory");
        constexpr int BATCH = 8;
#pragma unroll 1
        for (int j0 = 0; j0 < 16; j0 += BATCH) {
            float4 v[BATCH], old[BATCH];
            uint2 wv[BATCH];
            uint32_t keep[BATCH];
            bool live[BATCH];
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const int idx = (j0 + b) * 64 + lane, row = idx >> 4, c4 = idx & 15;
                const int m = m0 + 128 * wm + 64 * h2 + row, n = n0 + 64 * wn + 4 * c4;
                live[b] = m < M && n < N;   // N is a multiple of 16: the four columns are all in or all out
                const int mc = min(m, M - 1), nc = min(n, N - 4);
                v[b] = *reinterpret_cast<const float4 *>(est + row * 256 + c4 * 16);
                if (ACCUM) old[b] = *reinterpret_cast<const float4 *>(dW + (int64_t)mc * N + nc);
                if (DECAY) {
                    wv[b] = *reinterpret_cast<const uint2 *>(Wt + (int64_t)mc * N + nc);
                    keep[b] = mask[(int64_t)(mc >> 2) * (N >> 2) + (nc >> 2)] >> (4 * (mc & 3));
                }
            }
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const int idx = (j0 + b) * 64 + lane, row = idx >> 4, c4 = idx & 15;
                const int m = m0 + 128 * wm + 64 * h2 + row, n = n0 + 64 * wn + 4 * c4;
                float4 o = v[b];
                if (ACCUM) { o.x = old[b].x + o.x; o.y = old[b].y + o.y; o.z = old[b].z + o.z; o.w = old[b].w + o.w; }
                if (DECAY) {
                    if (!(keep[b] & 1u)) o.x = fmaf(lambda, s24_num<ET>::lo(wv[b].x), o.x);
                    if (!(keep[b] & 2u)) o.y = fmaf(lambda, s24_num<ET>::hi(wv[b].x), o.y);
                    if (!(keep[b] & 4u)) o.z = fmaf(lambda, s24_num<ET>::lo(wv[b].y), o.z);
                    if (!(keep[b] & 8u)) o.w = fmaf(lambda, s24_num<ET>::hi(wv[b].y), o.w);
                }
                if (live[b]) *reinterpret_cast<float4 *>(dW + (int64_t)m * N + n) = o;
            }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(big::wait_vm_lgkm0(0));   // LDS reads done before the other half overwrites
        asm volatile("" ::: "memory");
    }
}
}  // namespace sptn

// one thread per output, fp32 data (no fp32 sparse matrix instruction exists)
template <bool ACCUM>
__global__ __launch_bounds__(kThreads) void spmm_tn_f32_kernel(const float *__restrict__ Av, const uint16_t *__restrict__ Am,
                                                               const float *__restrict__ X, float *__restrict__ dW,
                                                               int64_t T, int64_t M, int64_t N)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N, n = idx - m * N;
    float acc = 0.0f;
    for (int64_t g = 0; g < T / 4; ++g) {
        const int64_t cr = (g / 16) * M + m;  // chunk-major storage: (chunk, row)
        const unsigned nib = (Am[cr * 4 + (g & 15) / 4] >> (4 * (g & 3))) & 0xFu;
        acc = fmaf(Av[cr * 32 + 2 * (g & 15)], X[(4 * g + (nib & 3u)) * N + n], acc);
        acc = fmaf(Av[cr * 32 + 2 * (g & 15) + 1], X[(4 * g + (nib >> 2)) * N + n], acc);
    }
    dW[idx] = ACCUM ? dW[idx] + acc : acc;
}

// ------------------------------------------------------------------ fp32 fallbacks (small correctness workload)
// One thread per output element, plain fp32 FMA; no matrix-core claim.
template <bool ACCUM>
__global__ __launch_bounds__(kThreads) void spmm_nt_f32_kernel(const float *__restrict__ B, const float *__restrict__ Av,
                                                               const uint16_t *__restrict__ Am, float *__restrict__ Out,
                                                               int64_t N, int64_t K, int64_t M, const float *__restrict__ bias)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= N * M) return;
    const int64_t n = idx / M, m = idx - n * M;
    float acc = 0.0f;
    for (int64_t g = 0; g < K / 4; ++g) {
        const int64_t cr = (g / 16) * M + m;  // chunk-major storage: (chunk, row)
        const unsigned nib = (Am[cr * 4 + (g & 15) / 4] >> (4 * (g & 3))) & 0xFu;
        acc = fmaf(Av[cr * 32 + 2 * (g & 15)], B[n * K + 4 * g + (nib & 3u)], acc);
        acc = fmaf(Av[cr * 32 + 2 * (g & 15) + 1], B[n * K + 4 * g + (nib >> 2)], acc);
    }
    if (bias != nullptr) acc += bias[m];
    Out[idx] = ACCUM ? Out[idx] + acc : acc;
}

__global__ __launch_bounds__(kThreads) void dense_nt_f32_kernel(const float *__restrict__ X, const float *__restrict__ W,
                                                                float *__restrict__ Y, int64_t N, int64_t K, int64_t M)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= N * M) return;
    const int64_t n = idx / M, m = idx - n * M;
    float acc = 0.0f;
    for (int64_t k = 0; k < K; ++k) acc = fmaf(X[n * K + k], W[m * K + k], acc);
    Y[idx] = acc;
}

template <bool ACCUM>
__global__ __launch_bounds__(kThreads) void dense_tn_f32_kernel(const float *__restrict__ dY, const float *__restrict__ X,
                                                                float *__restrict__ dW, int64_t T, int64_t M, int64_t N)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N, n = idx - m * N;
    float acc = 0.0f;
    for (int64_t t = 0; t < T; ++t) acc = fmaf(dY[t * M + m], X[t * N + n], acc);
    dW[idx] = ACCUM ? dW[idx] + acc : acc;
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float *__restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

inline unsigned ceil_div(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

unsigned long long *g_clock_probe = nullptr;   // device buffer of two counters, or none

// dtype and sizes first; pointers are only required when the output is not empty.
int check_gemm(const void *a, const void *b, const void *c, int64_t p, int64_t q, int64_t r, int dt, int64_t out_elems)
{
    S24_REQUIRE(s24_valid_dtype(dt), S24_ERR_DTYPE);
    S24_REQUIRE(p >= 0 && q >= 0 && r >= 0, S24_ERR_SHAPE);
    S24_REQUIRE(p < (1ll << 31) && q < (1ll << 31) && r < (1ll << 31), S24_ERR_SHAPE);
    // the large-tile kernels address a tile's operand rows with 32-bit byte offsets from a per-tile base:
    // 256 rows of the contraction axis, and all rows of one 64-chunk of a compressed operand, must span < 4 GB
    S24_REQUIRE(q < (1ll << 23) && r < (1ll << 23), S24_ERR_SHAPE);
    if (out_elems == 0) return S24_OK;
    S24_REQUIRE(a && b && c, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(a, 16) && s24_aligned(b, 16) && s24_aligned(c, 16), S24_ERR_ALIGN);
    return S24_OK;
}

// Runs `...` with T bound to the storage type of a 16-bit dtype.
#define S24_WITH_16BIT_TYPE(dt, ...)      \
    do {                                  \
        if ((dt) == S24_BF16) {           \
            using T = uint16_t;           \
            __VA_ARGS__;                  \
        } else {                          \
            using T = s24_half;           \
            __VA_ARGS__;                  \
        }                                 \
    } while (0)

// Compute units of the current device, read once (256 on MI355X; that figure also stands in where no device
// answers, so that the host-side checks behave the same without a GPU).
inline int s24_cu_count()
{
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            return v;
        return 256;
    }();
    return n;
}
inline bool fills_chip_256(int64_t m, int64_t n) { return (int64_t)ceil_div(m, 256) * ceil_div(n, 256) >= 3 * s24_cu_count() / 4; }

// Large tile (256 x 256, one workgroup per compute unit) or small tile (128 x 128, two per compute unit)?  The small
// tile moves twice the bytes per FLOP through L2, so it only pays where the large one leaves compute units idle (few
// tiles, or a last round that is mostly empty) or where the contraction is so short that a tile is mostly prologue
// and epilogue, which two co-resident workgroups overlap with each other's main loops.  Cost model in rounds of the
// large tile: a small-tile round (twice as many workgroups, half the work) takes 0.75 of a large one, 0.6 when the
// contraction is at most 1024 deep (measured: at K = 768 a large tile spends more time filling and draining than multiplying).
inline bool small_tile_pays(int64_t M, int64_t N, int64_t K)
{
    const int cus = s24_cu_count();
    const int64_t t256 = (int64_t)ceil_div(M, 256) * ceil_div(N, 256), t128 = (int64_t)ceil_div(M, 128) * ceil_div(N, 128);
    const double round_small = K <= 1024 ? 0.6 : 0.75;
    return round_small * (double)ceil_div(t128, 2 * cus) < (double)ceil_div(t256, cus);
}

// A grid of large tiles whose last round is mostly empty (320 tiles on 256 compute units: two rounds for 1.25 rounds
// of work) can give its last token-tile rows to the small tile instead: the first `slab` tokens run in whole rounds of
// large tiles, the rest as one resident set of small tiles.  Returns the slab's token count, or 0 where the cost
// model above does not favour the cut.  Tokens are independent rows of the product, so the result does not change.
inline int64_t large_tile_slab_tokens(int64_t M, int64_t N, int64_t K)
{
    const int cus = s24_cu_count();
    const int64_t tm = ceil_div(M, 256), tiles = tm * ceil_div(N, 256), rounds = (tiles + cus - 1) / cus;
    if (tiles <= cus || tiles % cus == 0 || tm > cus) return 0;
    const int64_t rows = ((rounds - 1) * cus) / tm, slab = 256 * rows;   // whole token-tile rows within rounds - 1 rounds
    const int64_t strip_tiles = (int64_t)ceil_div(M, 128) * ceil_div(N - slab, 128);
    const double round_small = K <= 1024 ? 0.6 : 0.75;
    const double cost = (double)ceil_div(rows * tm, cus) + round_small * (double)ceil_div(strip_tiles, 2 * cus);
    return cost < (double)rounds ? slab : 0;
}

// Out[N][M] = beta * Out + B[N][K] . A^T (+ bias[M], only with beta = 0)
int launch_spmm(const void *B, const void *Av, const uint16_t *Am, void *Out, int64_t N, int64_t K, int64_t M, float beta,
                int dt, hipStream_t st, const void *bias = nullptr)
{
    if (N == 0 || M == 0) return S24_OK;
    const bool accum = beta != 0.0f;
    if (dt == S24_F32) {
        const dim3 grid(ceil_div(N * M, kThreads)), block(kThreads);
        auto *b = static_cast<const float *>(B), *av = static_cast<const float *>(Av);
        auto *o = static_cast<float *>(Out);
        auto *d = static_cast<const float *>(bias);
        if (accum) hipLaunchKernelGGL(spmm_nt_f32_kernel<true>, grid, block, 0, st, b, av, Am, o, N, K, M, d);
        else hipLaunchKernelGGL(spmm_nt_f32_kernel<false>, grid, block, 0, st, b, av, Am, o, N, K, M, d);
        return s24_launch_status();
    }
    auto *b = static_cast<const uint16_t *>(B), *av = static_cast<const uint16_t *>(Av), *d = static_cast<const uint16_t *>(bias);
    auto *o = static_cast<uint16_t *>(Out);
    const int tm256 = (int)ceil_div(M, 256), tn256 = (int)ceil_div(N, 256), tm128 = (int)ceil_div(M, 128), tn128 = (int)ceil_div(N, 128);
    S24_REQUIRE((int64_t)tm128 * tn128 < (1ll << 30), S24_ERR_SHAPE);
    if (!small_tile_pays(M, N, K)) {
        if (const int64_t slab = large_tile_slab_tokens(M, N, K)) {
            const int rc = launch_spmm(B, Av, Am, Out, slab, K, M, beta, dt, st, bias);
            if (rc != S24_OK) return rc;
            return launch_spmm(b + slab * K, Av, Am, o + slab * M, N - slab, K, M, beta, dt, st, bias);
        }
        const int tiles_m = tm256, tiles_n = tn256;
        const int per_xcd = (tiles_m * tiles_n + 7) / 8;
        const dim3 grid(per_xcd * 8), block(big::THREADS);
        S24_WITH_16BIT_TYPE(dt, {
            if (accum)
                hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, true>), grid, block, 0, st, b, av, Am, o, (int)N, (int)K, (int)M,
                                   tiles_m, tiles_n, g_clock_probe, nullptr, 0, nullptr, nullptr);
            else if (d != nullptr)
                hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, false, false, S24_GATE_SILU, true>), grid, block, 0, st, b,
                                   av, Am, o, (int)N, (int)K, (int)M, tiles_m, tiles_n, g_clock_probe, nullptr, 0, nullptr, d);
            else
                hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false>), grid, block, 0, st, b, av, Am, o, (int)N, (int)K, (int)M,
                                   tiles_m, tiles_n, g_clock_probe, nullptr, 0, nullptr, nullptr);
        });
    } else {
        const int tiles_m = tm128, tiles_n = tn128;
        const int per_xcd = (tiles_m * tiles_n + 7) / 8;
        const dim3 grid(per_xcd * 8), block(256);
        S24_WITH_16BIT_TYPE(dt, {
            if (accum)
                hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, true, false, false, S24_GATE_SILU, false, 0, S24_ACT_RELU, 2>), grid,
                                   block, 0, st, b, av, Am, o, (int)N, (int)K, (int)M, tiles_m, tiles_n, nullptr, nullptr, 0,
                                   nullptr, nullptr);
            else if (d != nullptr)
                hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, false, false, S24_GATE_SILU, true, 0, S24_ACT_RELU, 2>), grid,
                                   block, 0, st, b, av, Am, o, (int)N, (int)K, (int)M, tiles_m, tiles_n, nullptr, nullptr, 0,
                                   nullptr, d);
            else
                hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, false, false, S24_GATE_SILU, false, 0, S24_ACT_RELU, 2>), grid,
                                   block, 0, st, b, av, Am, o, (int)N, (int)K, (int)M, tiles_m, tiles_n, nullptr, nullptr, 0,
                                   nullptr, nullptr);
        });
    }
    return s24_launch_status();
}

}  // namespace

extern "C" int s24_spmm_fwd(const void *X, const void *vals, const uint16_t *meta, void *Y, int64_t p, int64_t q, int64_t r,
                            s24_dtype dt, void *stream)
{
    return s24_spmm_fwd_bias(X, vals, meta, nullptr, Y, p, q, r, dt, stream);
}

extern "C" int s24_spmm_fwd_bias(const void *X, const void *vals, const uint16_t *meta, const void *bias, void *Y, int64_t p,
                                 int64_t q, int64_t r, s24_dtype dt, void *stream)
{
    S24_REQUIRE(q % 64 == 0 && r % 16 == 0 && q > 0, S24_ERR_SHAPE);
    const int rc = check_gemm(X, vals, Y, p, q, r, dt, p * r);
    if (rc != S24_OK || p * r == 0) return rc;
    S24_REQUIRE(meta != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(meta, 4) && s24_aligned(bias, 8), S24_ERR_ALIGN);
    return launch_spmm(X, vals, meta, Y, p, q, r, 0.0f, dt, static_cast<hipStream_t>(stream), bias);
}

extern "C" int s24_spmm_bwd_dx(const void *dY, const void *valsT, const uint16_t *metaT, void *dX, int64_t p, int64_t q,
                               int64_t r, float beta, s24_dtype dt, void *stream)
{
    S24_REQUIRE(r % 64 == 0 && q % 16 == 0 && r > 0, S24_ERR_SHAPE);
    S24_REQUIRE(beta == 0.0f || beta == 1.0f, S24_ERR_UNSUPPORTED);
    const int rc = check_gemm(dY, valsT, dX, p, q, r, dt, p * q);
    if (rc != S24_OK || p * q == 0) return rc;
    S24_REQUIRE(metaT != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(metaT, 4), S24_ERR_ALIGN);
    return launch_spmm(dY, valsT, metaT, dX, p, r, q, beta, dt, static_cast<hipStream_t>(stream));
}

extern "C" int s24_spmm_fwd_glu(const void *X, const void *vals, const uint16_t *meta, const void *bias, void *GU, void *H,
                                int64_t p, int64_t q, int64_t f, s24_gate gate, s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_gate(gate), S24_ERR_DTYPE);
    S24_REQUIRE(q % 64 == 0 && f % 16 == 0 && q > 0, S24_ERR_SHAPE);
    const int rc = check_gemm(X, vals, GU, p, q, 2 * f, dt, p * f);
    if (rc != S24_OK || p * f == 0) return rc;
    S24_REQUIRE(meta != nullptr && H != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(meta, 4) && s24_aligned(H, 16) && s24_aligned(bias, 8), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int tiles_m = (int)ceil_div(f, 128), tiles_n = (int)ceil_div(p, big::BN);
    if (dt != S24_F32 && (int64_t)tiles_m * tiles_n >= 3 * s24_cu_count() / 4) {
        const dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8), block(big::THREADS);
        auto *x = static_cast<const uint16_t *>(X), *av = static_cast<const uint16_t *>(vals), *d = static_cast<const uint16_t *>(bias);
        auto *gu = static_cast<uint16_t *>(GU), *h = static_cast<uint16_t *>(H);
#define S24_LAUNCH_FWD_GLU(G)                                                                                              \
    hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, true, false, G>), grid, block, 0, st, x, av, meta, gu, (int)p, \
                       (int)q, (int)(2 * f), tiles_m, tiles_n, g_clock_probe, h, (int)f, nullptr, d)
        S24_WITH_16BIT_TYPE(dt, {
            if (gate == S24_GATE_SILU) S24_LAUNCH_FWD_GLU(S24_GATE_SILU);
            else S24_LAUNCH_FWD_GLU(S24_GATE_GELU_ERF);
        });
#undef S24_LAUNCH_FWD_GLU
        return s24_launch_status();
    }
    // shapes the fused epilogue does not cover: the GEMM into [p][2f], then the stand-alone activation on its halves
    const int rc2 = launch_spmm(X, vals, meta, GU, p, q, 2 * f, 0.0f, dt, st, bias);
    if (rc2 != S24_OK) return rc2;
    return s24_glu_fwd(GU, S24_ROW_MAJOR, 2 * f, H, S24_ROW_MAJOR, f, p, f, gate, dt, st);
}

extern "C" int s24_spmm_fwd_swiglu(const void *X, const void *vals, const uint16_t *meta, void *GU, void *H, int64_t p,
                                   int64_t q, int64_t f, s24_dtype dt, void *stream)
{
    return s24_spmm_fwd_glu(X, vals, meta, nullptr, GU, H, p, q, f, S24_GATE_SILU, dt, stream);
}

extern "C" int s24_spmm_bwd_dx_glu(const void *dY, const void *valsT, const uint16_t *metaT, const void *GU, void *dGU,
                                   int64_t p, int64_t f, int64_t r, s24_gate gate, s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_gate(gate), S24_ERR_DTYPE);
    S24_REQUIRE(r % 64 == 0 && f % 16 == 0 && r > 0, S24_ERR_SHAPE);
    const int rc = check_gemm(dY, valsT, dGU, p, f, r, dt, p * f);
    if (rc != S24_OK || p * f == 0) return rc;
    S24_REQUIRE(metaT != nullptr && GU != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(metaT, 4) && s24_aligned(GU, 16), S24_ERR_ALIGN);
    const int tiles_m = (int)ceil_div(f, big::BM), tiles_n = (int)ceil_div(p, big::BN);
    // only the large-tile 16-bit kernel carries this epilogue; other shapes take s24_spmm_bwd_dx + s24_glu_bwd
    S24_REQUIRE(dt != S24_F32 && (int64_t)tiles_m * tiles_n >= 3 * s24_cu_count() / 4, S24_ERR_UNSUPPORTED);
    const dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8), block(big::THREADS);
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto *dy = static_cast<const uint16_t *>(dY), *av = static_cast<const uint16_t *>(valsT), *gu = static_cast<const uint16_t *>(GU);
    auto *o = static_cast<uint16_t *>(dGU);
#define S24_LAUNCH_BWD_GLU(G)                                                                                              \
    hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, false, true, G>), grid, block, 0, st, dy, av, metaT, o, (int)p, \
                       (int)r, (int)f, tiles_m, tiles_n, g_clock_probe, nullptr, 0, gu, nullptr)
    S24_WITH_16BIT_TYPE(dt, {
        if (gate == S24_GATE_SILU) S24_LAUNCH_BWD_GLU(S24_GATE_SILU);
        else S24_LAUNCH_BWD_GLU(S24_GATE_GELU_ERF);
    });
#undef S24_LAUNCH_BWD_GLU
    return s24_launch_status();
}

extern "C" int s24_spmm_bwd_dx_swiglu(const void *dY, const void *valsT, const uint16_t *metaT, const void *GU, void *dGU,
                                      int64_t p, int64_t f, int64_t r, s24_dtype dt, void *stream)
{
    return s24_spmm_bwd_dx_glu(dY, valsT, metaT, GU, dGU, p, f, r, S24_GATE_SILU, dt, stream);
}

extern "C" int s24_spmm_fwd_act(const void *X, const void *vals, const uint16_t *meta, const void *bias, void *Z, void *H,
                                int64_t p, int64_t q, int64_t r, s24_act act, s24_dtype dt, void *stream)
{
    S24_REQUIRE(act == S24_ACT_RELU || act == S24_ACT_GELU_ERF, S24_ERR_DTYPE);
    S24_REQUIRE(q % 64 == 0 && r % 16 == 0 && q > 0, S24_ERR_SHAPE);
    const int rc = check_gemm(X, vals, Z, p, q, r, dt, p * r);
    if (rc != S24_OK || p * r == 0) return rc;
    S24_REQUIRE(meta != nullptr && H != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(meta, 4) && s24_aligned(H, 16) && s24_aligned(bias, 8), S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt != S24_F32) {
        const bool small = small_tile_pays(r, p, q);
        const int tile = small ? 128 : 256;
        const int tiles_m = (int)ceil_div(r, tile), tiles_n = (int)ceil_div(p, tile);
        S24_REQUIRE((int64_t)tiles_m * tiles_n < (1ll << 30), S24_ERR_SHAPE);
        const dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8), block(small ? 256 : big::THREADS);
        auto *x = static_cast<const uint16_t *>(X), *av = static_cast<const uint16_t *>(vals), *d = static_cast<const uint16_t *>(bias);
        auto *z = static_cast<uint16_t *>(Z), *h = static_cast<uint16_t *>(H);
#define S24_LAUNCH_FWD_ACT_MI(A, BIASED, MI_)                                                                                       \
    hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, false, false, S24_GATE_SILU, BIASED, 1, A, MI_>), grid, block, 0, st, x, \
                       av, meta, z, (int)p, (int)q, (int)r, tiles_m, tiles_n, small ? nullptr : g_clock_probe, h, 0, nullptr, d)
#define S24_LAUNCH_FWD_ACT(A, BIASED)                 \
    do {                                              \
        if (small) S24_LAUNCH_FWD_ACT_MI(A, BIASED, 2); \
        else S24_LAUNCH_FWD_ACT_MI(A, BIASED, 4);     \
    } while (0)
        S24_WITH_16BIT_TYPE(dt, {
            if (act == S24_ACT_RELU && d != nullptr) S24_LAUNCH_FWD_ACT(S24_ACT_RELU, true);
            else if (act == S24_ACT_RELU) S24_LAUNCH_FWD_ACT(S24_ACT_RELU, false);
            else if (d != nullptr) S24_LAUNCH_FWD_ACT(S24_ACT_GELU_ERF, true);
            else S24_LAUNCH_FWD_ACT(S24_ACT_GELU_ERF, false);
        });
#undef S24_LAUNCH_FWD_ACT
#undef S24_LAUNCH_FWD_ACT_MI
        return s24_launch_status();
    }
    // fp32: the GEMM, then the stand-alone activation
    const int rc2 = launch_spmm(X, vals, meta, Z, p, q, r, 0.0f, dt, st, bias);
    if (rc2 != S24_OK) return rc2;
    return s24_act_fwd(Z, H, p * r, act, dt, st);
}

extern "C" int s24_spmm_bwd_dx_act(const void *dY, const void *valsT, const uint16_t *metaT, const void *Z, void *dZ,
                                   int64_t p, int64_t f, int64_t r, s24_act act, s24_dtype dt, void *stream)
{
    S24_REQUIRE(act == S24_ACT_RELU || act == S24_ACT_GELU_ERF, S24_ERR_DTYPE);
    S24_REQUIRE(r % 64 == 0 && f % 16 == 0 && r > 0, S24_ERR_SHAPE);
    const int rc = check_gemm(dY, valsT, dZ, p, f, r, dt, p * f);
    if (rc != S24_OK || p * f == 0) return rc;
    S24_REQUIRE(metaT != nullptr && Z != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(metaT, 4) && s24_aligned(Z, 16), S24_ERR_ALIGN);
    // the 16-bit kernels carry this epilogue; fp32 takes s24_spmm_bwd_dx + s24_act_bwd
    S24_REQUIRE(dt != S24_F32, S24_ERR_UNSUPPORTED);
    const bool small = small_tile_pays(f, p, r);
    const int tile = small ? 128 : 256;
    const int tiles_m = (int)ceil_div(f, tile), tiles_n = (int)ceil_div(p, tile);
    S24_REQUIRE((int64_t)tiles_m * tiles_n < (1ll << 30), S24_ERR_SHAPE);
    const dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8), block(small ? 256 : big::THREADS);
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto *dy = static_cast<const uint16_t *>(dY), *av = static_cast<const uint16_t *>(valsT), *z = static_cast<const uint16_t *>(Z);
    auto *o = static_cast<uint16_t *>(dZ);
#define S24_LAUNCH_BWD_ACT_MI(A, MI_)                                                                                                 \
    hipLaunchKernelGGL((big::spmm_nt_big_kernel<T, false, false, false, S24_GATE_SILU, false, 2, A, MI_>), grid, block, 0, st, dy, av, \
                       metaT, o, (int)p, (int)r, (int)f, tiles_m, tiles_n, small ? nullptr : g_clock_probe, nullptr, 0, z, nullptr)
#define S24_LAUNCH_BWD_ACT(A)                   \
    do {                                        \
        if (small) S24_LAUNCH_BWD_ACT_MI(A, 2); \
        else S24_LAUNCH_BWD_ACT_MI(A, 4);       \
    } while (0)
    S24_WITH_16BIT_TYPE(dt, {
        if (act == S24_ACT_RELU) S24_LAUNCH_BWD_ACT(S24_ACT_RELU);
        else S24_LAUNCH_BWD_ACT(S24_ACT_GELU_ERF);
    });
#undef S24_LAUNCH_BWD_ACT
#undef S24_LAUNCH_BWD_ACT_MI
    return s24_launch_status();
}

extern "C" int s24_dense_gemm(const void *X, const void *W, void *Y, int64_t p, int64_t q, int64_t r, s24_dtype dt,
                              void *stream)
{
    S24_REQUIRE(q % 64 == 0 && r % 16 == 0 && q > 0, S24_ERR_SHAPE);
    const int rc = check_gemm(X, W, Y, p, q, r, dt, p * r);
    if (rc != S24_OK || p * r == 0) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == S24_F32) {
        hipLaunchKernelGGL(dense_nt_f32_kernel, dim3(ceil_div(p * r, kThreads)), dim3(kThreads), 0, st,
                           static_cast<const float *>(X), static_cast<const float *>(W), static_cast<float *>(Y), p, q, r);
        return s24_launch_status();
    }
    auto *x = static_cast<const uint16_t *>(X), *w = static_cast<const uint16_t *>(W);
    auto *y = static_cast<uint16_t *>(Y);
    if (fills_chip_256(r, p)) {
        const int tiles_m = (int)ceil_div(r, bignt::BM), tiles_n = (int)ceil_div(p, bignt::BN);
        S24_WITH_16BIT_TYPE(dt, hipLaunchKernelGGL(bignt::dense_nt_big_kernel<T>, dim3(((tiles_m * tiles_n + 7) / 8) * 8),
                                                   dim3(bignt::THREADS), 0, st, x, w, y, (int)p, (int)q, (int)r, tiles_m,
                                                   tiles_n, g_clock_probe));
    } else {
        const dim3 grid(ceil_div(r, BM), ceil_div(p, BN)), block(kThreads);
        S24_REQUIRE(grid.y <= 65535, S24_ERR_SHAPE);
        S24_WITH_16BIT_TYPE(dt, hipLaunchKernelGGL(dense_nt_kernel<T>, grid, block, 0, st, x, w, y, (int)p, (int)q, (int)r));
    }
    return s24_launch_status();
}

namespace {
// One weight gradient as the batched kernel sees it (16-bit operands; W == nullptr: no decay term)
struct DwProblem {
    const uint16_t *dY, *X;
    float *dW;
    const uint16_t *W, *mask;
    int64_t p, q, r;
    float lambda;
};
// The window [m_off, m_off + mm) x [n_off, n_off + nn) of a problem's output, in tiles of `tile`
dmatn::DwWindow dw_window(const DwProblem &pr, int tile, int64_t m_off, int64_t mm, int64_t n_off, int64_t nn)
{
    dmatn::DwWindow w{};
    w.dY = pr.dY + m_off;
    w.X = pr.X + n_off;
    w.dW = pr.dW + m_off * pr.q + n_off;
    w.Wt = pr.W ? pr.W + m_off * pr.q + n_off : nullptr;
    w.mask = pr.W ? pr.mask + (m_off / 4) * (pr.q / 4) + n_off / 4 : nullptr;
    w.T = (int)pr.p;
    w.M = (int)mm;
    w.N = (int)nn;
    w.ldy = (int)pr.r;
    w.ldx = (int)pr.q;
    w.ldw = (int)pr.q;
    w.tiles_m = (int)ceil_div(mm, tile);
    w.tiles_n = (int)ceil_div(nn, tile);
    w.lambda = pr.lambda;
    return w;
}
// tile: 256 (large), or 128 (small; 32 tokens per stage when there are more tiles than compute units, else 64)
void launch_dw_batch(const dmatn::DwBatch &batch, int tile, bool accum, bool decay, int dt, hipStream_t st)
{
    const int slots = batch.first_slot[dmatn::kMaxBatch];   // per XCD
    const dim3 grid(slots * 8), block(dmatn::THREADS);
#define S24_LAUNCH_DW(WT, BT, ACC, DEC) \
    hipLaunchKernelGGL((dmatn::dense_tn_dma_kernel<T, WT, BT, ACC, DEC>), grid, block, 0, st, batch, g_clock_probe)
#define S24_LAUNCH_DW_TILE(WT, BT)                               \
    do {                                                         \
        if (accum && decay) S24_LAUNCH_DW(WT, BT, true, true);   \
        else if (accum) S24_LAUNCH_DW(WT, BT, true, false);      \
        else if (decay) S24_LAUNCH_DW(WT, BT, false, true);      \
        else S24_LAUNCH_DW(WT, BT, false, false);                \
    } while (0)
    S24_WITH_16BIT_TYPE(dt, {
        if (tile == 256) S24_LAUNCH_DW_TILE(4, 32);
        else if (slots * 8 > s24_cu_count()) S24_LAUNCH_DW_TILE(2, 32);
        else S24_LAUNCH_DW_TILE(2, 64);
    });
#undef S24_LAUNCH_DW_TILE
#undef S24_LAUNCH_DW
}

// Shared by s24_dense_dw and s24_dense_dw_decay.  W == nullptr: no decay term.
int run_dense_dw(const void *dY, const void *X, float *dW, int64_t p, int64_t q, int64_t r, float beta, int dt,
                 const void *W, int wdt, const uint16_t *mask, float lambda, hipStream_t st)
{
    const bool accum = beta != 0.0f;
    bool decay_pending = W != nullptr;
    if (p == 0) {  // empty contraction: dW = beta * dW (the GEMM kernels need at least one token)
        if (!accum) hipLaunchKernelGGL(fill_zero_kernel, dim3(ceil_div(q * r, kThreads)), dim3(kThreads), 0, st, dW, q * r);
    } else if (dt != S24_F32) {
        auto *a = static_cast<const uint16_t *>(dY), *b = static_cast<const uint16_t *>(X);
        const bool fuse = decay_pending && wdt == dt;   // the epilogue reads W in the operands' own 16-bit type
        auto *w = static_cast<const uint16_t *>(fuse ? W : nullptr);
        // One launch over the window [m_off, m_off + mm) x [n_off, n_off + nn) of the output, in tiles of `tile`
        auto launch = [&](int tile, int64_t m_off, int64_t mm, int64_t n_off, int64_t nn) {
            const DwProblem pr{a, b, dW, w, fuse ? mask : nullptr, p, q, r, lambda};
            dmatn::DwBatch batch{};
            batch.w[0] = dw_window(pr, tile, m_off, mm, n_off, nn);
            const int slots = (batch.w[0].tiles_m * batch.w[0].tiles_n + 7) / 8;
            for (int i = 1; i <= dmatn::kMaxBatch; ++i) batch.first_slot[i] = slots;
            launch_dw_batch(batch, tile, accum, fuse, dt, st);
        };
        // 256 x 256 tiles when they fill the chip, 128 x 128 tiles otherwise.  A grid of large tiles that is not a
        // whole number of rounds over the 256 compute units leaves the chip part empty in its last round (c4's
        // 1376 tiles: 5.375 rounds).  Where whole tile rows or columns can be cut off so that the rest is an exact
        // number of rounds and the cut-off strip is at most half a round of large tiles, the slab runs in large
        // tiles and the strip in small ones (at most 512 of them: one resident set, two workgroups per compute
        // unit), which costs 0.56 of a round instead of a whole one; a longer strip (c4's other weight, 0.69 of a
        // round) measured no better than the idle tail it replaces and stays in the single launch.  Every output
        // element belongs to exactly one launch either way, so nothing about the result changes.
        const int tm256 = (int)ceil_div(r, 256), tn256 = (int)ceil_div(q, 256), total = tm256 * tn256;
        const int cus = s24_cu_count();
        if (total < 3 * cus / 4) {
            launch(128, 0, r, 0, q);
        } else {
            int cut_m = 0, cut_n = 0;   // tile rows / columns kept in the large-tile slab (0: no such cut)
            if (total % cus != 0) {
                for (int k = tm256 - 1; k >= 1 && !cut_m; --k)
                    if ((k * tn256) % cus == 0 && (tm256 - k) * tn256 <= cus / 2) cut_m = k;
                for (int k = tn256 - 1; k >= 1 && !cut_n; --k)
                    if ((k * tm256) % cus == 0 && (tn256 - k) * tm256 <= cus / 2) cut_n = k;
            }
            if (cut_m && (!cut_n || cut_m * tn256 >= cut_n * tm256)) {
                launch(256, 0, 256ll * cut_m, 0, q);
                launch(128, 256ll * cut_m, r - 256ll * cut_m, 0, q);
            } else if (cut_n) {
                launch(256, 0, r, 0, 256ll * cut_n);
                launch(128, 0, r, 256ll * cut_n, q - 256ll * cut_n);
            } else {
                launch(256, 0, r, 0, q);
            }
        }
        if (fuse) decay_pending = false;
    } else {
        const dim3 grid(ceil_div(r * q, kThreads)), block(kThreads);
        auto *a = static_cast<const float *>(dY), *b = static_cast<const float *>(X);
        if (accum) hipLaunchKernelGGL(dense_tn_f32_kernel<true>, grid, block, 0, st, a, b, dW, p, r, q);
        else hipLaunchKernelGGL(dense_tn_f32_kernel<false>, grid, block, 0, st, a, b, dW, p, r, q);
    }
    const int rc = s24_launch_status();
    if (rc != S24_OK || !decay_pending) return rc;
    // shapes the fused epilogue does not cover: the stand-alone decay kernel on the finished gradient
    return s24_masked_decay_grad(dW, W, static_cast<s24_dtype>(wdt), mask, lambda, r, q, st);
}
}  // namespace

extern "C" int s24_dense_dw(const void *dY, const void *X, float *dW, int64_t p, int64_t q, int64_t r, float beta,
                            s24_dtype dt, void *stream)
{
    S24_REQUIRE(q % 16 == 0 && r % 16 == 0, S24_ERR_SHAPE);
    S24_REQUIRE(beta == 0.0f || beta == 1.0f, S24_ERR_UNSUPPORTED);
    const int rc = check_gemm(dY, X, dW, p, q, r, dt, q * r);
    if (rc != S24_OK || q * r == 0) return rc;
    return run_dense_dw(dY, X, dW, p, q, r, beta, dt, nullptr, dt, nullptr, 0.0f, static_cast<hipStream_t>(stream));
}

extern "C" int s24_dense_dw_decay(const void *dY, const void *X, float *dW, const void *W, s24_dtype wdt,
                                  const uint16_t *mask, float lambda, int64_t p, int64_t q, int64_t r, float beta,
                                  s24_dtype dt, void *stream)
{
    S24_REQUIRE(q % 16 == 0 && r % 16 == 0, S24_ERR_SHAPE);
    S24_REQUIRE(beta == 0.0f || beta == 1.0f, S24_ERR_UNSUPPORTED);
    S24_REQUIRE(s24_valid_dtype(wdt), S24_ERR_DTYPE);
    const int rc = check_gemm(dY, X, dW, p, q, r, dt, q * r);
    if (rc != S24_OK || q * r == 0) return rc;
    S24_REQUIRE(W && mask, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(W, 16) && s24_aligned(mask, 4), S24_ERR_ALIGN);
    return run_dense_dw(dY, X, dW, p, q, r, beta, dt, W, wdt, mask, lambda, static_cast<hipStream_t>(stream));
}

extern "C" int s24_dense_dw_batch(const s24_dw_problem *problems, int count, float beta, s24_dtype dt, void *stream)
{
    S24_REQUIRE(s24_valid_dtype(dt), S24_ERR_DTYPE);
    S24_REQUIRE(count >= 0 && count <= dmatn::kMaxBatch, S24_ERR_SHAPE);
    S24_REQUIRE(beta == 0.0f || beta == 1.0f, S24_ERR_UNSUPPORTED);
    if (count == 0) return S24_OK;
    S24_REQUIRE(problems != nullptr, S24_ERR_NULL);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // every problem is checked before anything is launched
    bool shared_grid = dt != S24_F32;
    int64_t total = 0;
    for (int i = 0; i < count; ++i) {
        const s24_dw_problem &pr = problems[i];
        S24_REQUIRE(pr.q % 16 == 0 && pr.r % 16 == 0, S24_ERR_SHAPE);
        const int rc = check_gemm(pr.dY, pr.X, pr.dW, pr.p, pr.q, pr.r, dt, pr.q * pr.r);
        if (rc != S24_OK) return rc;
        if (pr.W != nullptr && pr.q * pr.r != 0) {
            S24_REQUIRE(pr.mask != nullptr, S24_ERR_NULL);
            S24_REQUIRE(s24_aligned(pr.W, 16) && s24_aligned(pr.mask, 4), S24_ERR_ALIGN);
        }
        const int64_t tiles = (int64_t)ceil_div(pr.r, 256) * ceil_div(pr.q, 256);
        // one grid for all of them: 16-bit data, tokens to contract, every problem large enough for the large tile,
        // and the decay term on all of them or on none
        shared_grid = shared_grid && pr.p > 0 && tiles >= 64 && (pr.W != nullptr) == (problems[0].W != nullptr);
        total += tiles;
    }
    const bool accum = beta != 0.0f, decay = problems[0].W != nullptr;
    DwProblem prs[dmatn::kMaxBatch];
    for (int i = 0; i < count; ++i) {
        const s24_dw_problem &pr = problems[i];
        prs[i] = DwProblem{static_cast<const uint16_t *>(pr.dY), static_cast<const uint16_t *>(pr.X), pr.dW,
                           static_cast<const uint16_t *>(pr.W), pr.mask, pr.p, pr.q, pr.r, pr.lambda};
    }
    const int cus = s24_cu_count();
    if (!shared_grid || total < 3 * cus / 4 || count == 1) {
        // Problems that would each run in small tiles anyway (fewer than 192 large ones) share one small-tile grid:
        // a GPT-2-small layer's two gradients are 144 small tiles each, 0.56 of the chip one after the other.
        bool small_grid = dt != S24_F32 && count > 1;
        for (int i = 0; i < count; ++i) {
            const s24_dw_problem &pr = problems[i];
            small_grid = small_grid && pr.p > 0 && pr.q * pr.r != 0 && (pr.W != nullptr) == decay &&
                         (int64_t)ceil_div(pr.r, 256) * ceil_div(pr.q, 256) < 3 * cus / 4;
        }
        if (small_grid) {
            dmatn::DwBatch batch{};
            int first = 0;
            for (int i = 0; i < count; ++i) {
                batch.w[i] = dw_window(prs[i], 128, 0, prs[i].r, 0, prs[i].q);
                batch.first_slot[i] = first;
                first += (batch.w[i].tiles_m * batch.w[i].tiles_n + 7) / 8;
            }
            for (int i = count; i <= dmatn::kMaxBatch; ++i) batch.first_slot[i] = first;
            launch_dw_batch(batch, 128, accum, decay, dt, st);
            return s24_launch_status();
        }
        for (int i = 0; i < count; ++i) {
            const s24_dw_problem &pr = problems[i];
            if (pr.q * pr.r == 0) continue;
            const int rc = run_dense_dw(pr.dY, pr.X, pr.dW, pr.p, pr.q, pr.r, beta, dt, pr.W, dt, pr.mask, pr.lambda, st);
            if (rc != S24_OK) return rc;
        }
        return S24_OK;
    }
    // The tiles of all problems make one list.  If its length is not a whole number of rounds over the 256 compute
    // units, look for a problem from which whole tile columns (or rows) amounting to exactly the excess, and to at
    // most half a round, can be cut: that strip runs in small tiles afterwards, the rest in whole rounds.
    int cut = -1, cut_cols = 0, cut_rows = 0;
    const int excess = (int)(total % cus);
    if (excess != 0 && excess <= cus / 2) {
        for (int i = 0; i < count && cut < 0; ++i) {
            const int tm = (int)ceil_div(prs[i].r, 256), tn = (int)ceil_div(prs[i].q, 256);
            if (excess % tm == 0 && excess / tm < tn) { cut = i; cut_cols = excess / tm; }
            else if (excess % tn == 0 && excess / tn < tm) { cut = i; cut_rows = excess / tn; }
        }
    }
    dmatn::DwBatch batch{};
    int first = 0;
    for (int i = 0; i < count; ++i) {
        // the cut removes the LAST tile rows / columns, the ragged edge included: what stays is a multiple of 256
        const int64_t keep_m = i == cut && cut_rows ? 256ll * ((int64_t)ceil_div(prs[i].r, 256) - cut_rows) : prs[i].r;
        const int64_t keep_n = i == cut && cut_cols ? 256ll * ((int64_t)ceil_div(prs[i].q, 256) - cut_cols) : prs[i].q;
        batch.w[i] = dw_window(prs[i], 256, 0, keep_m, 0, keep_n);
        batch.first_slot[i] = first;
        first += (batch.w[i].tiles_m * batch.w[i].tiles_n + 7) / 8;
    }
    for (int i = count; i <= dmatn::kMaxBatch; ++i) batch.first_slot[i] = first;
    launch_dw_batch(batch, 256, accum, decay, dt, st);
    if (cut >= 0) {
        dmatn::DwBatch strip{};
        const int64_t m_off = cut_rows ? batch.w[cut].M : 0, n_off = cut_cols ? batch.w[cut].N : 0;
        strip.w[0] = dw_window(prs[cut], 128, m_off, prs[cut].r - m_off, n_off, prs[cut].q - n_off);
        const int slots = (strip.w[0].tiles_m * strip.w[0].tiles_n + 7) / 8;
        for (int i = 1; i <= dmatn::kMaxBatch; ++i) strip.first_slot[i] = slots;
        launch_dw_batch(strip, 128, accum, decay, dt, st);
    }
    return s24_launch_status();
}

extern "C" int s24_spmm_dw(const void *vals, const uint16_t *meta, const void *X, float *dW, const void *W, s24_dtype wdt,
                           const uint16_t *mask, float lambda, int64_t p, int64_t q, int64_t r, float beta, s24_dtype dt,
                           void *stream)
{
    S24_REQUIRE(p % 64 == 0 && q % 16 == 0 && r % 16 == 0, S24_ERR_SHAPE);
    S24_REQUIRE(beta == 0.0f || beta == 1.0f, S24_ERR_UNSUPPORTED);
    const int rc = check_gemm(vals, X, dW, p, q, r, dt, q * r);
    if (rc != S24_OK || q * r == 0) return rc;
    if (W != nullptr) {
        S24_REQUIRE(s24_valid_dtype(wdt), S24_ERR_DTYPE);
        S24_REQUIRE(mask != nullptr, S24_ERR_NULL);
        S24_REQUIRE(s24_aligned(W, 16) && s24_aligned(mask, 4), S24_ERR_ALIGN);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool accum = beta != 0.0f;
    bool decay_pending = W != nullptr;
    if (p == 0) {
        if (!accum) hipLaunchKernelGGL(fill_zero_kernel, dim3(ceil_div(q * r, kThreads)), dim3(kThreads), 0, st, dW, q * r);
    } else {
        S24_REQUIRE(meta != nullptr, S24_ERR_NULL);
        S24_REQUIRE(s24_aligned(meta, 4), S24_ERR_ALIGN);
        if (dt != S24_F32) {
            const int tiles_m = (int)ceil_div(r, sptn::BM), tiles_n = (int)ceil_div(q, sptn::BN);
            const dim3 grid(((tiles_m * tiles_n + 7) / 8) * 8), block(sptn::THREADS);
            auto *av = static_cast<const uint16_t *>(vals), *x = static_cast<const uint16_t *>(X);
            const bool fuse = decay_pending && wdt == dt;
            auto *w = static_cast<const uint16_t *>(fuse ? W : nullptr);
#define S24_LAUNCH_SPDW(ACC, DEC)                                                                                           \
    hipLaunchKernelGGL((sptn::spmm_tn_big_kernel<T, ACC, DEC>), grid, block, 0, st, av, meta, x, dW, (int)p, (int)r, (int)q, \
                       tiles_m, tiles_n, g_clock_probe, w, mask, lambda)
            S24_WITH_16BIT_TYPE(dt, {
                if (accum && fuse) S24_LAUNCH_SPDW(true, true);
                else if (accum) S24_LAUNCH_SPDW(true, false);
                else if (fuse) S24_LAUNCH_SPDW(false, true);
                else S24_LAUNCH_SPDW(false, false);
            });
#undef S24_LAUNCH_SPDW
            if (fuse) decay_pending = false;
        } else {
            const dim3 grid(ceil_div(r * q, kThreads)), block(kThreads);
            auto *av = static_cast<const float *>(vals), *x = static_cast<const float *>(X);
            if (accum) hipLaunchKernelGGL(spmm_tn_f32_kernel<true>, grid, block, 0, st, av, meta, x, dW, p, r, q);
            else hipLaunchKernelGGL(spmm_tn_f32_kernel<false>, grid, block, 0, st, av, meta, x, dW, p, r, q);
        }
    }
    const int rc2 = s24_launch_status();
    if (rc2 != S24_OK || !decay_pending) return rc2;
    return s24_masked_decay_grad(dW, W, wdt, mask, lambda, r, q, st);
}

extern "C" int s24_set_clock_probe(void *two_counters)
{
    S24_REQUIRE(s24_aligned(two_counters, 8), S24_ERR_ALIGN);
    g_clock_probe = static_cast<unsigned long long *>(two_counters);
    return S24_OK;
}
