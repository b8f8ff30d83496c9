// Transposable 2:4 mask search and prune/compress (Sec. 5.1 and Sec. 5 item 1).
//
// One lane owns one aligned 4x4 block.  A workgroup of 256 lanes walks a tile
// of 32 x 32 blocks (128 x 128 weights), four blocks per lane.  The compressed
// operands are stored chunk-major (64 of the contraction axis per chunk, all
// rows of a chunk together), so a tile covers two chunks of each orientation
// and the column-wise operand, after an LDS transpose, leaves in 8 KB runs.
//
// Scoring.  A legal block is a choice of one of six column pairs per row
// whose columns each get picked twice.  Rows 0-1 and rows 2-3 are scored
// separately ("top" and "bottom" halves) and matched through the column-count
// vector of the top half, which leaves 19 classes:
//   6  where both top rows use the same pair (bottom rows both use its
//      complement): four column sums of the halves;
//   1  where the top rows use complementary pairs (so do the bottom rows):
//      one whole row plus the two largest per-column gains of the other row;
//   12 where the top rows share exactly one column x and miss one column w:
//      column sum x (top) + column sum w (bottom) + the better crossing of the
//      two remaining columns in each half, which only depends on that pair.
// That is about 100 additions and 45 maxima per block instead of 90 x 7
// additions, and yields the same maximum because every legal block falls in
// exactly one class and each class maximum is taken over exactly its blocks.
//
// Exactness and tie-break.  Scores are held in fp64.  Let 2^(E+1) bound the
// largest magnitude of the block and eps = 2^(E-47).  If every nonzero
// magnitude is a multiple of 2048*eps, all partial sums are integers times
// eps below 2^52*eps, hence exact.  Each cell (i,j) is first increased by
// beta_j * 6^(3-i) * eps with beta = (0,2,3,4): the total added to a pattern
// is below 2048*eps, cannot reorder different true scores, and orders equal
// scores exactly like the pattern ids (smaller id = larger bonus).  The bonus
// is read back from the low 11 bits of (best + 2^52*eps) and indexes a table
// that returns the block mask and id.  Blocks whose magnitudes span more
// binades than that window take a slow path that scores all 90 patterns in
// 320-bit fixed point.
#include "s24_common.h"

namespace {

// Column pairs in row-string order ("0011" < "0101" < ... < "1100"): pair k
// keeps columns kC1[k] < kC2[k]; the complementary pair is 5 - k.
__host__ __device__ constexpr int pair_c1(int k) { return k == 0 ? 2 : (k <= 2 ? 1 : 0); }
__host__ __device__ constexpr int pair_c2(int k) { return (k == 0 || k == 1 || k == 3) ? 3 : ((k == 2 || k == 4) ? 2 : 1); }
__host__ __device__ constexpr unsigned pair_bits(int k) { return (1u << pair_c1(k)) | (1u << pair_c2(k)); }
__host__ __device__ constexpr int pair_of(int a, int b)
{
    const int lo = a < b ? a : b, hi = a < b ? b : a;
    for (int k = 0; k < 6; ++k)
        if (pair_c1(k) == lo && pair_c2(k) == hi) return k;
    return -1;
}

constexpr int kRowMult[4] = {216, 36, 6, 1};
constexpr int kColBonus[4] = {0, 2, 3, 4};
constexpr int kBonusBase = 2 * (216 + 36 + 6 + 1);  // every row contributes at least 2

struct MaskLut {
    uint16_t mask[1296];
    uint8_t id[1296];
};

// Index: sum_i 6^(3-i) * (5 - k_i) for row pair indices k_i.  Walking
// (k0,k1,k2,k3) in ascending order visits the legal blocks in id order.
constexpr MaskLut make_lut()
{
    MaskLut t{};
    int n = 0;
    for (int a = 0; a < 6; ++a)
        for (int b = 0; b < 6; ++b)
            for (int c = 0; c < 6; ++c)
                for (int d = 0; d < 6; ++d) {
                    const unsigned rows[4] = {pair_bits(a), pair_bits(b), pair_bits(c), pair_bits(d)};
                    bool ok = true;
                    for (int j = 0; j < 4; ++j) {
                        int s = 0;
                        for (int i = 0; i < 4; ++i) s += (rows[i] >> j) & 1u;
                        if (s != 2) ok = false;
                    }
                    if (!ok) continue;
                    const int x = 216 * (5 - a) + 36 * (5 - b) + 6 * (5 - c) + (5 - d);
                    t.mask[x] = (uint16_t)(rows[0] | rows[1] << 4 | rows[2] << 8 | rows[3] << 12);
                    t.id[x] = (uint8_t)n;
                    ++n;
                }
    return t;
}

__device__ const MaskLut g_lut = make_lut();

struct PatList {
    uint16_t mask[S24_NUM_PATTERNS];
};
constexpr PatList make_patlist()
{
    PatList p{};
    const MaskLut t = make_lut();
    for (int x = 0; x < 1296; ++x)
        if (t.mask[x] != 0) p.mask[t.id[x]] = t.mask[x];
    return p;
}
__device__ const PatList g_patterns = make_patlist();

// What the compressor needs for a bf16 block, precomputed per pattern id (48 bytes each).
// A selector is a v_perm_b32 byte selector that picks two of the four 16-bit values held in a
// register pair {hi : lo} (positions 2,3 : positions 0,1) and packs them into one dword.
struct CompressEntry {
    uint32_t rowsel[4];   // row i: its two kept columns out of {cols 2,3 : cols 0,1}
    uint32_t colsel[4];   // column j: its two kept rows out of {rows 2,3 : rows 0,1}
    uint32_t rowmeta_lo;  // metadata nibbles of rows 0 and 1 at bits 0 and 16
    uint32_t rowmeta_hi;  // rows 2 and 3
    uint32_t colmeta;     // nibbles of columns 0..3 at bits 0, 4, 8, 12
    uint32_t pad;
};
struct CompressLut {
    CompressEntry e[S24_NUM_PATTERNS];
};
constexpr uint32_t perm_selector(int p0, int p1)
{
    return (uint32_t)(2 * p0) | ((uint32_t)(2 * p0 + 1) << 8) | ((uint32_t)(2 * p1) << 16) | ((uint32_t)(2 * p1 + 1) << 24);
}
constexpr CompressLut make_compress_lut()
{
    CompressLut t{};
    const PatList pl = make_patlist();
    for (int id = 0; id < S24_NUM_PATTERNS; ++id) {
        const unsigned m = pl.mask[id];
        uint32_t rowmeta[4] = {0, 0, 0, 0};
        for (int i = 0; i < 4; ++i) {
            int kept[2] = {0, 0}, n = 0;
            for (int j = 0; j < 4; ++j)
                if ((m >> (4 * i + j)) & 1u) kept[n++] = j;
            t.e[id].rowsel[i] = perm_selector(kept[0], kept[1]);
            rowmeta[i] = (uint32_t)(kept[0] | (kept[1] << 2));
        }
        t.e[id].rowmeta_lo = rowmeta[0] | (rowmeta[1] << 16);
        t.e[id].rowmeta_hi = rowmeta[2] | (rowmeta[3] << 16);
        for (int j = 0; j < 4; ++j) {
            int kept[2] = {0, 0}, n = 0;
            for (int i = 0; i < 4; ++i)
                if ((m >> (4 * i + j)) & 1u) kept[n++] = i;
            t.e[id].colsel[j] = perm_selector(kept[0], kept[1]);
            t.e[id].colmeta |= (uint32_t)(kept[0] | (kept[1] << 2)) << (4 * j);
        }
    }
    return t;
}
__device__ const CompressLut g_clut = make_compress_lut();

// Pattern id of a given block mask through the bonus-indexed table: row nibble -> pair index k
// (0 for anything illegal), then the same mixed-radix index the search produces.
__device__ __forceinline__ unsigned lut_index_of_mask(unsigned m)
{
    unsigned x = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned m4 = (m >> (4 * i)) & 0xFu;
        // k for m4 = 3,5,6 in the low word (4 bits each), for m4 = 9,10,12 in the high word
        const unsigned tbl = (m4 & 8u) ? 0x00000130u : 0x02405000u;
        const unsigned k = (tbl >> (4 * (m4 & 7u))) & 7u;
        x = x * 6u + (5u - k);
    }
    return x;
}

// ---------------------------------------------------------------------------
// Slow path: exact scores of all 90 patterns in fixed point.  A magnitude given
// as an fp32 bit pattern is sig * 2^(shift-149) with sig < 2^24; a score is kept
// as ten limbs of 32 payload bits (units of 2^-149), enough for eight fp32
// magnitudes of any exponent.  First maximum in id order wins.
// ---------------------------------------------------------------------------
struct Mag16 { uint32_t v[16]; };

__device__ __noinline__ unsigned slow_best_pattern(Mag16 mag)
{
    // Deliberately loop-based with locally indexed arrays: this path is rare, and
    // keeping it small keeps the register budget of the common path.
    uint32_t sig[16], limb[16], off[16];
#pragma unroll 1
    for (int t = 0; t < 16; ++t) {
        const uint32_t e = mag.v[t] >> 23;
        sig[t] = (mag.v[t] & 0x7FFFFFu) | (e ? 0x800000u : 0u);
        const uint32_t shift = (e ? e : 1u) - 1u;
        limb[t] = shift >> 5;
        off[t] = shift & 31u;
    }
    uint32_t best[10];
#pragma unroll 1
    for (int L = 0; L < 10; ++L) best[L] = 0;
    unsigned best_id = 0;
#pragma unroll 1
    for (unsigned k = 0; k < S24_NUM_PATTERNS; ++k) {
        const unsigned pm = g_patterns.mask[k];
        uint64_t acc[10];
#pragma unroll 1
        for (int L = 0; L < 10; ++L) acc[L] = 0;
#pragma unroll 1
        for (int t = 0; t < 16; ++t) {
            if (!((pm >> t) & 1u)) continue;
            const uint64_t v = (uint64_t)sig[t] << off[t];
            acc[limb[t]] += (uint32_t)v;
            acc[limb[t] + 1] += (uint32_t)(v >> 32);   // limb <= 7, so limb + 1 <= 8
        }
        uint32_t s[10];
        uint64_t carry = 0;
#pragma unroll 1
        for (int L = 0; L < 10; ++L) {
            const uint64_t x = acc[L] + carry;
            s[L] = (uint32_t)x;
            carry = x >> 32;
        }
        // lexicographic compare from the top limb: greater = strictly larger score
        bool greater = false, decided = false;
#pragma unroll 1
        for (int L = 9; L >= 0; --L) {
            if (!decided && s[L] != best[L]) {
                greater = s[L] > best[L];
                decided = true;
            }
        }
        if (greater) {
#pragma unroll 1
            for (int L = 0; L < 10; ++L) best[L] = s[L];
            best_id = k;
        }
    }
    return (unsigned)g_patterns.mask[best_id] | (best_id << 16);
}

// ---------------------------------------------------------------------------
// Middle path: the 90 sums one by one in fp64, first maximum in id order.  Exact as long as every sum of
// eight magnitudes fits fp64's 53 bits, i.e. the block spans at most 26 binades of fp32 data (42 of bf16
// data); used for blocks too wide for the fast path's window, which also has to hold the tie-break bits.
// ---------------------------------------------------------------------------
__device__ __noinline__ unsigned mid_best_pattern(Mag16 mag)
{
    double a[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) a[t] = (double)__uint_as_float(mag.v[t]);
    double best = -1.0;
    unsigned best_id = 0;
#pragma unroll 1
    for (unsigned k = 0; k < S24_NUM_PATTERNS; ++k) {
        const unsigned pm = g_patterns.mask[k];
        double sum = 0.0;
#pragma unroll
        for (int t = 0; t < 16; ++t) sum += ((pm >> t) & 1u) ? a[t] : 0.0;
        if (sum > best) {
            best = sum;
            best_id = k;
        }
    }
    return (unsigned)g_patterns.mask[best_id] | (best_id << 16);
}

// ---------------------------------------------------------------------------
// Fast path.  mag[4*i+j] = |w_ij| as fp32 bit patterns.  Returns mask | id<<16.
// WINDOW = binades below the block maximum within which every element is a
// multiple of 2048*eps (29 for bf16 data, 13 for fp32 data).
// ---------------------------------------------------------------------------
template <int WINDOW, int WIDE>
__device__ __forceinline__ unsigned best_pattern(const uint32_t (&mag)[16], const uint16_t *lut_mask, const uint8_t *lut_id)
{
    uint32_t mx = 0, mn = 0xFFFFFFFFu;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        mx = max(mx, mag[t]);
        mn = min(mn, mag[t] - 1u);  // zero wraps to the top and never wins
    }
    const uint32_t emax = max(mx >> 23, 1u);
    const uint32_t emin = (mn == 0xFFFFFFFFu) ? 255u : max(mn >> 23, 1u);
    if (emin + WINDOW < emax) {
        Mag16 m16;
#pragma unroll
        for (int t = 0; t < 16; ++t) m16.v[t] = mag[t];
        return (emin + WIDE >= emax) ? mid_best_pattern(m16) : slow_best_pattern(m16);
    }

    const double eps = __hiloint2double((int)((emax + 849u) << 20), 0);       // 2^(E-47), E = emax-127
    const double big = __hiloint2double((int)((emax + 849u + 52u) << 20), 0);  // 2^52 * eps
    double a[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const double v = (double)__uint_as_float(mag[4 * i + j]);
            a[i][j] = (j == 0) ? v : __builtin_fma((double)(kColBonus[j] * kRowMult[i]), eps, v);
        }
    // column sums of the top (rows 0,1) and bottom (rows 2,3) halves
    double dt[4], db[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        dt[j] = a[0][j] + a[1][j];
        db[j] = a[2][j] + a[3][j];
    }
    // (i) both top rows keep the pair {c1,c2}, both bottom rows its complement
    double best = 0.0;
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        const double tot = (dt[pair_c1(k)] + dt[pair_c2(k)]) + (db[pair_c1(5 - k)] + db[pair_c2(5 - k)]);
        best = (k == 0) ? tot : __builtin_fmax(best, tot);
    }
    // (ii) complementary pairs in each half: all of row 1 plus the two largest gains of swapping a
    // column to row 0 (and the same for rows 3 and 2)
    {
        auto half = [](const double (&r0)[4], const double (&r1)[4]) {
            const double d0 = r0[0] - r1[0], d1 = r0[1] - r1[1], d2 = r0[2] - r1[2], d3 = r0[3] - r1[3];
            const double m1 = __builtin_fmax(d0, d1), n1 = __builtin_fmin(d0, d1);
            const double m2 = __builtin_fmax(d2, d3), n2 = __builtin_fmin(d2, d3);
            const double hi = __builtin_fmax(m1, m2), lo = __builtin_fmin(m1, m2);
            const double second = __builtin_fmax(lo, __builtin_fmax(n1, n2));
            return ((r1[0] + r1[1]) + (r1[2] + r1[3])) + (hi + second);
        };
        best = __builtin_fmax(best, half(a[0], a[1]) + half(a[2], a[3]));
    }
    // (iii) top rows share column x and keep one each of {y,z}; bottom rows share w and keep the
    // other of {y,z}: dt[x] + db[w] + best crossing of {y,z} in the top + in the bottom
    double cross[6];   // indexed by the pair {y,z}
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        const int y = pair_c1(k), z = pair_c2(k);
        cross[k] = __builtin_fmax(a[0][y] + a[1][z], a[0][z] + a[1][y]) +
                   __builtin_fmax(a[2][y] + a[3][z], a[2][z] + a[3][y]);
    }
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w == x) continue;
            int y = -1, z = -1;
            for (int c = 0; c < 4; ++c)
                if (c != x && c != w) (y < 0 ? y : z) = c;
            best = __builtin_fmax(best, (dt[x] + db[w]) + cross[pair_of(y, z)]);
        }
    const unsigned bonus = (unsigned)__double2loint(best + big) & 0x7FFu;
    const unsigned x = min(bonus - (unsigned)kBonusBase, 1295u);
    return (unsigned)lut_mask[x] | ((unsigned)lut_id[x] << 16);
}

// ---------------------------------------------------------------------------
// Integer fast path (bf16 data).  The same class decomposition and the same tie-break bonus as above, in
// 32-bit integers, which the vector unit adds and compares at twice the rate of fp64: with E the exponent of the
// block's largest magnitude, every magnitude times 2^(155-E) is an integer below 2^29 whose lowest set bit is at
// or above bit 11 as long as it lies within ten binades of the largest (8 significand bits + 10 + 11 = 29), so a
// sum of eight stays below 2^32 and the low 11 bits are free for the bonus.  The product with a power of two and the
// conversion to an integer are exact.  Returns kHardBlock for a block that does not fit (an element more than ten
// binades down, a zero or subnormal element, a block maximum below 2^-99): those take the fp64 path above.
// ---------------------------------------------------------------------------
constexpr unsigned kHardBlock = 0xFFFFFFFFu;

__device__ __forceinline__ unsigned int_best_pattern(const uint32_t (&mag)[16], const uint16_t *lut_mask, const uint8_t *lut_id)
{
    uint32_t mx = mag[0], mn = mag[0];
#pragma unroll
    for (int t = 1; t < 16; ++t) {
        mx = max(mx, mag[t]);
        mn = min(mn, mag[t]);
    }
    const uint32_t E = mx >> 23, emin = mn >> 23;
    if (emin == 0u || emin + 10u < E || E < 28u) return kHardBlock;
    const float scale = __uint_as_float((282u - E) << 23);   // 2^(155-E)
    // r = the scaled magnitudes; the tie-break bonus of a cell, B(i, j), never gets an instruction of its own: every
    // sum below that takes a cell in adds the cell's bonus as part of a compile-time constant (a three-operand add),
    // and every candidate total contains each of its eight cells exactly once.
    uint32_t r[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) r[i][j] = (uint32_t)(__uint_as_float(mag[4 * i + j]) * scale);
    auto B = [](int i, int j) { return (uint32_t)(kColBonus[j] * kRowMult[i]); };
    uint32_t dt[4], db[4];   // both top rows / both bottom rows keep column j
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        dt[j] = r[0][j] + r[1][j] + (B(0, j) + B(1, j));
        db[j] = r[2][j] + r[3][j] + (B(2, j) + B(3, j));
    }
    uint32_t st[4][4], sb[4][4];   // row 0 keeps column p and row 1 column q (p != q); rows 2 and 3 likewise
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (p == q) continue;
            st[p][q] = r[0][p] + r[1][q] + (B(0, p) + B(1, q));
            sb[p][q] = r[2][p] + r[3][q] + (B(2, p) + B(3, q));
        }
    // (i) both top rows keep the pair {c1,c2}, both bottom rows its complement
    uint32_t best = 0;
#pragma unroll
    for (int k = 0; k < 6; ++k)
        best = max(best, (dt[pair_c1(k)] + dt[pair_c2(k)]) + (db[pair_c1(5 - k)] + db[pair_c2(5 - k)]));
    // (ii) complementary pairs in each half: row 0 (row 2) keeps {y,z}, row 1 (row 3) the other two columns {w,x}
    {
        uint32_t top = 0, bot = 0;
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const int y = pair_c1(k), z = pair_c2(k), w = pair_c1(5 - k), x = pair_c2(5 - k);
            top = max(top, st[y][w] + st[z][x]);
            bot = max(bot, sb[y][w] + sb[z][x]);
        }
        best = max(best, top + bot);
    }
    // (iii) top rows share column x, bottom rows share column w, the two remaining columns cross in each half
    uint32_t cross[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        const int y = pair_c1(k), z = pair_c2(k);
        cross[k] = max(st[y][z], st[z][y]) + max(sb[y][z], sb[z][y]);
    }
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w == x) continue;
            int y = -1, z = -1;
            for (int c = 0; c < 4; ++c)
                if (c != x && c != w) (y < 0 ? y : z) = c;
            best = max(best, dt[x] + db[w] + cross[pair_of(y, z)]);
        }
    const unsigned xi = min((best & 0x7FFu) - (unsigned)kBonusBase, 1295u);
    return (unsigned)lut_mask[xi] | ((unsigned)lut_id[xi] << 16);
}

// ---------------------------------------------------------------------------
// Per-dtype access to one block row (four consecutive weights).
// ---------------------------------------------------------------------------
template <typename T> struct RowOps;

template <> struct RowOps<uint16_t> {  // bf16
    using Row = uint2;     // four bf16
    using Pair = uint32_t; // two bf16
    static constexpr int kWindow = 29, kWide = 42;
    static __device__ __forceinline__ Row load(const uint16_t *p) { return *reinterpret_cast<const uint2 *>(p); }
    static __device__ __forceinline__ uint32_t bits(const Row &r, int j)
    {
        const uint64_t v = ((uint64_t)r.y << 32) | r.x;
        return (uint32_t)(v >> (16 * j)) & 0xFFFFu;
    }
    static __device__ __forceinline__ uint32_t mag(const Row &r, int j)  // compile-time j
    {
        const uint32_t d = (j < 2) ? r.x : r.y;
        return (j & 1) ? (d & 0x7FFF0000u) : ((d << 16) & 0x7FFF0000u);
    }
    static __device__ __forceinline__ Pair pair(uint32_t lo, uint32_t hi) { return lo | (hi << 16); }
};

// IEEE binary16: the same 16-bit moves as bf16; a magnitude widens to fp32 exactly (binary16 subnormals are fp32
// normals).  An element with fp32 exponent e is a multiple of 2^(e-10), so the fast path's window is 26 binades,
// and eight of them sum exactly in fp64 over 39 binades, which is all binary16 has: no block needs the slow path.
template <> struct RowOps<s24_half> {
    using Row = uint2;
    using Pair = uint32_t;
    static constexpr int kWindow = 26, kWide = 39;
    static __device__ __forceinline__ Row load(const s24_half *p) { return *reinterpret_cast<const uint2 *>(p); }
    static __device__ __forceinline__ uint32_t bits(const Row &r, int j) { return RowOps<uint16_t>::bits(r, j); }
    static __device__ __forceinline__ uint32_t mag(const Row &r, int j)  // compile-time j
    {
        const uint32_t d = (j < 2) ? r.x : r.y;
        return __float_as_uint(s24_num<s24_half>::widen(((j & 1) ? (d >> 16) : d) & 0x7FFFu));
    }
    static __device__ __forceinline__ Pair pair(uint32_t lo, uint32_t hi) { return lo | (hi << 16); }
};

template <> struct RowOps<float> {
    using Row = uint4;
    using Pair = uint2;
    static constexpr int kWindow = 13, kWide = 26;
    static __device__ __forceinline__ Row load(const float *p) { return *reinterpret_cast<const uint4 *>(p); }
    static __device__ __forceinline__ uint32_t bits(const Row &r, int j)
    {
        return j == 0 ? r.x : (j == 1 ? r.y : (j == 2 ? r.z : r.w));
    }
    static __device__ __forceinline__ uint32_t mag(const Row &r, int j) { return bits(r, j) & 0x7FFFFFFFu; }
    static __device__ __forceinline__ Pair pair(uint32_t lo, uint32_t hi) { return make_uint2(lo, hi); }
};

constexpr int kTile = 32;        // blocks per tile edge
constexpr int kPitch = kTile + 1;

template <typename T, bool SEARCH, bool COMPRESS>
__global__ __launch_bounds__(256) void mask_compress_kernel(const T *__restrict__ W, int64_t ldw, int br, int bq,
                                                            const uint16_t *__restrict__ mask_in,
                                                            uint16_t *__restrict__ mask_out, uint8_t *__restrict__ index_out,
                                                            T *__restrict__ vals, uint16_t *__restrict__ meta,
                                                            T *__restrict__ valsT, uint16_t *__restrict__ metaT)
{
    using Ops = RowOps<T>;
    using Row = typename Ops::Row;
    using Pair = typename Ops::Pair;
    constexpr bool FAST = COMPRESS && sizeof(T) == 2;   // bf16: table-driven compressor
    // bf16 search on its own: integer scoring with the blocks it cannot take queued for the fp64 path.  (In the fused
    // search + compress kernel the four blocks' rows held in registers across the queue cost more than the cheaper
    // scoring saves: measured 4-8 % slower, so it keeps the fp64 scoring inside its loop.)
    constexpr bool DEFER = SEARCH && !COMPRESS && sizeof(T) == 2 && RowOps<T>::kWindow == 29;
    __shared__ int s_nhard;
    __shared__ uint16_t s_hard[DEFER ? 1024 : 1];
    __shared__ uint32_t s_fix[DEFER ? 1024 : 1];
    __shared__ uint16_t s_lut_mask[SEARCH ? 1296 : 1];
    __shared__ uint8_t s_lut_id[(SEARCH || FAST) ? 1296 : 1];
    __shared__ uint4 s_clut[FAST ? 3 * S24_NUM_PATTERNS : 1];
    __shared__ Pair s_valsT[COMPRESS ? 4 * kTile * kPitch : 1];
    __shared__ uint8_t s_nibT[COMPRESS ? 4 * kTile * kPitch : 1];

    const int tid = threadIdx.x;
    if (DEFER && tid == 0) s_nhard = 0;
    if constexpr (SEARCH || FAST) {
        for (int x = tid; x < 1296; x += 256) {
            if constexpr (SEARCH) s_lut_mask[x] = g_lut.mask[x];
            s_lut_id[x] = g_lut.id[x];
        }
        if constexpr (FAST) {
            const uint4 *src = reinterpret_cast<const uint4 *>(&g_clut);
            for (int x = tid; x < 3 * S24_NUM_PATTERNS; x += 256) s_clut[x] = src[x];
        }
        __syncthreads();
    }
    const int bj0 = blockIdx.x * kTile, bi0 = blockIdx.y * kTile;
    const int lbj = tid & 31;
    const int bj = bj0 + lbj;
    const int64_t R = 4 * (int64_t)br, Q = 4 * (int64_t)bq;  // rows of vals / of valsT

    // first weight row of this lane's first block; block s of the lane lies 8 s block rows further down
    const T *wrow = W + (int64_t)(4 * (bi0 + (tid >> 5))) * ldw + 4 * bj;
    auto fetch = [&](Row (&dst)[4], const T *p, bool ok) {
        if (ok) {
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[i] = Ops::load(p + i * ldw);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[i] = Row{};
        }
    };
    auto magnitudes = [&](const Row (&rows)[4], uint32_t (&mag)[16]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) mag[4 * i + j] = Ops::mag(rows[i], j);
    };
    // What follows the search for block s of this lane (rows in registers, mask m and pattern id known):
    // the mask and id stores and, when compressing, both compressed orientations.
    auto emit = [&](const Row (&rows)[4], unsigned m, unsigned id, int s) {
        const int lbi = (tid >> 5) + 8 * s;
        const int bi = bi0 + lbi;
        const bool valid = (bi < br) && (bj < bq);
        if constexpr (SEARCH) {
            if (valid) {
                if (mask_out) mask_out[(int64_t)bi * bq + bj] = (uint16_t)m;
                if (index_out) index_out[(int64_t)bi * bq + bj] = (uint8_t)id;
            }
        }
        if constexpr (FAST) {
            if constexpr (!SEARCH) id = s_lut_id[min(lut_index_of_mask(m), 1295u)];
            const uint4 rsel = s_clut[3 * id], csel = s_clut[3 * id + 1], mt = s_clut[3 * id + 2];
            const uint32_t rs[4] = {rsel.x, rsel.y, rsel.z, rsel.w}, cs[4] = {csel.x, csel.y, csel.z, csel.w};
            // along q: one dword (two kept bf16) per block row.  The four lanes of a quad (four neighbouring blocks
            // of one block row) transpose their 4 x 4 dwords among themselves, two exchanges with the lane one away and
            // two with the lane two away, so that lane k of the quad ends up with row k of all four blocks: 16
            // contiguous bytes of that row's run, one store instead of four 4-byte ones.  (br and bq are multiples
            // of 16: a quad is all inside the matrix or all outside.)
            uint32_t pr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[i] = __builtin_amdgcn_perm(rows[i].y, rows[i].x, rs[i]);
            {
                const bool odd = lbj & 1, upper = lbj & 2;
#pragma unroll
                for (int i = 0; i < 4; i += 2) {   // with lane ^ 1: an even lane hands over row i+1, an odd one row i
                    const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(odd ? pr[i] : pr[i + 1]), 0xB1, 0xF, 0xF, false);
                    if (odd) pr[i] = got;
                    else pr[i + 1] = got;
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {      // with lane ^ 2: a lower lane hands over entry j+2, an upper one entry j
                    const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(upper ? pr[j] : pr[j + 2]), 0x4E, 0xF, 0xF, false);
                    if (upper) pr[j] = got;
                    else pr[j + 2] = got;
                }
            }
            if (valid)
                *reinterpret_cast<uint4 *>(reinterpret_cast<uint32_t *>(vals) + ((int64_t)(bj >> 4) * R + 4 * bi + (lbj & 3)) * 16 + (bj & 12)) =
                    make_uint4(pr[0], pr[1], pr[2], pr[3]);
            uint32_t nib_lo = mt.x, nib_hi = mt.y;
            nib_lo |= (uint32_t)__shfl_down((int)nib_lo, 1) << 4;
            nib_hi |= (uint32_t)__shfl_down((int)nib_hi, 1) << 4;
            nib_lo |= (uint32_t)__shfl_down((int)nib_lo, 2) << 8;
            nib_hi |= (uint32_t)__shfl_down((int)nib_hi, 2) << 8;
            if (valid && (lbj & 3) == 0) {
                const int w = bj >> 2;  // metadata word of the row: chunk w/4, word w%4
                uint16_t *mrow = meta + ((int64_t)(w >> 2) * R + 4 * bi) * 4 + (w & 3);
                mrow[0] = (uint16_t)(nib_lo & 0xFFFFu);
                mrow[4] = (uint16_t)(nib_lo >> 16);
                mrow[8] = (uint16_t)(nib_hi & 0xFFFFu);
                mrow[12] = (uint16_t)(nib_hi >> 16);
            }
            // along r: gather each column from the four rows, pick its two kept rows, park in LDS
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t half = (j & 1) ? 0x07060302u : 0x05040100u;
                const uint32_t r0 = (j < 2) ? rows[0].x : rows[0].y, r1 = (j < 2) ? rows[1].x : rows[1].y;
                const uint32_t r2 = (j < 2) ? rows[2].x : rows[2].y, r3 = (j < 2) ? rows[3].x : rows[3].y;
                const uint32_t col_lo = __builtin_amdgcn_perm(r1, r0, half);  // rows 0,1 of column j
                const uint32_t col_hi = __builtin_amdgcn_perm(r3, r2, half);  // rows 2,3
                const int a = (j * kTile + lbj) * kPitch + lbi;
                s_valsT[a] = __builtin_amdgcn_perm(col_hi, col_lo, cs[j]);
                s_nibT[a] = (uint8_t)((mt.z >> (4 * j)) & 0xFu);
            }
        } else if constexpr (COMPRESS) {
            // along q: two kept weights and one nibble per block row
            uint32_t nib_lo = 0, nib_hi = 0;  // nibbles of rows (0,1) and (2,3), 16 bits apart
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned m4 = (m >> (4 * i)) & 0xFu;
                const int i0 = (__ffs((int)m4) - 1) & 3;
                const int i1 = (31 - __clz((int)(m4 | 1u))) & 3;
                const Pair pr = Ops::pair(Ops::bits(rows[i], i0), Ops::bits(rows[i], i1));
                // chunk bj/16 of row 4bi+i, pair bj%16 of its 16 pairs
                if (valid) reinterpret_cast<Pair *>(vals)[((int64_t)(bj >> 4) * R + 4 * bi + i) * 16 + (bj & 15)] = pr;
                const uint32_t nib = (uint32_t)(i0 | (i1 << 2));
                if (i < 2) nib_lo |= nib << (16 * i);
                else nib_hi |= nib << (16 * (i - 2));
            }
            // four neighbouring lanes (same block row) form one metadata word per row
            nib_lo |= (uint32_t)__shfl_down((int)nib_lo, 1) << 4;
            nib_hi |= (uint32_t)__shfl_down((int)nib_hi, 1) << 4;
            nib_lo |= (uint32_t)__shfl_down((int)nib_lo, 2) << 8;
            nib_hi |= (uint32_t)__shfl_down((int)nib_hi, 2) << 8;
            if (valid && (lbj & 3) == 0) {
                const int w = bj >> 2;  // metadata word of the row: chunk w/4, word w%4
                uint16_t *mrow = meta + ((int64_t)(w >> 2) * R + 4 * bi) * 4 + (w & 3);
                mrow[0] = (uint16_t)(nib_lo & 0xFFFFu);
                mrow[4] = (uint16_t)(nib_lo >> 16);
                mrow[8] = (uint16_t)(nib_hi & 0xFFFFu);
                mrow[12] = (uint16_t)(nib_hi >> 16);
            }
            // along r: kept rows of each column go through LDS to be written transposed
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned c = m >> j;
                const unsigned cm = (c & 1u) | ((c >> 3) & 2u) | ((c >> 6) & 4u) | ((c >> 9) & 8u);
                const int i0 = (__ffs((int)cm) - 1) & 3;
                const int i1 = (31 - __clz((int)(cm | 1u))) & 3;
                uint32_t e[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) e[i] = Ops::bits(rows[i], j);
                const uint32_t v0 = i0 == 0 ? e[0] : (i0 == 1 ? e[1] : (i0 == 2 ? e[2] : e[3]));
                const uint32_t v1 = i1 == 0 ? e[0] : (i1 == 1 ? e[1] : (i1 == 2 ? e[2] : e[3]));
                const int a = (j * kTile + lbj) * kPitch + lbi;
                s_valsT[a] = Ops::pair(v0, v1);
                s_nibT[a] = (uint8_t)(i0 | (i1 << 2));
            }
        }
    };

    if constexpr (DEFER) {
        // bf16 search: all four blocks of the lane are scored by the integer fast path first; the few blocks it
        // cannot take (about one in forty for normally distributed weights) are queued in LDS and scored afterwards
        // by the fp64 path, one per lane, so that a rare block costs one lane's time instead of stalling its whole
        // wave in a divergent branch.
        Row blk[4][4];
        unsigned res[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) fetch(blk[s], wrow + (int64_t)(32 * s) * ldw, (bi0 + (tid >> 5) + 8 * s < br) && (bj < bq));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bool valid = (bi0 + (tid >> 5) + 8 * s < br) && (bj < bq);
            uint32_t mag[16];
            magnitudes(blk[s], mag);
            res[s] = valid ? int_best_pattern(mag, s_lut_mask, s_lut_id) : 0x33CCu;   // off the edge: pattern 0, never stored
            if (res[s] == kHardBlock) s_hard[atomicAdd(&s_nhard, 1)] = (uint16_t)(256 * s + tid);
        }
        __syncthreads();
        const int nhard = s_nhard;
        for (int e = tid; e < nhard; e += 256) {
            const int code = s_hard[e], hs = code >> 8, owner = code & 255;
            const T *p = W + (int64_t)(4 * (bi0 + (owner >> 5) + 8 * hs)) * ldw + 4 * (bj0 + (owner & 31));
            Row rows[4];
            fetch(rows, p, true);
            uint32_t mag[16];
            magnitudes(rows, mag);
            s_fix[code] = best_pattern<Ops::kWindow, Ops::kWide>(mag, s_lut_mask, s_lut_id);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const unsigned r = res[s] == kHardBlock ? s_fix[256 * s + tid] : res[s];
            emit(blk[s], r & 0xFFFFu, r >> 16, s);
        }
    } else {
        // The rows of the next block are requested before the current one is scored.
        Row nxt[4];
        fetch(nxt, wrow, (bi0 + (tid >> 5) < br) && (bj < bq));
#pragma unroll 1
        for (int s = 0; s < 4; ++s) {
            const int bi = bi0 + (tid >> 5) + 8 * s;
            const bool valid = (bi < br) && (bj < bq);
            Row rows[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) rows[i] = nxt[i];
            wrow += 32 * ldw;
            if (s < 3) fetch(nxt, wrow, (bi + 8 < br) && (bj < bq));
            unsigned m = 0, id = 0;
            if constexpr (SEARCH) {
                uint32_t mag[16];
                magnitudes(rows, mag);
                const unsigned res = best_pattern<Ops::kWindow, Ops::kWide>(mag, s_lut_mask, s_lut_id);
                m = res & 0xFFFFu;
                id = res >> 16;
            } else {
                m = valid ? mask_in[(int64_t)bi * bq + bj] : 0x33CCu;
            }
            emit(rows, m, id, s);
        }
    }
    if constexpr (COMPRESS) {
        __syncthreads();
        // valsT: two chunks (16 pairs each) of 128 columns of W.  One item = four consecutive pairs of
        // one column; consecutive lanes take consecutive items of a column, then the next column, so a
        // chunk of the tile leaves as one contiguous run.
        Pair *outT = reinterpret_cast<Pair *>(valsT);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = tid + 256 * it;                    // 1024 items
            const int quad = idx & 3, col = (idx >> 2) & 127, half = idx >> 9;   // col = 4*lbj + j
            const int j = col & 3, lb = col >> 2;
            const int lbi = 16 * half + 4 * quad, bi = bi0 + lbi;
            if (bj0 + lb < bq && bi < br) {   // br is a multiple of 16: a quad is all in or all out
                const Pair *src = &s_valsT[(j * kTile + lb) * kPitch + lbi];
                Pair *dst = outT + ((int64_t)(bi >> 4) * Q + 4 * (bj0 + lb) + j) * 16 + (bi & 15);
                if constexpr (sizeof(Pair) == 4) {
                    *reinterpret_cast<uint4 *>(dst) = make_uint4(src[0], src[1], src[2], src[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) dst[e] = src[e];
                }
            }
        }
        // metaT: per column two chunks of four words; one thread packs the 16 nibbles of one (column, chunk)
        {
            const int col = tid & 127, half = tid >> 7;
            const int j = col & 3, lb = col >> 2;
            if (bj0 + lb < bq && bi0 + 16 * half < br) {
                const uint8_t *n = &s_nibT[(j * kTile + lb) * kPitch + 16 * half];
                uint32_t w01 = 0, w23 = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    w01 |= (uint32_t)n[e] << (4 * e);
                    w23 |= (uint32_t)n[8 + e] << (4 * e);
                }
                const int kc = (bi0 >> 4) + half;   // chunk index along r
                *reinterpret_cast<uint2 *>(metaT + ((int64_t)kc * Q + 4 * (bj0 + lb) + j) * 4) = make_uint2(w01, w23);
            }
        }
    }
}

template <typename T>
int launch(const void *W, int64_t r, int64_t q, int64_t ldw, const uint16_t *mask_in, uint16_t *mask_out,
           uint8_t *index_out, void *vals, uint16_t *meta, void *valsT, uint16_t *metaT, bool compress, hipStream_t st)
{
    const int br = (int)(r / 4), bq = (int)(q / 4);
    if (br == 0 || bq == 0) return S24_OK;
    const dim3 grid((bq + kTile - 1) / kTile, (br + kTile - 1) / kTile), block(256);
    const T *w = static_cast<const T *>(W);
    if (!compress)
        hipLaunchKernelGGL((mask_compress_kernel<T, true, false>), grid, block, 0, st, w, ldw, br, bq, nullptr, mask_out,
                           index_out, nullptr, nullptr, nullptr, nullptr);
    else if (mask_in)
        hipLaunchKernelGGL((mask_compress_kernel<T, false, true>), grid, block, 0, st, w, ldw, br, bq, mask_in, nullptr,
                           nullptr, static_cast<T *>(vals), meta, static_cast<T *>(valsT), metaT);
    else
        hipLaunchKernelGGL((mask_compress_kernel<T, true, true>), grid, block, 0, st, w, ldw, br, bq, nullptr, mask_out,
                           nullptr, static_cast<T *>(vals), meta, static_cast<T *>(valsT), metaT);
    return s24_launch_status();
}

// ------------------------------------------------------------------ monitors
// Flip count: || m_new - m_old ||_1 over all mask cells.  Eight blocks (one 16-byte load of each mask) per
// thread and pass; wave sums by cross-lane adds, one 64-bit atomic per wave.
__global__ __launch_bounds__(256) void clear_counter_kernel(unsigned long long *counter) { *counter = 0ull; }

__global__ __launch_bounds__(256) void mask_flips_kernel(const uint16_t *__restrict__ mask_new,
                                                         const uint16_t *__restrict__ mask_old, int64_t nblocks,
                                                         uint32_t *__restrict__ block_flips,
                                                         unsigned long long *__restrict__ total)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    unsigned count = 0;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v * 8 < nblocks; v += stride) {
        const int64_t b0 = v * 8;
        if (b0 + 8 <= nblocks) {
            const uint4 a = *reinterpret_cast<const uint4 *>(mask_new + b0), b = *reinterpret_cast<const uint4 *>(mask_old + b0);
            const uint32_t x[4] = {a.x ^ b.x, a.y ^ b.y, a.z ^ b.z, a.w ^ b.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                count += __builtin_popcount(x[k]);
                if (block_flips) {
                    block_flips[b0 + 2 * k] += __builtin_popcount(x[k] & 0xFFFFu);
                    block_flips[b0 + 2 * k + 1] += __builtin_popcount(x[k] >> 16);
                }
            }
        } else {
            for (int64_t b = b0; b < nblocks; ++b) {
                const unsigned c = __builtin_popcount((unsigned)(mask_new[b] ^ mask_old[b]));
                count += c;
                if (block_flips) block_flips[b] += c;
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) count += __shfl_down(count, off, 64);
    // one atomic per workgroup: thousands of them on one address would cost more than the scan itself
    __shared__ unsigned s_part[4];
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = count;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long sum = (unsigned long long)s_part[0] + s_part[1] + s_part[2] + s_part[3];
        if (sum != 0) atomicAdd(total, sum);
    }
}

// L1-norm gap: one block per thread, all 90 kept norms in fp64 (exact while the block's exponent spread
// stays inside fp64's 53 bits, which it does for any bf16 block spanning up to 29 binades), best and
// second best tracked on the way.
template <typename T>
__global__ __launch_bounds__(256) void l1_gap_kernel(const T *__restrict__ W, int64_t ldw, int br, int bq,
                                                     double *__restrict__ gap)
{
    __shared__ uint16_t s_pat[S24_NUM_PATTERNS];
    if (threadIdx.x < S24_NUM_PATTERNS) s_pat[threadIdx.x] = g_patterns.mask[threadIdx.x];
    __syncthreads();
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)br * bq) return;
    const int bi = (int)(idx / bq), bj = (int)(idx - (int64_t)bi * bq);
    double a[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const T *row = W + (int64_t)(4 * bi + i) * ldw + 4 * bj;
        if constexpr (sizeof(T) == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(row);
            a[4 * i] = fabs((double)s24_num<T>::lo(v.x));
            a[4 * i + 1] = fabs((double)s24_num<T>::hi(v.x));
            a[4 * i + 2] = fabs((double)s24_num<T>::lo(v.y));
            a[4 * i + 3] = fabs((double)s24_num<T>::hi(v.y));
        } else {
            const float4 v = *reinterpret_cast<const float4 *>(row);
            a[4 * i] = fabs((double)v.x);
            a[4 * i + 1] = fabs((double)v.y);
            a[4 * i + 2] = fabs((double)v.z);
            a[4 * i + 3] = fabs((double)v.w);
        }
    }
    double first = 0.0, second = 0.0;
#pragma unroll 1
    for (int k = 0; k < S24_NUM_PATTERNS; ++k) {
        const unsigned m = s_pat[k];
        double sum = 0.0;
#pragma unroll
        for (int t = 0; t < 16; ++t) sum += ((m >> t) & 1u) ? a[t] : 0.0;
        if (k == 0) {
            first = sum;
        } else if (sum > first) {
            second = first;
            first = sum;
        } else if (k == 1 || sum > second) {
            second = sum;
        }
    }
    gap[idx] = first - second;
}

// Shape and dtype are checked first; an empty matrix (r or q zero) is accepted
// whatever the pointers are, since nothing will be read or written.
int check_weight(const void *W, int dt, int64_t r, int64_t q, int64_t ldw, int64_t gran)
{
    S24_REQUIRE(s24_valid_dtype(dt), S24_ERR_DTYPE);
    S24_REQUIRE(r >= 0 && q >= 0 && r % gran == 0 && q % gran == 0 && ldw >= q, S24_ERR_SHAPE);
    S24_REQUIRE(r / 4 < (1ll << 30) && q / 4 < (1ll << 30), S24_ERR_SHAPE);
    if (r == 0 || q == 0) return S24_OK;
    S24_REQUIRE(W != nullptr, S24_ERR_NULL);
    const size_t row_bytes = dt == S24_F32 ? 16 : 8;  // one block row is loaded as a single vector
    S24_REQUIRE(s24_aligned(W, row_bytes) && (ldw * s24_elem_size(dt)) % row_bytes == 0, S24_ERR_ALIGN);
    return S24_OK;
}

}  // namespace

extern "C" int s24_transposable_mask(const void *W, s24_dtype dt, int64_t r, int64_t q, int64_t ldw, uint16_t *mask,
                                     uint8_t *index, void *stream)
{
    const int rc = check_weight(W, dt, r, q, ldw, 4);
    if (rc != S24_OK || r == 0 || q == 0) return rc;
    S24_REQUIRE(mask != nullptr, S24_ERR_NULL);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == S24_BF16)
        return launch<uint16_t>(W, r, q, ldw, nullptr, mask, index, nullptr, nullptr, nullptr, nullptr, false, st);
    if (dt == S24_F16)
        return launch<s24_half>(W, r, q, ldw, nullptr, mask, index, nullptr, nullptr, nullptr, nullptr, false, st);
    return launch<float>(W, r, q, ldw, nullptr, mask, index, nullptr, nullptr, nullptr, nullptr, false, st);
}

extern "C" int s24_compress(const void *W, s24_dtype dt, int64_t r, int64_t q, int64_t ldw, const uint16_t *mask,
                            void *vals, uint16_t *meta, void *valsT, uint16_t *metaT, uint16_t *mask_out, void *stream)
{
    const int rc = check_weight(W, dt, r, q, ldw, 64);
    if (rc != S24_OK || r == 0 || q == 0) return rc;
    S24_REQUIRE(vals && meta && valsT && metaT, S24_ERR_NULL);
    // the kernel stores 16 bytes of values and 8 bytes of index words at a time (and the GEMMs that consume the
    // operands copy them in 16-byte pieces)
    S24_REQUIRE(s24_aligned(vals, 16) && s24_aligned(valsT, 16) && s24_aligned(meta, 8) && s24_aligned(metaT, 8) &&
                    s24_aligned(mask, 2) && s24_aligned(mask_out, 2),
                S24_ERR_ALIGN);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == S24_BF16)
        return launch<uint16_t>(W, r, q, ldw, mask, mask_out, nullptr, vals, meta, valsT, metaT, true, st);
    if (dt == S24_F16)
        return launch<s24_half>(W, r, q, ldw, mask, mask_out, nullptr, vals, meta, valsT, metaT, true, st);
    return launch<float>(W, r, q, ldw, mask, mask_out, nullptr, vals, meta, valsT, metaT, true, st);
}

extern "C" int s24_mask_flips(const uint16_t *mask_new, const uint16_t *mask_old, int64_t nblocks, uint32_t *block_flips,
                              uint64_t *flips, void *stream)
{
    S24_REQUIRE(nblocks >= 0, S24_ERR_SHAPE);
    S24_REQUIRE(flips != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(flips, 8), S24_ERR_ALIGN);
    if (nblocks > 0) {
        S24_REQUIRE(mask_new && mask_old, S24_ERR_NULL);
        S24_REQUIRE(s24_aligned(mask_new, 16) && s24_aligned(mask_old, 16) && s24_aligned(block_flips, 4), S24_ERR_ALIGN);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto *total = reinterpret_cast<unsigned long long *>(flips);
    hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, st, total);
    if (nblocks > 0) {
        const int64_t vecs = (nblocks + 7) / 8;
        const unsigned grid = (unsigned)((vecs + 255) / 256 < 1024 ? (vecs + 255) / 256 : 1024);
        hipLaunchKernelGGL(mask_flips_kernel, dim3(grid), dim3(256), 0, st, mask_new, mask_old, nblocks, block_flips, total);
    }
    return s24_launch_status();
}

extern "C" int s24_l1_norm_gap(const void *W, s24_dtype dt, int64_t r, int64_t q, int64_t ldw, double *gap, void *stream)
{
    const int rc = check_weight(W, dt, r, q, ldw, 4);
    if (rc != S24_OK || r == 0 || q == 0) return rc;
    S24_REQUIRE(gap != nullptr, S24_ERR_NULL);
    S24_REQUIRE(s24_aligned(gap, 8), S24_ERR_ALIGN);
    const int br = (int)(r / 4), bq = (int)(q / 4);
    const int64_t n = (int64_t)br * bq;
    S24_REQUIRE((n + 255) / 256 < (1ll << 31), S24_ERR_SHAPE);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (dt == S24_BF16)
        hipLaunchKernelGGL(l1_gap_kernel<uint16_t>, grid, block, 0, st, static_cast<const uint16_t *>(W), ldw, br, bq, gap);
    else if (dt == S24_F16)
        hipLaunchKernelGGL(l1_gap_kernel<s24_half>, grid, block, 0, st, static_cast<const s24_half *>(W), ldw, br, bq, gap);
    else
        hipLaunchKernelGGL(l1_gap_kernel<float>, grid, block, 0, st, static_cast<const float *>(W), ldw, br, bq, gap);
    return s24_launch_status();
}
