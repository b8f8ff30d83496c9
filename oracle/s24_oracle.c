/*
 * s24 oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what the 2:4-sparse FFN
 * training step computes (arXiv 2404.01847).  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code, table,
 * header or helper with the HIP library; nothing here was derived from the GPU
 * kernels and no expected value stored anywhere comes from them.
 *
 * Conventions (paper Sec. 3.1): X is p x q (tokens x in-features), W is r x q
 * (out-features x in-features), Z/Y is p x r; all row-major.  dtype 0 = fp32,
 * 1 = bf16 (raw uint16 bit patterns), 2 = IEEE binary16 (raw uint16 bit
 * patterns; the paper's own precision is fp16 mixed precision, Sec. 6).
 * Floating-point results are returned in fp64; every input is widened exactly
 * before any arithmetic.
 *
 * Readings taken where the paper is silent:
 *   - order of the 90 block patterns: lexicographic on the 16-character
 *     row-major string m00 m01 ... m33 with '0' < '1';
 *   - argmax tie-break: first (smallest id) maximal pattern;
 *   - pattern scores are compared as exact real numbers;
 *   - a block mask is stored as uint16 with bit (4i+j) = m_ij;
 *   - compressed format: kept values in column order, one 4-bit metadata
 *     nibble i0 | i1<<2 per group of four, nibbles packed little-endian;
 *     orc_pack_chunk_major() permutes it into the chunk-major storage order
 *     the GPU library exchanges (64 of the contraction axis per chunk).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * facts that do not come from this file (exhaustive enumeration in Python,
 * exact rational arithmetic, numpy/torch library routines, closed forms,
 * finite differences).  No function is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
enum { ORC_ACT_RELU = 0, ORC_ACT_GELU_ERF = 1 };
enum { ORC_GATE_SILU = 0, ORC_GATE_GELU_ERF = 1 };
enum { ORC_ROW_MAJOR = 0, ORC_COL_MAJOR = 1 };

/* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.
 * e = 0: +-f * 2^-24;  e = 31: infinity (f = 0) or NaN;  else +-(1024 + f) * 2^(e-25). */
static double half_bits_to_double(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)f, -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

static double widen(const void *base, int dt, size_t idx)
{
    if (dt == ORC_F32)
        return (double)((const float *)base)[idx];
    if (dt == ORC_F16)
        return half_bits_to_double(((const uint16_t *)base)[idx]);
    uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------ */
/* Pattern table (Sec. 5.1 step 1: all legal 4x4 blocks, found by      */
/* exhaustive inspection; the paper's count is n_t = 90).              */
/* ------------------------------------------------------------------ */

/* Walk every 16-character binary string in lexicographic order ('0'<'1');
 * character t (t = 4i+j) is m_ij.  Keep those with two ones in each row and
 * each column.  Returns the number found; out[] receives the uint16 encodings
 * (bit t = character t) in that order. */
int orc_pattern_table(uint16_t *out, int cap)
{
    int n = 0;
    for (uint32_t s = 0; s < 65536u; ++s) {
        int m[4][4];
        for (int t = 0; t < 16; ++t)
            m[t / 4][t % 4] = (int)((s >> (15 - t)) & 1u); /* char t, MSB first */
        int ok = 1;
        for (int i = 0; i < 4 && ok; ++i)
            if (m[i][0] + m[i][1] + m[i][2] + m[i][3] != 2) ok = 0;
        for (int j = 0; j < 4 && ok; ++j)
            if (m[0][j] + m[1][j] + m[2][j] + m[3][j] != 2) ok = 0;
        if (!ok) continue;
        uint16_t enc = 0;
        for (int t = 0; t < 16; ++t)
            if (m[t / 4][t % 4]) enc |= (uint16_t)(1u << t);
        if (n < cap) out[n] = enc;
        ++n;
    }
    return n;
}

/* ------------------------------------------------------------------ */
/* Mask search (Sec. 5.1 problem formulation; Alg. 1 = argmax over all */
/* patterns of the retained L1 norm of the block).                     */
/* ------------------------------------------------------------------ */

/* Exact wide accumulator: a non-negative fixed-point number in units of
 * 2^-149 (the smallest fp32 subnormal), ten limbs of 32 payload bits each
 * kept in 64-bit words so that eight additions cannot overflow a limb. */
#define WIDE_LIMBS 10
typedef struct { uint64_t limb[WIDE_LIMBS]; } wide_t;

static void wide_add(wide_t *acc, double a)
{
    if (a == 0.0) return;
    int e;
    double m = frexp(a, &e);               /* a = m * 2^e, 0.5 <= m < 1 */
    uint64_t mi = (uint64_t)ldexp(m, 53);  /* exact: a has <= 53 bits    */
    int low = e - 53;
    while ((mi & 1u) == 0) { mi >>= 1; ++low; }
    /* a = mi * 2^low with mi odd; inputs come from fp32/bf16, so mi < 2^24
     * and low >= -149. */
    int shift = low + 149;
    int li = shift / 32, off = shift % 32;
    uint64_t v = mi << off;                 /* < 2^56 */
    acc->limb[li] += v & 0xFFFFFFFFu;
    acc->limb[li + 1] += v >> 32;
}

static void wide_normalise(wide_t *a)
{
    uint64_t carry = 0;
    for (int i = 0; i < WIDE_LIMBS; ++i) {
        uint64_t t = a->limb[i] + carry;
        a->limb[i] = t & 0xFFFFFFFFu;
        carry = t >> 32;
    }
}

static int wide_cmp(const wide_t *a, const wide_t *b)
{
    for (int i = WIDE_LIMBS - 1; i >= 0; --i) {
        if (a->limb[i] > b->limb[i]) return 1;
        if (a->limb[i] < b->limb[i]) return -1;
    }
    return 0;
}

/* Is every sum of up to eight of these magnitudes exactly representable in
 * fp64?  True when (highest possible bit of a sum) - (lowest set bit of any
 * element) fits in 53 bits. */
static int fp64_sums_exact(const double a[16])
{
    int top = -100000, low = 100000, any = 0;
    for (int t = 0; t < 16; ++t) {
        if (a[t] == 0.0) continue;
        int e;
        double m = frexp(a[t], &e);
        uint64_t mi = (uint64_t)ldexp(m, 53);
        int l = e - 53;
        while ((mi & 1u) == 0) { mi >>= 1; ++l; }
        if (e > top) top = e;   /* a[t] < 2^e */
        if (l < low) low = l;
        any = 1;
    }
    if (!any) return 1;
    return (top + 3) - low <= 53;  /* sum of 8 values < 2^(top+3) */
}

/* Best pattern for one block of magnitudes a[4i+j] = |w_ij|.
 * mode 0: fp64 sums when provably exact, wide accumulator otherwise;
 * mode 1: always the wide accumulator. */
static int block_argmax(const double a[16], const uint16_t *pat, int npat, int mode)
{
    int best = 0;
    if (mode == 0 && fp64_sums_exact(a)) {
        double best_s = -1.0;
        for (int k = 0; k < npat; ++k) {
            double s = 0.0;
            for (int t = 0; t < 16; ++t)
                if ((pat[k] >> t) & 1u) s += a[t];
            if (s > best_s) { best_s = s; best = k; }   /* strict: first maximum wins */
        }
        return best;
    }
    wide_t best_w;
    memset(&best_w, 0, sizeof best_w);
    for (int k = 0; k < npat; ++k) {
        wide_t s;
        memset(&s, 0, sizeof s);
        for (int t = 0; t < 16; ++t)
            if ((pat[k] >> t) & 1u) wide_add(&s, a[t]);
        wide_normalise(&s);
        if (k == 0 || wide_cmp(&s, &best_w) > 0) { best_w = s; best = k; }
    }
    return best;
}

/* mask[(r/4) x (q/4)] uint16 block masks, index (optional) = pattern id.
 * ldw = row stride of W in elements.  Returns 0, or -1 on a bad shape. */
int orc_transposable_mask(const void *W, int dt, int64_t r, int64_t q, int64_t ldw,
                          uint16_t *mask, uint8_t *index, int mode)
{
    if (r < 0 || q < 0 || (r % 4) || (q % 4) || ldw < q) return -1;
    uint16_t pat[90];
    if (orc_pattern_table(pat, 90) != 90) return -2;
    int64_t br = r / 4, bq = q / 4;
#pragma omp parallel for schedule(static)
    for (int64_t bi = 0; bi < br; ++bi) {
        for (int64_t bj = 0; bj < bq; ++bj) {
            double a[16];
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j)
                    a[4 * i + j] = fabs(widen(W, dt, (size_t)((4 * bi + i) * ldw + 4 * bj + j)));
            int k = block_argmax(a, pat, 90, mode);
            mask[bi * bq + bj] = pat[k];
            if (index) index[bi * bq + bj] = (uint8_t)k;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Unbiased 2:4 pruning of the output gradient for the weight-gradient */
/* GEMM (Eq. 4: grad W = S_z(grad Z^T) X; Eq. 6: S_z = MVUE).          */
/*                                                                     */
/* The paper names the estimator and cites it; it does not spell it    */
/* out.  What is built here follows from the two words: for a group    */
/* (a_0..a_3) keep two elements, element j with probability pi_j, and  */
/* store a_j / pi_j, so that the expectation is a_j (unbiased); the    */
/* total variance sum_j a_j^2 (1/pi_j - 1) under sum_j pi_j = 2,       */
/* pi_j <= 1 is least for pi_j proportional to |a_j|, capped at 1.     */
/*   uncapped (2 max|a| <= S = sum|a|): pi_j = 2|a_j|/S, kept value    */
/*     sign(a_j) S/2;                                                  */
/*   capped: the largest is kept as it is, one of the other three with */
/*     pi_j = |a_j|/R (R = S - max|a|, their sum), kept value          */
/*     sign(a_j) R.                                                    */
/* Two elements with these marginals are drawn by systematic sampling: */
/* one uniform u in [0,1) and the points u, u+1 on the line of the     */
/* cumulated pi.  All decisions are taken in fp32 in exactly the       */
/* operation order written below, and u comes from a counter-based     */
/* integer hash of (seed, feature, token group), so that another       */
/* implementation can reproduce every bit.                             */
/* ------------------------------------------------------------------ */

static uint16_t f32_to_half_bits(float f);   /* defined with orc_round_f16 below */

/* fp32 -> bf16 bits, round to nearest even (finite inputs) */
static uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

/* 23 random bits for (feature, token group): u = bits * 2^-23, so that u + 1 is exact in fp32 */
static uint32_t mvue_bits(uint32_t seed, uint32_t feature, uint32_t group)
{
    /* the seed is mixed on its own before it meets the feature, and that key before it meets the token group, so
       that neighbouring seeds (one per step and operand) share no draws in any rearrangement */
    const uint32_t key = mix32(mix32(seed) + feature * 0x9E3779B9U);
    return mix32(key + group * 0x85EBCA6BU) >> 9;
}

/* one group: a[4] in, kept positions i0 < i1 and their values out */
static void mvue_group(const float a[4], uint32_t bits, int *i0, int *i1, float *v0, float *v1)
{
    float m[4];
    for (int i = 0; i < 4; ++i) m[i] = fabsf(a[i]);
    const float S = (m[0] + m[1]) + (m[2] + m[3]);
    const float m01 = m[0] > m[1] ? m[0] : m[1], m23 = m[2] > m[3] ? m[2] : m[3];
    const float mx = m01 > m23 ? m01 : m23;
    const int capped = 2.0f * mx > S;          /* then mx is larger than the other three together: it is unique */
    const float R = S - mx;                    /* the others' sum, as fp32 gives it */
    const float D = capped ? R : S, scale = capped ? 1.0f : 2.0f;
    const float inv = D > 0.0f ? 1.0f / D : 0.0f;
    float pi[4], mag[4];
    for (int i = 0; i < 4; ++i) {
        const float t = (scale * m[i]) * inv;
        pi[i] = t < 1.0f ? t : 1.0f;
        mag[i] = capped ? R : 0.5f * S;
        if (capped && m[i] == mx) { pi[i] = 1.0f; mag[i] = m[i]; }
    }
    const float c1 = pi[0], c2 = c1 + pi[1], c3 = c2 + pi[2];
    const float u = (float)bits * 0x1p-23f, v = u + 1.0f;
    int a0 = (u >= c1) + (u >= c2) + (u >= c3);
    int a1 = (v >= c1) + (v >= c2) + (v >= c3);
    if (a1 == a0) {            /* only on rounding knife edges and in groups with fewer than two non-zeros */
        if (a0 < 3) a1 = a0 + 1;
        else { a0 = 2; a1 = 3; }
    }
    *i0 = a0; *i1 = a1;
    *v0 = m[a0] == 0.0f ? 0.0f : copysignf(mag[a0], a[a0]);
    *v1 = m[a1] == 0.0f ? 0.0f : copysignf(mag[a1], a[a1]);
}

/* dY [p][ld] (dtype dt) -> compressed S_z(dY^T): rows = the r features, contraction axis = the p tokens,
 * vals [r][p/2] (dtype dt, rounded to nearest even for bf16 and binary16), meta [r][p/16] as in orc_compress. */
int orc_mvue24(const void *dY, int dt, int64_t p, int64_t r, int64_t ld, uint32_t seed, void *vals, uint16_t *meta)
{
    if (p < 0 || r < 0 || (p % 16) || ld < r) return -1;
    const int64_t groups = p / 4;
#pragma omp parallel for schedule(static)
    for (int64_t f = 0; f < r; ++f) {
        for (int64_t w = 0; w < p / 16; ++w) meta[f * (p / 16) + w] = 0;
        for (int64_t g = 0; g < groups; ++g) {
            float a[4];
            for (int i = 0; i < 4; ++i) a[i] = (float)widen(dY, dt, (size_t)((4 * g + i) * ld + f));
            int i0, i1;
            float v0, v1;
            mvue_group(a, mvue_bits(seed, (uint32_t)f, (uint32_t)g), &i0, &i1, &v0, &v1);
            const size_t o = (size_t)(f * (p / 2) + 2 * g);
            if (dt == 0) {
                ((float *)vals)[o] = v0;
                ((float *)vals)[o + 1] = v1;
            } else if (dt == ORC_F16) {
                ((uint16_t *)vals)[o] = f32_to_half_bits(v0);
                ((uint16_t *)vals)[o + 1] = f32_to_half_bits(v1);
            } else {
                ((uint16_t *)vals)[o] = f32_to_bf16_bits(v0);
                ((uint16_t *)vals)[o + 1] = f32_to_bf16_bits(v1);
            }
            meta[f * (p / 16) + g / 4] |= (uint16_t)((i0 | (i1 << 2)) << (4 * (g % 4)));
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Monitors: flip count (Sec. 4.1, definition of the flip rate) and    */
/* L1-norm gap of a block (Sec. 4.2).                                  */
/* ------------------------------------------------------------------ */

/* total = || m_new - m_old ||_1 over all mask cells (each changed cell counts one); the flip rate is
 * total / (16 * nblocks).  block_flips (optional) accumulates every block's own count. */
int orc_mask_flips(const uint16_t *mask_new, const uint16_t *mask_old, int64_t nblocks, uint32_t *block_flips,
                   uint64_t *total)
{
    if (nblocks < 0) return -1;
    uint64_t sum = 0;
    for (int64_t b = 0; b < nblocks; ++b) {
        unsigned x = (unsigned)(mask_new[b] ^ mask_old[b]), c = 0;
        for (int t = 0; t < 16; ++t) c += (x >> t) & 1u;
        if (block_flips) block_flips[b] += c;
        sum += c;
    }
    *total = sum;
    return 0;
}

/* a - b for normalised a >= b, rounded once to the 64-bit significand of long double and then to double
 * (exact whenever the difference has at most 53 significant bits). */
static double wide_diff(const wide_t *a, const wide_t *b)
{
    int64_t d[WIDE_LIMBS];
    int64_t borrow = 0;
    for (int i = 0; i < WIDE_LIMBS; ++i) {
        int64_t t = (int64_t)a->limb[i] - (int64_t)b->limb[i] - borrow;
        borrow = t < 0;
        d[i] = t + (borrow << 32);
    }
    long double x = 0.0L;
    for (int i = WIDE_LIMBS - 1; i >= 0; --i) x = x * 4294967296.0L + (long double)d[i];
    return (double)ldexpl(x, -149);
}

/* gap[(r/4) x (q/4)]: for every block, the kept L1 norm of the best of the 90 patterns minus that of the
 * second best pattern (another pattern: zero when two patterns tie for the best), from exact sums. */
int orc_l1_norm_gap(const void *W, int dt, int64_t r, int64_t q, int64_t ldw, double *gap)
{
    if (r < 0 || q < 0 || (r % 4) || (q % 4) || ldw < q) return -1;
    uint16_t pat[90];
    if (orc_pattern_table(pat, 90) != 90) return -2;
    int64_t br = r / 4, bq = q / 4;
#pragma omp parallel for schedule(static)
    for (int64_t bi = 0; bi < br; ++bi) {
        for (int64_t bj = 0; bj < bq; ++bj) {
            double a[16];
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j)
                    a[4 * i + j] = fabs(widen(W, dt, (size_t)((4 * bi + i) * ldw + 4 * bj + j)));
            wide_t first, second;
            memset(&first, 0, sizeof first);
            memset(&second, 0, sizeof second);
            for (int k = 0; k < 90; ++k) {
                wide_t s;
                memset(&s, 0, sizeof s);
                for (int t = 0; t < 16; ++t)
                    if ((pat[k] >> t) & 1u) wide_add(&s, a[t]);
                wide_normalise(&s);
                if (k == 0) { first = s; continue; }
                if (wide_cmp(&s, &first) > 0) { second = first; first = s; }
                else if (k == 1 || wide_cmp(&s, &second) > 0) second = s;
            }
            gap[bi * bq + bj] = wide_diff(&first, &second);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Compress ("enforcing the mask", Sec. 5 item 1; sparse_W and         */
/* sparse_W_T of the workflow in App. B).                              */
/* ------------------------------------------------------------------ */

static int mask_bit(const uint16_t *mask, int64_t bq, int64_t row, int64_t col)
{
    uint16_t b = mask[(row / 4) * bq + (col / 4)];
    return (b >> (4 * (row % 4) + (col % 4))) & 1;
}

/* vals[r][q/2], meta[r][q/16] (uint16) for W along q; valsT[q][r/2],
 * metaT[q][r/16] for W^T along r.  Element size follows dt (4 or 2 bytes);
 * values are bit copies.  Needs q % 16 == 0 and r % 16 == 0 for whole
 * metadata words.  Returns 0, -1 bad shape, -3 if a group does not hold
 * exactly two kept elements. */
int orc_compress(const void *W, int dt, int64_t r, int64_t q, int64_t ldw, const uint16_t *mask,
                 void *vals, uint16_t *meta, void *valsT, uint16_t *metaT)
{
    if (r <= 0 || q <= 0 || (r % 16) || (q % 16) || ldw < q) return -1;
    size_t es = dt == ORC_F32 ? 4 : 2;
    int64_t bq = q / 4;
    int bad = 0;
    memset(meta, 0, (size_t)(r * (q / 16)) * sizeof(uint16_t));
    memset(metaT, 0, (size_t)(q * (r / 16)) * sizeof(uint16_t));
    /* W along q */
    for (int64_t o = 0; o < r; ++o)
        for (int64_t g = 0; g < q / 4; ++g) {
            int kept[4], n = 0;
            for (int c = 0; c < 4; ++c)
                if (mask_bit(mask, bq, o, 4 * g + c)) kept[n < 4 ? n++ : 3] = c;
            if (n != 2) { bad = 1; continue; }
            for (int s = 0; s < 2; ++s)
                memcpy((char *)vals + (size_t)(o * (q / 2) + 2 * g + s) * es,
                       (const char *)W + (size_t)(o * ldw + 4 * g + kept[s]) * es, es);
            unsigned nib = (unsigned)kept[0] | ((unsigned)kept[1] << 2);
            meta[o * (q / 16) + g / 4] |= (uint16_t)(nib << (4 * (g % 4)));
        }
    /* W^T along r: row i of W^T is column i of W */
    for (int64_t i = 0; i < q; ++i)
        for (int64_t g = 0; g < r / 4; ++g) {
            int kept[4], n = 0;
            for (int c = 0; c < 4; ++c)
                if (mask_bit(mask, bq, 4 * g + c, i)) kept[n < 4 ? n++ : 3] = c;
            if (n != 2) { bad = 1; continue; }
            for (int s = 0; s < 2; ++s)
                memcpy((char *)valsT + (size_t)(i * (r / 2) + 2 * g + s) * es,
                       (const char *)W + (size_t)((4 * g + kept[s]) * ldw + i) * es, es);
            unsigned nib = (unsigned)kept[0] | ((unsigned)kept[1] << 2);
            metaT[i * (r / 16) + g / 4] |= (uint16_t)(nib << (4 * (g % 4)));
        }
    return bad ? -3 : 0;
}

/* Re-layout of a compressed operand for the matrix-core kernels (a permutation,
 * no arithmetic).  The paper leaves the compressed format to its spMM library;
 * the reading taken here groups the contraction axis in chunks of 64: chunk c
 * of row o holds 32 kept values and 4 metadata words, and all rows of one chunk
 * are stored together:
 *     vals_p[c][o][0..31] = vals[o][32c .. 32c+31]
 *     meta_p[c][o][0..3]  = meta[o][4c .. 4c+3]
 * R rows, K = contraction length (multiple of 64). */
int orc_pack_chunk_major(const void *vals, const uint16_t *meta, int dt, int64_t R, int64_t K,
                         void *vals_p, uint16_t *meta_p)
{
    if (R < 0 || K < 0 || K % 64) return -1;
    size_t es = dt == ORC_F32 ? 4 : 2;
    int64_t nc = K / 64;
    for (int64_t c = 0; c < nc; ++c)
        for (int64_t o = 0; o < R; ++o) {
            for (int j = 0; j < 32; ++j)
                memcpy((char *)vals_p + (size_t)((c * R + o) * 32 + j) * es,
                       (const char *)vals + (size_t)(o * (K / 2) + 32 * c + j) * es, es);
            for (int j = 0; j < 4; ++j)
                meta_p[(c * R + o) * 4 + j] = meta[o * (K / 16) + 4 * c + j];
        }
    return 0;
}

static int meta_idx(const uint16_t *meta, int64_t words_per_row, int64_t row, int64_t g, int s)
{
    unsigned nib = (meta[row * words_per_row + g / 4] >> (4 * (g % 4))) & 0xFu;
    return (int)((nib >> (2 * s)) & 3u);
}

/* ------------------------------------------------------------------ */
/* GEMMs (Eq. 1-3).  `rows`, when not NULL, lists the nrows output     */
/* rows to compute (so large shapes can be sampled); otherwise all.    */
/* ------------------------------------------------------------------ */

/* Y[t][o] = sum_g sum_s vals[o][2g+s] * X[t][4g + idx_s]   (Eq. 2) */
int orc_spmm_fwd(const void *X, const void *vals, const uint16_t *meta, int dt,
                 int64_t p, int64_t q, int64_t r, const int64_t *rows, int64_t nrows, double *Y)
{
    if (q % 16 || r % 4) return -1;
    if (!rows) nrows = p;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < nrows; ++n) {
        int64_t t = rows ? rows[n] : n;
        for (int64_t o = 0; o < r; ++o) {
            double acc = 0.0;
            for (int64_t g = 0; g < q / 4; ++g)
                for (int s = 0; s < 2; ++s) {
                    int c = meta_idx(meta, q / 16, o, g, s);
                    acc += widen(vals, dt, (size_t)(o * (q / 2) + 2 * g + s)) *
                           widen(X, dt, (size_t)(t * q + 4 * g + c));
                }
            Y[n * r + o] = acc;
        }
    }
    return 0;
}

/* dX[t][i] = beta*dX0[t][i] + sum_g sum_s valsT[i][2g+s] * dY[t][4g + idx_s]   (Eq. 3) */
int orc_spmm_bwd_dx(const void *dY, const void *valsT, const uint16_t *metaT, int dt,
                    int64_t p, int64_t q, int64_t r, double beta, const double *dX0,
                    const int64_t *rows, int64_t nrows, double *dX)
{
    if (r % 16 || q % 4) return -1;
    if (!rows) nrows = p;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < nrows; ++n) {
        int64_t t = rows ? rows[n] : n;
        for (int64_t i = 0; i < q; ++i) {
            double acc = 0.0;
            for (int64_t g = 0; g < r / 4; ++g)
                for (int s = 0; s < 2; ++s) {
                    int c = meta_idx(metaT, r / 16, i, g, s);
                    acc += widen(valsT, dt, (size_t)(i * (r / 2) + 2 * g + s)) *
                           widen(dY, dt, (size_t)(t * r + 4 * g + c));
                }
            dX[n * q + i] = (dX0 ? beta * dX0[n * q + i] : 0.0) + acc;
        }
    }
    return 0;
}

/* dW[o][i] = beta*dW0[o][i] + sum_t dY[t][o] * X[t][i]   (Eq. 1, third GEMM; dense).
 * rows selects output rows o. dW0 is indexed like the output. */
int orc_dense_dw(const void *dY, const void *X, int dt, int64_t p, int64_t q, int64_t r,
                 double beta, const double *dW0, const int64_t *rows, int64_t nrows, double *dW)
{
    if (!rows) nrows = r;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < nrows; ++n) {
        int64_t o = rows ? rows[n] : n;
        for (int64_t i = 0; i < q; ++i) {
            double acc = 0.0;
            for (int64_t t = 0; t < p; ++t)
                acc += widen(dY, dt, (size_t)(t * r + o)) * widen(X, dt, (size_t)(t * q + i));
            dW[n * q + i] = (dW0 ? beta * dW0[n * q + i] : 0.0) + acc;
        }
    }
    return 0;
}

/* Y[t][o] = sum_i X[t][i] * W[o][i]   (Eq. 1, first GEMM; dense comparison) */
int orc_dense_gemm(const void *X, const void *W, int dt, int64_t p, int64_t q, int64_t r,
                   const int64_t *rows, int64_t nrows, double *Y)
{
    if (!rows) nrows = p;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < nrows; ++n) {
        int64_t t = rows ? rows[n] : n;
        for (int64_t o = 0; o < r; ++o) {
            double acc = 0.0;
            for (int64_t i = 0; i < q; ++i)
                acc += widen(X, dt, (size_t)(t * q + i)) * widen(W, dt, (size_t)(o * q + i));
            Y[n * r + o] = acc;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Masked decay on gradients (Eq. 10): G = dW + lambda * (not m) .* W  */
/* ------------------------------------------------------------------ */
int orc_masked_decay(const float *dW, const void *W, int wdt, const uint16_t *mask, float lambda,
                     int64_t r, int64_t q, double *G)
{
    if (r % 4 || q % 4) return -1;
    int64_t bq = q / 4;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < r; ++o)
        for (int64_t i = 0; i < q; ++i) {
            double g = (double)dW[o * q + i];
            if (!mask_bit(mask, bq, o, i)) g += (double)lambda * widen(W, wdt, (size_t)(o * q + i));
            G[o * q + i] = g;
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Activations (Sec. 5.2).  Gated: act(Z1) .* Z2 with the gate first;  */
/* SwiGLU uses silu(x) = x * sigmoid(x), no biases.                    */
/* ------------------------------------------------------------------ */
static double sigmoid(double x)
{
    if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

/* G, U are p x f matrices with row stride ld (elements); H is p x f dense. */
int orc_swiglu_fwd(const void *G, const void *U, int dt, int64_t p, int64_t f, int64_t ld, double *H)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < p; ++t)
        for (int64_t c = 0; c < f; ++c) {
            double g = widen(G, dt, (size_t)(t * ld + c)), u = widen(U, dt, (size_t)(t * ld + c));
            H[t * f + c] = g * sigmoid(g) * u;
        }
    return 0;
}

/* dG = dH .* U .* silu'(G), dU = dH .* silu(G); silu'(x) = s(x) (1 + x (1 - s(x))).
 * dH is p x f dense; G, U have row stride ld; dG, dU dense p x f. */
int orc_swiglu_bwd(const void *dH, const void *G, const void *U, int dt, int64_t p, int64_t f,
                   int64_t ld, double *dG, double *dU)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < p; ++t)
        for (int64_t c = 0; c < f; ++c) {
            double g = widen(G, dt, (size_t)(t * ld + c)), u = widen(U, dt, (size_t)(t * ld + c));
            double d = widen(dH, dt, (size_t)(t * f + c));
            double s = sigmoid(g);
            dG[t * f + c] = d * u * s * (1.0 + g * (1.0 - s));
            dU[t * f + c] = d * g * s;
        }
    return 0;
}

int orc_act_fwd(const void *Z, int dt, int64_t n, int act, double *H)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        double z = widen(Z, dt, (size_t)k);
        if (act == ORC_ACT_RELU) H[k] = z > 0.0 ? z : 0.0;
        else H[k] = 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
    }
    return 0;
}

/* dZ = dH .* act'(Z); relu'(0) := 0; gelu'(z) = Phi(z) + z phi(z). */
int orc_act_bwd(const void *dH, const void *Z, int dt, int64_t n, int act, double *dZ)
{
    const double inv_sqrt_2pi = 0.39894228040143267794;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        double z = widen(Z, dt, (size_t)k), d = widen(dH, dt, (size_t)k), dz;
        if (act == ORC_ACT_RELU) dz = z > 0.0 ? 1.0 : 0.0;
        else dz = 0.5 * (1.0 + erf(z / sqrt(2.0))) + z * inv_sqrt_2pi * exp(-0.5 * z * z);
        dZ[k] = d * dz;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Gated activation on the output Z = [Z1 | Z2] of the concatenated    */
/* gate/up GEMM (Sec. 5.2 step 3): H = act(Z1) .* Z2, act = GELU (the   */
/* paper's GEGLU) or SiLU (SwiGLU).  Z is p x 2r, H is p x r; each is   */
/* stored row-major (element (t,c) at t*ld + c) or, as the activations  */
/* of the paper's sparse GEMMs are (App. A.2), column-major (c*ld + t). */
/* The biases of Sec. 5.2 belong to step 2: they are part of Z.         */
/* ------------------------------------------------------------------ */
static size_t at(int layout, int64_t ld, int64_t t, int64_t c)
{
    return (size_t)(layout == ORC_COL_MAJOR ? c * ld + t : t * ld + c);
}

static double gate_value(int gate, double x)
{
    return gate == ORC_GATE_SILU ? x * sigmoid(x) : 0.5 * x * (1.0 + erf(x / sqrt(2.0)));
}

static double gate_slope(int gate, double x)
{
    if (gate == ORC_GATE_SILU) {
        double s = sigmoid(x);
        return s * (1.0 + x * (1.0 - s));
    }
    return 0.5 * (1.0 + erf(x / sqrt(2.0))) + x * 0.39894228040143267794 * exp(-0.5 * x * x);
}

/* H (dense p x r, row-major fp64) = act(Z1) .* Z2 */
int orc_glu_fwd(const void *Z, int dt, int layout, int64_t ldz, int64_t p, int64_t r, int gate, double *H)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < p; ++t)
        for (int64_t c = 0; c < r; ++c) {
            double z1 = widen(Z, dt, at(layout, ldz, t, c)), z2 = widen(Z, dt, at(layout, ldz, t, r + c));
            H[t * r + c] = gate_value(gate, z1) * z2;
        }
    return 0;
}

/* dZ (dense p x 2r, row-major fp64) = [dH .* Z2 .* act'(Z1) | dH .* act(Z1)]; dH is p x r in its own layout */
int orc_glu_bwd(const void *dH, int layout_h, int64_t ldh, const void *Z, int dt, int layout, int64_t ldz, int64_t p,
                int64_t r, int gate, double *dZ)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < p; ++t)
        for (int64_t c = 0; c < r; ++c) {
            double z1 = widen(Z, dt, at(layout, ldz, t, c)), z2 = widen(Z, dt, at(layout, ldz, t, r + c));
            double d = widen(dH, dt, at(layout_h, ldh, t, c));
            dZ[t * 2 * r + c] = d * z2 * gate_slope(gate, z1);
            dZ[t * 2 * r + r + c] = d * gate_value(gate, z1);
        }
    return 0;
}

/* Gradient of the bias d of Z = X W^T + d (Sec. 5.2 step 2): db[c] = sum over tokens of dZ[t][c]. */
int orc_bias_grad(const void *dZ, int dt, int layout, int64_t ld, int64_t p, int64_t n, double *db)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n; ++c) {
        double s = 0.0;
        for (int64_t t = 0; t < p; ++t) s += widen(dZ, dt, at(layout, ld, t, c));
        db[c] = s;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Round fp64 -> binary16 the way a GPU epilogue does from its fp32    */
/* accumulator: fp64 -> fp32 (the C cast, round to nearest even), then */
/* fp32 -> binary16, round to nearest even, overflow to infinity,      */
/* gradual underflow.                                                  */
/* ------------------------------------------------------------------ */
static uint16_t f32_to_half_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);            /* NaN */
    if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);           /* >= 65520 rounds to infinity */
    /* the nearest multiple of the target spacing: 2^(e-10) for |x| in [2^e, 2^(e+1)), e >= -14; 2^-24 below */
    double m = fabs((double)f);
    int e;
    (void)frexp(m, &e);                  /* m = frac * 2^e, frac in [0.5, 1): binade exponent is e - 1 */
    int q = (e - 1 < -14 ? -14 : e - 1) - 10;
    double scaled = ldexp(m, -q);        /* exact */
    double n = nearbyint(scaled);        /* default rounding mode: to nearest, ties to even */
    double v = ldexp(n, q);              /* a binary16 value, possibly the next binade's first */
    /* encode v */
    if (v == 0.0) return sign;
    (void)frexp(v, &e);
    if (e - 1 < -14) return (uint16_t)(sign | (uint16_t)ldexp(v, 24));
    return (uint16_t)(sign | (uint16_t)(((e - 1 + 15) << 10) + ((int)ldexp(v, 10 - (e - 1)) - 1024)));
}

void orc_round_f16(const double *x, int64_t n, uint16_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) out[k] = f32_to_half_bits((float)x[k]);
}

/* ------------------------------------------------------------------ */
/* Round fp64 -> bf16 (round-to-nearest-even), so a chained reference  */
/* can hand each stage the same rounded activations the GPU stages see.*/
/* ------------------------------------------------------------------ */
void orc_round_bf16(const double *x, int64_t n, uint16_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        float f = (float)x[k]; /* fp32 first: the GPU rounds its fp32 accumulator */
        uint32_t u;
        memcpy(&u, &f, 4);
        if ((u & 0x7F800000u) == 0x7F800000u) { out[k] = (uint16_t)(u >> 16); continue; }
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7FFFu + lsb;
        out[k] = (uint16_t)(u >> 16);
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
