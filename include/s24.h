/*
 * s24 -- the 2:4-sparse FFN training step of arXiv 2404.01847 on AMD MI355X (gfx950).
 *
 * C ABI.  Notation follows the paper (Sec. 3.1): X is p x q (tokens x
 * in-features, batch and sequence axes flattened), W is r x q (out-features x
 * in-features), Z/Y is p x r.  Every matrix is row-major and dense in memory
 * unless a leading dimension is given.
 *
 * Pointers: every data pointer is a DEVICE pointer owned by the caller, except
 * where a comment says "host".  The library never allocates, frees or
 * synchronises; each call only enqueues kernels on `stream` (a hipStream_t
 * passed as void*, NULL = the default stream) and returns.
 *
 * Limits: every size is below 2^31, and the feature extents of the GEMM entry points (q, r, 2f) below 2^23: the
 * kernels address one tile's operand rows with 32-bit byte offsets from a per-tile base (S24_ERR_SHAPE beyond).
 *
 * Errors: every entry point returns an s24_status.  Arguments are validated on
 * the host before anything is launched, so a failing call has no effect on
 * device memory.  Nothing throws or aborts.  Inputs are assumed finite.
 *
 * Data formats
 *   block mask   uint16 per aligned 4x4 block, mask[(r/4)][(q/4)], bit (4i+j) =
 *                m_ij (i = row, j = column inside the block).
 *   pattern id   the 90 legal blocks (two ones in every row and column) are
 *                numbered in lexicographic order of the 16-character row-major
 *                string m00 m01 ... m33 with '0' < '1'.
 *   compressed   for a matrix A (R x K, K a multiple of 64) that keeps exactly two
 *                of every four consecutive elements along K.  Per row the kept
 *                elements in order (bit copies) form K/2 values, and every 16
 *                columns give one uint16 of metadata: group g (columns
 *                4g..4g+3) contributes the nibble  i0 | i1 << 2  (i0 < i1 the
 *                kept column offsets) at bits 4*(g mod 4) of word g/4.
 *                Storage is chunk-major, 64 columns per chunk, all rows of a
 *                chunk together:  vals[K/64][R][32]  (value j of chunk c of row
 *                o is the row's kept value 32c+j)  and  meta[K/64][R][4]  (word
 *                4c+j of the row).  One chunk of one row is exactly what one
 *                lane pair feeds to two sparse matrix-core instructions.
 *   dtypes       S24_BF16 buffers hold raw bfloat16, S24_F16 buffers IEEE binary16 (the paper trains in fp16
 *                mixed precision, Sec. 6), S24_F32 buffers float.  Both 16-bit types run the same kernels on
 *                the matrix cores (fp32 accumulation, one rounding to the storage type); S24_F32 runs plain
 *                fp32 kernels kept for checking.  binary16 results overflow to infinity like any IEEE
 *                conversion: scaling the loss is the caller's business.
 *   layouts      a logical [p][n] activation matrix is S24_ROW_MAJOR (element (t, c) at t*ld + c) or
 *                S24_COL_MAJOR (at c*ld + t, the layout the paper's sparse GEMMs emit, App. A.2).  The GEMMs of
 *                this library read and write row-major; the gated activation and the bias gradient take both.
 */
#ifndef S24_H
#define S24_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    S24_OK = 0,
    S24_ERR_NULL = -1,        /* a required pointer is NULL */
    S24_ERR_SHAPE = -2,       /* a size is negative or not a multiple of what the call needs */
    S24_ERR_DTYPE = -3,       /* unknown dtype / activation enum */
    S24_ERR_ALIGN = -4,       /* a pointer or leading dimension breaks the 16-byte alignment rule */
    S24_ERR_LAUNCH = -5,      /* the HIP runtime refused a launch */
    S24_ERR_UNSUPPORTED = -6  /* valid request that this build does not implement */
} s24_status;

typedef enum { S24_F32 = 0, S24_BF16 = 1, S24_F16 = 2 } s24_dtype;   /* S24_F16: IEEE binary16, the paper's own precision (Sec. 6) */
typedef enum { S24_ACT_RELU = 0, S24_ACT_GELU_ERF = 1 } s24_act;
typedef enum { S24_GATE_SILU = 0, S24_GATE_GELU_ERF = 1 } s24_gate;     /* SwiGLU / GEGLU (Sec. 5.2) */
typedef enum { S24_ROW_MAJOR = 0, S24_COL_MAJOR = 1 } s24_layout;       /* element (t, c) at t*ld + c / c*ld + t */

#define S24_NUM_PATTERNS 90

/* Text for a status code (host, static storage). */
const char *s24_strerror(int status);

/* The 90 legal block masks in pattern-id order (Sec. 5.1, step 1: the mask
 * blocks found by exhaustive inspection, n_t = 90).  `out` is a HOST array. */
int s24_pattern_table(uint16_t out[S24_NUM_PATTERNS]);

/* Transposable mask search (Sec. 5.1 problem formulation; Alg. 1).
 * For every aligned 4x4 block of W picks, among the 90 legal patterns, the one
 * that keeps the largest sum of |w|; scores are compared exactly and ties go
 * to the smallest pattern id.
 *   W      [r][ldw] device, dtype dt, ldw >= q elements
 *   mask   [r/4][q/4] device, out
 *   index  [r/4][q/4] device, out, pattern ids; may be NULL
 * r, q multiples of 4 (S24_ERR_SHAPE otherwise); W and ldw*elemsize 8-byte
 * aligned for the 16-bit types, 16-byte for f32 (S24_ERR_ALIGN). */
int s24_transposable_mask(const void *W, s24_dtype dt, int64_t r, int64_t q, int64_t ldw,
                          uint16_t *mask, uint8_t *index, void *stream);

/* Prune and compress (Sec. 5 item 1 "enforcing the mask"; the sparse_W and
 * sparse_W_T operands of the App. B workflow).  Emits the compressed form of
 * M.*W along q (vals, meta) and of (M.*W)^T along r (valsT, metaT).
 *   mask      [r/4][q/4] device, in; NULL = search the mask in the same pass
 *   vals      [q/64][r][32]  meta  [q/64][r][4]    (rows of W, chunks along q)
 *   valsT     [r/64][q][32]  metaT [r/64][q][4]    (rows of W^T, chunks along r)
 *   mask_out  [r/4][q/4] device, out, may be NULL (only used when mask == NULL)
 * r, q multiples of 64; vals and valsT 16-byte aligned, meta and metaT 8-byte aligned (S24_ERR_ALIGN).  A given
 * mask must be legal (two kept per row and column of each block); an illegal mask gives unspecified values but no
 * fault.  The chunk-major storage described at the top of this file is the only form the library emits or reads:
 * it is what the sparse matrix-core instructions consume verbatim, and it is a pure permutation of the row-major
 * form (value j of chunk c of row o <-> kept value 32c + j of that row; word j of chunk c <-> word 4c + j). */
int s24_compress(const void *W, s24_dtype dt, int64_t r, int64_t q, int64_t ldw,
                 const uint16_t *mask, void *vals, uint16_t *meta, void *valsT, uint16_t *metaT,
                 uint16_t *mask_out, void *stream);

/* Forward sparse GEMM (Eq. 2):  Y[p][r] = X[p][q] . (M.*W)^T, contraction over
 * q against the compressed weight (vals [q/64][r][32], meta [q/64][r][4]).
 * 16-bit in / fp32 accumulate / 16-bit out (f32 throughout for S24_F32).
 * p >= 1; q multiple of 64; r multiple of 16. */
int s24_spmm_fwd(const void *X, const void *vals, const uint16_t *meta, void *Y,
                 int64_t p, int64_t q, int64_t r, s24_dtype dt, void *stream);

/* Z = X (M.*W)^T + d (Sec. 5.2 step 2): s24_spmm_fwd with the bias d[r] (dtype dt, 8-byte aligned, may be NULL)
 * added to the fp32 accumulator before the one rounding to the storage type. */
int s24_spmm_fwd_bias(const void *X, const void *vals, const uint16_t *meta, const void *bias, void *Y,
                      int64_t p, int64_t q, int64_t r, s24_dtype dt, void *stream);

/* The three steps of Sec. 5.2 in one pass, for either gate: the compressed operand holds the stacked weight
 * [W_gate; W_up] as in s24_spmm_fwd_swiglu, bias is the stacked d[2f] or NULL.  Writes
 * GU[p][2f] = Z = X (M.*W)^T + d and H[p][f] = act(Z_1) .* Z_2 (act = GELU for S24_GATE_GELU_ERF, the paper's
 * GEGLU; SiLU for S24_GATE_SILU), Z rounded to the storage type before H is formed: the same bits as
 * s24_spmm_fwd_bias followed by s24_glu_fwd.  q multiple of 64; f multiple of 16. */
int s24_spmm_fwd_glu(const void *X, const void *vals, const uint16_t *meta, const void *bias, void *GU, void *H,
                     int64_t p, int64_t q, int64_t f, s24_gate gate, s24_dtype dt, void *stream);

/* s24_spmm_bwd_dx_swiglu for either gate: dGU[p][2f] = [dH .* Z_2 .* act'(Z_1) | dH .* act(Z_1)] with
 * dH = dY (M.*W_down) consumed tile by tile.  Same bits as s24_spmm_bwd_dx followed by s24_glu_bwd; the same
 * S24_ERR_UNSUPPORTED rule (fp32, or fewer output tiles of 256 x 256 than three quarters of the device's compute units:
 * 192 on MI355X). */
int s24_spmm_bwd_dx_glu(const void *dY, const void *valsT, const uint16_t *metaT, const void *GU, void *dGU,
                        int64_t p, int64_t f, int64_t r, s24_gate gate, s24_dtype dt, void *stream);

/* Forward of an ungated layer with its activation in the same pass (Eq. 2; the ReLU / GELU layers of the
 * GPT-2-shaped workloads): Z[p][r] = X (M.*W)^T + bias (bias may be NULL) and H[p][r] = act(Z), Z rounded to the
 * storage type before H is formed: the same bits as s24_spmm_fwd_bias followed by s24_act_fwd. */
int s24_spmm_fwd_act(const void *X, const void *vals, const uint16_t *meta, const void *bias, void *Z, void *H,
                     int64_t p, int64_t q, int64_t r, s24_act act, s24_dtype dt, void *stream);

/* Input gradient of the second projection of an ungated layer with the backward of the activation in the same pass
 * (Eq. 3): dZ[p][f] = (dY[p][r] (M.*W_2)) .* act'(Z), the product rounded to the storage type before the
 * multiplication: the same bits as s24_spmm_bwd_dx followed by s24_act_bwd.  fp32 returns S24_ERR_UNSUPPORTED and
 * leaves everything untouched (use the two calls).  r multiple of 64; f of 16. */
int s24_spmm_bwd_dx_act(const void *dY, const void *valsT, const uint16_t *metaT, const void *Z, void *dZ,
                        int64_t p, int64_t f, int64_t r, s24_act act, s24_dtype dt, void *stream);

/* Forward of a gated layer in one pass (Eq. 2 + Sec. 5.2): the compressed operand holds the stacked weight
 * [W_gate; W_up] (2f rows of q, gate rows first: vals [q/64][2f][32], meta [q/64][2f][4]).  Writes
 * GU[p][2f] = X . (M.*W)^T (its halves are G = Z_1 and U = Z_2, both needed by the backward pass) and
 * H[p][f] = silu(G) .* U with G and U rounded to the storage type first, i.e. the same bits as s24_spmm_fwd
 * followed by s24_swiglu_fwd on the halves.  q multiple of 64; f multiple of 16. */
int s24_spmm_fwd_swiglu(const void *X, const void *vals, const uint16_t *meta, void *GU, void *H, int64_t p,
                        int64_t q, int64_t f, s24_dtype dt, void *stream);

/* Backward sparse GEMM for the input gradient (Eq. 3):
 * dX[p][q] = beta*dX + dY[p][r] . (M.*W), contraction over r against the
 * compressed transpose (valsT [r/64][q][32], metaT [r/64][q][4]); legal because the
 * mask is transposable (Eq. 5).  beta is 0 or 1 (1 sums the gate and up
 * branches of a gated FFN).  r multiple of 64; q multiple of 16. */
int s24_spmm_bwd_dx(const void *dY, const void *valsT, const uint16_t *metaT, void *dX,
                    int64_t p, int64_t q, int64_t r, float beta, s24_dtype dt, void *stream);

/* Input gradient of the down projection of a gated layer with the backward of the activation in the same pass
 * (Eq. 3 + Sec. 5.2): dH = dY[p][r] . (M.*W_down) (valsT [r/64][f][32], metaT [r/64][f][4]) is formed tile by
 * tile, rounded to the storage type and consumed on the spot:  dGU[p][2f] = [dH .* U .* silu'(G) | dH .* silu(G)]
 * with G and U the halves of GU[p][2f].  Same bits as s24_spmm_bwd_dx followed by s24_swiglu_bwd.  Only the
 * large-tile 16-bit kernel has this epilogue: fp32, and outputs of fewer tiles of 256 x 256 than three quarters of the
 * device's compute units (192 on MI355X), return
 * S24_ERR_UNSUPPORTED and leave everything untouched (use the two calls).  r multiple of 64; f of 16. */
int s24_spmm_bwd_dx_swiglu(const void *dY, const void *valsT, const uint16_t *metaT, const void *GU, void *dGU,
                           int64_t p, int64_t f, int64_t r, s24_dtype dt, void *stream);

/* Dense weight gradient (Eq. 1, third GEMM; straight-through estimator):
 * dW[r][q] = beta*dW + dY[p][r]^T . X[p][q], fp32 output, beta 0 or 1
 * (1 accumulates over micro-batches).  q, r multiples of 16. */
int s24_dense_dw(const void *dY, const void *X, float *dW, int64_t p, int64_t q, int64_t r,
                 float beta, s24_dtype dt, void *stream);

/* Weight gradient with the masked decay term added in the same pass (Eq. 1 third GEMM + Eq. 10):
 * dW[r][q] = beta*dW + dY^T . X + lambda * W on the cells the mask prunes.  W [r][q] (dtype wdt, dense)
 * and mask [r/4][q/4] as in s24_masked_decay_grad; everything else as in s24_dense_dw.  The result has
 * the same bits as s24_dense_dw followed by s24_masked_decay_grad.  The decay term does not depend on
 * the batch: with beta = 1 accumulation over micro-batches it is passed (lambda != 0) once. */
int s24_dense_dw_decay(const void *dY, const void *X, float *dW, const void *W, s24_dtype wdt,
                       const uint16_t *mask, float lambda, int64_t p, int64_t q, int64_t r, float beta,
                       s24_dtype dt, void *stream);

/* Several weight gradients in one pass (Eq. 1 + Eq. 10 for up to four weights of a layer, e.g. the two or three of
 * an FFN): the same result, bit for bit, as s24_dense_dw_decay (W != NULL) or s24_dense_dw (W == NULL) on each
 * problem with the same beta, but the tiles of all problems share one grid, so that the compute units which the
 * last, partial round of one GEMM would leave idle take tiles of the next, and if the joint tile count exceeds a
 * whole number of rounds by at most half a round, that excess is cut off as whole tile columns or rows of one
 * problem and run in small tiles.  `problems` is a HOST array of `count` <= 4 entries, read during the call:
 *   dY [p][r], X [p][q] (dtype dt), dW [r][q] fp32, W [r][q] (dtype dt) or NULL, mask [r/4][q/4] (with W), lambda.
 * Problems that are each too small for the large tile share one grid of small tiles in the same way.  Problems that
 * fit neither shared grid (fp32, no tokens, an empty output, small and large outputs mixed, decay on some but not
 * all) are run one after the other instead.  All problems are validated before the first launch. */
typedef struct {
    const void *dY;
    const void *X;
    float *dW;
    const void *W;
    const uint16_t *mask;
    int64_t p, q, r;
    float lambda;
} s24_dw_problem;
int s24_dense_dw_batch(const s24_dw_problem *problems, int count, float beta, s24_dtype dt, void *stream);

/* Unbiased 2:4 pruning of the output gradient (Eq. 6: S_z = MVUE) into the compressed operand of the sparse
 * weight-gradient GEMM (Eq. 4).  Of every four consecutive tokens of one feature two are kept, element j with
 * probability pi_j proportional to |dY_j| (capped at one) and stored as dY_j / pi_j; the pair is drawn by
 * systematic sampling from one uniform number per group, a counter-based hash of (seed, feature, group), so
 * the result is a pure function of its arguments.
 *   dY     [p][ld] device, dtype dt, ld >= r
 *   vals   [p/64][r][32] (dtype dt), meta [p/64][r][4]: the compressed form of S_z(dY^T), whose rows are the r
 *          features and whose contraction axis is the p tokens, in the chunk-major storage described above
 * p multiple of 64. */
int s24_mvue24(const void *dY, s24_dtype dt, int64_t p, int64_t r, int64_t ld, uint32_t seed, void *vals,
               uint16_t *meta, void *stream);

/* Sparse weight gradient (Eq. 4): dW[r][q] = beta*dW + S_z(dY^T) . X (+ lambda * W on pruned cells when W is
 * not NULL, as in s24_dense_dw_decay), contraction over the p tokens against the compressed operand made by
 * s24_mvue24 (vals [p/64][r][32], meta [p/64][r][4]).  X [p][q], fp32 output.  p multiple of 64; q, r of 16. */
int s24_spmm_dw(const void *vals, const uint16_t *meta, const void *X, float *dW, const void *W, s24_dtype wdt,
                const uint16_t *mask, float lambda, int64_t p, int64_t q, int64_t r, float beta, s24_dtype dt,
                void *stream);

/* Dense comparison GEMM (Eq. 1, first GEMM): Y[p][r] = X[p][q] . W[r][q]^T,
 * same tiling family as the sparse kernels.  q multiple of 64; r of 16. */
int s24_dense_gemm(const void *X, const void *W, void *Y, int64_t p, int64_t q, int64_t r,
                   s24_dtype dt, void *stream);

/* Masked decay on gradients (Eq. 10), in place:
 * G[r][q] (fp32) += lambda * W on the cells the mask prunes; kept cells are
 * left bit-identical.  W has dtype wdt; mask is [r/4][q/4].  q multiple of 16. */
int s24_masked_decay_grad(float *G, const void *W, s24_dtype wdt, const uint16_t *mask,
                          float lambda, int64_t r, int64_t q, void *stream);

/* Gated activation (Sec. 5.2, with SiLU in place of GELU and no biases):
 * H[p][f] = silu(G) .* U, the gate G being the first operand (Z_1).  G and U
 * are p x f with row stride ld_gu elements (so they may be the two halves of
 * one [p][2f] buffer); H is dense.  f, ld_gu multiples of 8. */
int s24_swiglu_fwd(const void *G, const void *U, void *H, int64_t p, int64_t f, int64_t ld_gu,
                   s24_dtype dt, void *stream);

/* Backward of the gated activation: dG = dH .* U .* silu'(G), dU = dH .* silu(G),
 * silu'(x) = s(x)(1 + x(1 - s(x))).  dH is dense p x f; dG, dU are written
 * with row stride ld_gu like G and U. */
int s24_swiglu_bwd(const void *dH, const void *G, const void *U, void *dG, void *dU,
                   int64_t p, int64_t f, int64_t ld_gu, s24_dtype dt, void *stream);

/* Gated activation on the output of the concatenated GEMM (Sec. 5.2 step 3): Z is [p][2f] = [Z_1 | Z_2] with
 * leading dimension ldz in layout lz, H is [p][f] with ldh in layout lh;  H = act(Z_1) .* Z_2.  The four layout
 * pairs are all served: equal layouts by a streaming kernel, different ones through 64 x 64 LDS tiles, so
 * that a column-major Z (what the paper's Table 4 measures) can feed a row-major consumer without a
 * separate transpose.  f and both leading dimensions multiples of 8 elements; p a multiple of 8 unless both
 * layouts are row-major; Z and H 16-byte aligned. */
int s24_glu_fwd(const void *Z, s24_layout lz, int64_t ldz, void *H, s24_layout lh, int64_t ldh, int64_t p, int64_t f,
                s24_gate gate, s24_dtype dt, void *stream);

/* Backward of s24_glu_fwd: dZ (layout and leading dimension of Z) = [dH .* Z_2 .* act'(Z_1) | dH .* act(Z_1)];
 * gelu'(z) = Phi(z) + z phi(z), silu'(z) = s(z)(1 + z(1 - s(z))).  dH is [p][f] with ldh in layout lh. */
int s24_glu_bwd(const void *dH, s24_layout lh, int64_t ldh, const void *Z, s24_layout lz, int64_t ldz, void *dZ,
                int64_t p, int64_t f, s24_gate gate, s24_dtype dt, void *stream);

/* Gradient of the bias of Sec. 5.2 step 2:  db[c] = beta*db[c] + sum over the p tokens of dZ[t][c], c < n.
 * dZ is [p][n] with leading dimension ld in the given layout; db is fp32 on the device; beta is 0 or 1.  The sum
 * runs in fp32 in a fixed order (no atomics): the result is reproducible.  n, ld multiples of 8; p a multiple of
 * 8 for a column-major dZ. */
int s24_bias_grad(const void *dZ, s24_layout layout, int64_t ld, int64_t p, int64_t n, float *db, float beta,
                  s24_dtype dt, void *stream);

/* Ungated activations of the smaller workloads: H = act(Z), n elements.
 * GELU is the erf form.  n multiple of 8. */
int s24_act_fwd(const void *Z, void *H, int64_t n, s24_act act, s24_dtype dt, void *stream);

/* dZ = dH .* act'(Z); relu'(0) = 0; gelu'(z) = Phi(z) + z phi(z). */
int s24_act_bwd(const void *dH, const void *Z, void *dZ, int64_t n, s24_act act, s24_dtype dt,
                void *stream);

/* Flip count (Sec. 4.1, definition of the flip rate): *flips = || m_new - m_old ||_1 over all mask cells,
 * i.e. the number of cells whose mask bit differs; the flip rate r_t is *flips / (16 * nblocks).
 *   mask_new, mask_old  [nblocks] device, 16-byte aligned
 *   block_flips         [nblocks] device uint32, may be NULL: every block's own count is ADDED to its entry
 *                       (the cumulative per-block flip number of Sec. 4.2)
 *   flips               device uint64, overwritten */
int s24_mask_flips(const uint16_t *mask_new, const uint16_t *mask_old, int64_t nblocks, uint32_t *block_flips,
                   uint64_t *flips, void *stream);

/* L1-norm gap (Sec. 4.2): gap[r/4][q/4] (device, fp64) = for every 4x4 block of W the kept L1 norm of the
 * best legal pattern minus that of the second best one (zero when two patterns tie for the best).  W as in
 * s24_transposable_mask.  The 90 sums are taken in fp64: exact, and the gap correctly rounded, whenever the
 * block's exponent spread fits fp64 (29 binades for bf16 data, 13 for fp32, always for binary16); beyond that the sums carry
 * fp64 rounding. */
int s24_l1_norm_gap(const void *W, s24_dtype dt, int64_t r, int64_t q, int64_t ldw, double *gap, void *stream);

/* Instrumentation, not part of the method: registers a DEVICE buffer of two uint64 (8-byte aligned), or
 * NULL to switch the probe off (the default).  While a buffer is registered, workgroup 0 of every
 * large-tile 16-bit GEMM launched by s24_spmm_fwd / s24_spmm_bwd_dx / s24_dense_dw / s24_dense_gemm
 * overwrites it with {core-clock cycles, ticks of the fixed 100 MHz reference} between its first and its
 * last instruction: cycles / ticks * 100 MHz is the core clock the chip held under that kernel.  The
 * setting is process-wide and not synchronised with launches in flight; the caller keeps the buffer alive
 * until it has unregistered it and the stream has drained. */
int s24_set_clock_probe(void *two_counters);

/* Instrumentation, not part of the method: the measured ceilings a roofline of this library is read against.
 * s24_probe_matrix_rate launches `workgroups` workgroups of 8 waves, each wave issuing 4 * iters matrix-core
 * instructions on registers only (no LDS, no memory): v_mfma_f32_32x32x16_bf16 (sparse == 0, 32768 FLOP each) or
 * v_smfmac_f32_32x32x32_bf16 (sparse != 0, 65536 dense-equivalent FLOP each).  sink [workgroups * 512] floats,
 * device, receives one checksum per lane.  s24_probe_copy copies `bytes` (a multiple of 16; src and dst 16-byte
 * aligned, not overlapping) device to device in 16-byte accesses.  The caller times the launches. */
int s24_probe_matrix_rate(int sparse, int workgroups, int iters, float *sink, void *stream);
int s24_probe_copy(const void *src, void *dst, int64_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* S24_H */
