"""Pins of the CPU oracle against facts that do not come from the oracle:
the paper's pattern count, exhaustive enumeration and exact rational
arithmetic written here in Python, numpy/torch library routines, closed forms
and finite differences.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import s24_inputs as si

HERE = os.path.dirname(os.path.abspath(__file__))


def skey(enc):
    return "".join("1" if (enc >> t) & 1 else "0" for t in range(16))


def expand_mask(mask):
    """uint16 block masks [r/4,q/4] -> 0/1 array [r,q] (bit 4i+j = m_ij)."""
    br, bq = mask.shape
    out = np.zeros((br * 4, bq * 4), dtype=np.uint8)
    for i in range(4):
        for j in range(4):
            out[i::4, j::4] = (mask >> (4 * i + j)) & 1
    return out


def f64(a):
    return si.to_f32(a).astype(np.float64)


# ---------------------------------------------------------------- patterns
def test_pattern_count_is_90_as_in_paper():
    # Sec. 5.1 step 1: "mask diversity n_t = 90"
    assert len(oracle.pattern_table()) == 90


def test_pattern_table_equals_independent_enumeration(legal_blocks):
    tab = [int(v) for v in oracle.pattern_table()]
    assert tab == legal_blocks
    assert [skey(v) for v in tab] == sorted(skey(v) for v in tab)


def test_pattern_table_invariants():
    tab = [int(v) for v in oracle.pattern_table()]
    assert len(set(tab)) == 90
    for t in range(16):                      # every cell is set in exactly half of the patterns
        assert sum((v >> t) & 1 for v in tab) == 45
    assert sum(tab) == 45 * 65535

    def transpose(v):
        return sum((((v >> (4 * i + j)) & 1) << (4 * j + i)) for i in range(4) for j in range(4))

    assert {transpose(v) for v in tab} == set(tab)          # closed under transpose
    assert sum(transpose(v) == v for v in tab) == 18
    assert {(~v) & 0xFFFF for v in tab} == set(tab)         # and under complement
    firsts = [v & 0xF for v in tab]
    assert all(firsts.count(x) == 15 for x in set(firsts)) and len(set(firsts)) == 6
    # first and last in string order
    assert tab[0] == 0x33CC and tab[89] == 0xCC33


def test_pattern_golden_file_matches():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "pattern_table.txt")) if not l.startswith("#")]
    tab = oracle.pattern_table()
    assert [int(b, 16) for _, b in rows] == [int(v) for v in tab]


# ---------------------------------------------------------------- mask search
def brute_force_block(vals16, legal_blocks):
    """Exact optimum of one block with rational arithmetic, first in string order."""
    mags = [abs(Fraction(float(v))) for v in vals16]
    best, best_s = None, None
    for enc in legal_blocks:   # already in string order
        s = sum(mags[t] for t in range(16) if (enc >> t) & 1)
        if best_s is None or s > best_s:
            best, best_s = enc, s
    return best


def check_against_brute_force(W, legal_blocks, **kw):
    mask, index = oracle.transposable_mask(W, want_index=True, **kw)
    Wf = si.to_f32(W)
    r, q = Wf.shape
    for bi in range(r // 4):
        for bj in range(q // 4):
            blk = Wf[4 * bi:4 * bi + 4, 4 * bj:4 * bj + 4].reshape(-1)
            want = brute_force_block(blk, legal_blocks)
            assert int(mask[bi, bj]) == want, (bi, bj, blk)
            assert legal_blocks[int(index[bi, bj])] == want


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_mask_matches_exact_brute_force_random(dtype, legal_blocks):
    W = si.random_matrix(11, (32, 48), 0.02, dtype)
    check_against_brute_force(W, legal_blocks)
    check_against_brute_force(W, legal_blocks, exact_wide=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("kind", ["few", "equal", "zeros", "tiny", "range", "subnormal", "window"])
def test_mask_matches_exact_brute_force_ties(dtype, kind, legal_blocks):
    W = si.tie_matrix(5, 16, 32, dtype, kind)
    check_against_brute_force(W, legal_blocks)
    check_against_brute_force(W, legal_blocks, exact_wide=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_mask_fast_and_wide_paths_agree(dtype):
    for kind in ["few", "equal", "zeros", "tiny", "range", "subnormal", "window"]:
        W = si.tie_matrix(9, 64, 128, dtype, kind)
        a = oracle.transposable_mask(W)
        b = oracle.transposable_mask(W, exact_wide=True)
        assert np.array_equal(a, b), kind
    W = si.random_matrix(3, (128, 256), 0.02, dtype)
    assert np.array_equal(oracle.transposable_mask(W), oracle.transposable_mask(W, exact_wide=True))


@pytest.mark.parametrize("dtype,big_exp", [("f32", 27), ("f32", 30), ("f32", 45), ("f32", 100),
                                           ("bf16", 43), ("bf16", 47), ("bf16", 60), ("bf16", 100)])
def test_mask_margin_below_fp64_resolution(dtype, big_exp, legal_blocks):
    """Blocks in which the best pattern beats an earlier one by one unit in the last place of 1 while both hold six
    cells of 2^big_exp: sums of eight fp64 terms stop seeing the margin a few binades past the width the oracle's
    exactness check allows (53 bits), so a check that let such blocks take the fp64 route would return the earlier
    pattern.  Expected values: by construction, and by rational arithmetic."""
    from util import absorbed_margin_blocks
    W, want = absorbed_margin_blocks(legal_blocks, dtype, big_exp)
    assert len(want) >= 80
    for kw in ({}, {"exact_wide": True}):
        got = oracle.transposable_mask(W, **kw)
        assert [int(v) for v in got[0]] == want, kw
    check_against_brute_force(W[:, :64], legal_blocks)


def test_mask_every_block_is_legal():
    W = si.random_matrix(4, (256, 512), 0.02, "bf16")
    m = expand_mask(oracle.transposable_mask(W))
    assert (m.reshape(256, 128, 4).sum(-1) == 2).all()                # 2 per row group
    assert (m.reshape(64, 4, 512).sum(1) == 2).all()                   # 2 per column group
    assert m.sum() == m.size // 2


def test_mask_all_equal_block_picks_first_pattern():
    W = np.full((4, 4), 0.375, dtype=np.float32)
    assert int(oracle.transposable_mask(W)[0, 0]) == 0x33CC
    W[1, 2] = -0.375
    assert int(oracle.transposable_mask(W)[0, 0]) == 0x33CC


def test_mask_planted_pattern_is_recovered(legal_blocks):
    rng = np.random.default_rng(0)
    W = np.zeros((4, 4 * 90), dtype=np.float32)
    for k, enc in enumerate(legal_blocks):
        for t in range(16):
            big = (enc >> t) & 1
            W[t // 4, 4 * k + t % 4] = (1.0 if big else 0.01) * (1 + 0.1 * rng.random()) * rng.choice([-1, 1])
    mask, index = oracle.transposable_mask(W, want_index=True)
    assert [int(v) for v in mask[0]] == legal_blocks
    assert [int(v) for v in index[0]] == list(range(90))


def test_mask_invariant_to_sign_and_power_of_two_scale():
    W = si.to_f32(si.random_matrix(6, (64, 64), 0.02, "bf16"))
    base = oracle.transposable_mask(W)
    rng = np.random.default_rng(1)
    flips = rng.choice([-1.0, 1.0], size=W.shape).astype(np.float32)
    assert np.array_equal(oracle.transposable_mask(W * flips), base)
    assert np.array_equal(oracle.transposable_mask(W * np.float32(2.0 ** -9)), base)
    assert np.array_equal(oracle.transposable_mask(W * np.float32(2.0 ** 20)), base)


def test_mask_transpose_retains_same_magnitude():
    W = si.to_f32(si.random_matrix(8, (64, 96), 0.02, "bf16"))
    m = expand_mask(oracle.transposable_mask(W))
    mt = expand_mask(oracle.transposable_mask(np.ascontiguousarray(W.T)))
    a = np.abs(W).astype(np.float64)
    kept = (a * m).reshape(16, 4, 24, 4).sum(axis=(1, 3))
    kept_t = (a.T * mt).reshape(24, 4, 16, 4).sum(axis=(1, 3))
    assert np.array_equal(kept, kept_t.T)       # sums of bf16 magnitudes are exact in fp64


def test_mask_retained_l1_bounded_by_one_sided_optima():
    W = si.to_f32(si.random_matrix(10, (64, 64), 0.02, "bf16"))
    a = np.abs(W).astype(np.float64)
    m = expand_mask(oracle.transposable_mask(W))
    kept = (a * m).reshape(16, 4, 16, 4).sum(axis=(1, 3))
    row_opt = np.sort(a.reshape(64, 16, 4), axis=-1)[..., 2:].sum(-1).reshape(16, 4, 16).sum(1)
    col_opt = np.sort(a.reshape(16, 4, 64), axis=1)[:, 2:, :].sum(1).reshape(16, 16, 4).sum(-1)
    assert (kept <= row_opt).all() and (kept <= col_opt).all()
    assert (kept < row_opt).any()      # the transposable constraint does bind somewhere


def test_mask_bad_shape_is_rejected():
    with pytest.raises(ValueError):
        oracle.transposable_mask(np.zeros((6, 8), dtype=np.float32))


# ---------------------------------------------------------------- compress
def decode(vals, meta, width):
    """Python decoder of the compressed form (written here, not in the oracle)."""
    rows = vals.shape[0]
    out = np.zeros((rows, width), dtype=vals.dtype)
    for o in range(rows):
        for g in range(width // 4):
            nib = (int(meta[o, g // 4]) >> (4 * (g % 4))) & 0xF
            i0, i1 = nib & 3, nib >> 2
            assert i0 < i1
            out[o, 4 * g + i0] = vals[o, 2 * g]
            out[o, 4 * g + i1] = vals[o, 2 * g + 1]
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_compress_decodes_to_masked_weight_bitwise(dtype):
    W = si.random_matrix(12, (32, 64), 0.02, dtype)
    W[3, 5] = 0          # a kept or pruned exact zero must not disturb the indices
    W[0:4, 0:4] = 0
    mask = oracle.transposable_mask(W)
    m = expand_mask(mask).astype(bool)
    vals, meta, valsT, metaT = oracle.compress(W, mask)
    masked = np.where(m, W, np.zeros_like(W))
    assert np.array_equal(decode(vals, meta, 64), masked)
    assert np.array_equal(decode(valsT, metaT, 32), masked.T)
    legal = {0b0100, 0b1000, 0b1100, 0b1001, 0b1101, 0b1110}
    for mm in (meta, metaT):
        nibs = {(int(w) >> s) & 0xF for w in mm.reshape(-1) for s in (0, 4, 8, 12)}
        assert nibs <= legal


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_pack_is_the_documented_permutation(dtype):
    W = si.random_matrix(13, (80, 192), 0.02, dtype)
    mask = oracle.transposable_mask(W)
    vals, meta, valsT, metaT = oracle.compress(W, mask)
    vp, mp = oracle.pack(vals, meta)
    assert np.array_equal(vp, vals.reshape(80, 3, 32).transpose(1, 0, 2))
    assert np.array_equal(mp, meta.reshape(80, 3, 4).transpose(1, 0, 2))
    with pytest.raises(ValueError):
        oracle.pack(valsT, metaT)          # contraction length 80 is not a multiple of 64


def test_compress_rejects_illegal_mask():
    W = si.random_matrix(1, (16, 16), 0.02, "f32")
    mask = oracle.transposable_mask(W)
    mask[0, 0] = 0x000F
    with pytest.raises(ValueError):
        oracle.compress(W, mask)


# ---------------------------------------------------------------- GEMMs
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_sparse_gemms_equal_dense_gemm_on_masked_weight(dtype):
    p, q, r = 24, 64, 48
    W = si.random_matrix(20, (r, q), 0.02, dtype)
    X = si.random_matrix(21, (p, q), 1.0, dtype)
    dY = si.random_matrix(22, (p, r), 1.0, dtype)
    mask = oracle.transposable_mask(W)
    vals, meta, valsT, metaT = oracle.compress(W, mask)
    Wm = f64(W) * expand_mask(mask)
    Y = oracle.spmm_fwd(X, vals, meta)
    np.testing.assert_allclose(Y, f64(X) @ Wm.T, rtol=1e-12, atol=1e-13)
    dX = oracle.spmm_bwd_dx(dY, valsT, metaT)
    np.testing.assert_allclose(dX, f64(dY) @ Wm, rtol=1e-12, atol=1e-13)
    dX0 = np.random.default_rng(0).standard_normal((p, q))
    dXb = oracle.spmm_bwd_dx(dY, valsT, metaT, beta=1.0, dX0=dX0)
    np.testing.assert_allclose(dXb, dX0 + f64(dY) @ Wm, rtol=1e-12, atol=1e-13)
    rows = np.array([5, 0, 23], dtype=np.int64)
    assert np.array_equal(oracle.spmm_fwd(X, vals, meta, rows=rows), Y[rows])
    assert np.array_equal(oracle.spmm_bwd_dx(dY, valsT, metaT, rows=rows), dX[rows])
    # torch as a second library
    Yt = torch.from_numpy(f64(X)) @ torch.from_numpy(Wm).T
    np.testing.assert_allclose(Y, Yt.numpy(), rtol=1e-12, atol=1e-13)


def test_sparse_gemm_one_hot_rows_reproduce_masked_weight():
    q, r = 32, 16
    W = si.random_matrix(23, (r, q), 0.02, "bf16")
    mask = oracle.transposable_mask(W)
    vals, meta, valsT, metaT = oracle.compress(W, mask)
    Wm = f64(W) * expand_mask(mask)
    eye_q = si.f32_to_bf16_bits(torch.eye(q))
    eye_r = si.f32_to_bf16_bits(torch.eye(r))
    assert np.array_equal(oracle.spmm_fwd(eye_q, vals, meta), Wm.T)      # Y = I (MW)^T
    assert np.array_equal(oracle.spmm_bwd_dx(eye_r, valsT, metaT), Wm)   # dX = I (MW)
    # not symmetric, so a transposed operand would show
    assert not np.array_equal(Wm[:, :16], Wm[:, :16].T)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_dense_gemms_match_library(dtype):
    p, q, r = 40, 24, 16
    X = si.random_matrix(30, (p, q), 1.0, dtype)
    dY = si.random_matrix(31, (p, r), 1.0, dtype)
    W = si.random_matrix(32, (r, q), 0.02, dtype)
    dW = oracle.dense_dw(dY, X)
    np.testing.assert_allclose(dW, f64(dY).T @ f64(X), rtol=1e-12, atol=1e-13)
    dW0 = np.random.default_rng(2).standard_normal((r, q))
    np.testing.assert_allclose(oracle.dense_dw(dY, X, beta=1.0, dW0=dW0), dW0 + f64(dY).T @ f64(X), rtol=1e-12)
    rows = np.array([3, 15], dtype=np.int64)
    assert np.array_equal(oracle.dense_dw(dY, X, rows=rows), dW[rows])
    np.testing.assert_allclose(oracle.dense_gemm(X, W), f64(X) @ f64(W).T, rtol=1e-12, atol=1e-13)
    # rank one: p = 1 is exactly the outer product
    assert np.array_equal(oracle.dense_dw(dY[:1], X[:1]), np.outer(f64(dY)[0], f64(X)[0]))


# ---------------------------------------------------------------- masked decay (Eq. 10)
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_masked_decay_touches_only_pruned_cells(dtype):
    r, q, lam = 32, 48, np.float32(2e-4)
    W = si.random_matrix(40, (r, q), 0.02, dtype)
    dW = si.random_matrix(41, (r, q), 1e-3, "f32")
    mask = oracle.transposable_mask(W)
    m = expand_mask(mask).astype(bool)
    G = oracle.masked_decay(dW, W, mask, lam)
    assert np.array_equal(G[m], dW.astype(np.float64)[m])                      # kept: untouched
    want = dW.astype(np.float64) + np.float64(lam) * f64(W)
    np.testing.assert_allclose(G[~m], want[~m], rtol=1e-15)                    # pruned: + lambda w
    assert (~m).sum() == m.size // 2
    assert np.array_equal(oracle.masked_decay(dW, W, mask, 0.0), dW.astype(np.float64))
    # sign: the term pulls pruned weights towards zero under gradient descent
    big = np.abs(f64(W)) > 1e-3
    sel = ~m & big
    assert (np.sign(G - dW)[sel] == np.sign(f64(W))[sel]).all()


# ---------------------------------------------------------------- activations
def test_swiglu_matches_library_and_special_values():
    g = si.random_matrix(50, (8, 32), 2.0, "bf16")
    u = si.random_matrix(51, (8, 32), 1.0, "bf16")
    H = oracle.swiglu_fwd(g, u)
    tg, tu = torch.from_numpy(f64(g)), torch.from_numpy(f64(u))
    np.testing.assert_allclose(H, (torch.nn.functional.silu(tg) * tu).numpy(), rtol=1e-13, atol=1e-300)
    z = si.f32_to_bf16_bits(torch.tensor([[0.0, 88.0, -88.0, 300.0, -300.0, -0.0, 1.0, -1.0]]))
    one = si.f32_to_bf16_bits(torch.ones(1, 8))
    h = oracle.swiglu_fwd(z, one)[0]
    assert h[0] == 0 and h[5] == 0 and np.isfinite(h).all()
    assert h[1] == 88.0 and h[3] == 300.0 and abs(h[2]) < 1e-30 and abs(h[4]) < 1e-100
    np.testing.assert_allclose(h[6], 1 / (1 + np.exp(-1.0)), rtol=1e-15)
    # gate is the FIRST operand: swapping operands changes the result
    assert not np.allclose(oracle.swiglu_fwd(u, g), H)


def test_swiglu_bwd_matches_autograd_and_finite_differences():
    g = si.random_matrix(52, (4, 16), 2.0, "bf16")
    u = si.random_matrix(53, (4, 16), 1.0, "bf16")
    d = si.random_matrix(54, (4, 16), 1.0, "bf16")
    dG, dU = oracle.swiglu_bwd(d, g, u)
    tg = torch.from_numpy(f64(g)).requires_grad_()
    tu = torch.from_numpy(f64(u)).requires_grad_()
    (torch.nn.functional.silu(tg) * tu).backward(torch.from_numpy(f64(d)))
    np.testing.assert_allclose(dG, tg.grad.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dU, tu.grad.numpy(), rtol=1e-12, atol=1e-15)
    # central differences on the closed form, in fp64
    G, U, D = f64(g), f64(u), f64(d)
    silu = lambda x: x / (1 + np.exp(-x))
    eps = 1e-6
    np.testing.assert_allclose(dG, D * U * (silu(G + eps) - silu(G - eps)) / (2 * eps), rtol=1e-6, atol=1e-8)
    H = oracle.swiglu_fwd(g, u)
    nz = U != 0
    np.testing.assert_allclose(dU[nz] / D[nz], (H / np.where(nz, U, 1))[nz], rtol=1e-12)
    # silu'(0) = 1/2
    z = np.zeros((1, 16), dtype=np.uint16)
    one = si.f32_to_bf16_bits(torch.ones(1, 16))
    dg0, du0 = oracle.swiglu_bwd(one, z, one)
    assert (dg0 == 0.5).all() and (du0 == 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_relu_and_gelu_match_library(dtype):
    z = si.random_matrix(60, (6, 40), 1.5, dtype)
    d = si.random_matrix(61, (6, 40), 1.0, dtype)
    z.reshape(-1)[:3] = 0
    tz = torch.from_numpy(f64(z))
    np.testing.assert_array_equal(oracle.act_fwd(z, oracle.ACT_RELU), torch.relu(tz).numpy())
    np.testing.assert_allclose(oracle.act_fwd(z, oracle.ACT_GELU_ERF),
                               torch.nn.functional.gelu(tz, approximate="none").numpy(), rtol=1e-13, atol=1e-300)
    dz = oracle.act_bwd(d, z, oracle.ACT_RELU)
    np.testing.assert_array_equal(dz, f64(d) * (f64(z) > 0))          # relu'(0) = 0
    tz2 = tz.clone().requires_grad_()
    torch.nn.functional.gelu(tz2, approximate="none").backward(torch.from_numpy(f64(d)))
    np.testing.assert_allclose(oracle.act_bwd(d, z, oracle.ACT_GELU_ERF), tz2.grad.numpy(), rtol=1e-12, atol=1e-15)
    # GELU(0) = 0, GELU'(0) = 1/2
    zero = np.zeros((1, 4), dtype=z.dtype)
    one = si.f32_to_bf16_bits(torch.ones(1, 4)) if dtype == "bf16" else np.ones((1, 4), dtype=z.dtype)
    assert (oracle.act_fwd(zero, oracle.ACT_GELU_ERF) == 0).all()
    assert (oracle.act_bwd(one, zero, oracle.ACT_GELU_ERF) == 0.5).all()


def test_round_bf16_matches_torch():
    x = np.random.default_rng(7).standard_normal(4096) * np.exp(np.random.default_rng(8).uniform(-30, 30, 4096))
    x[:4] = [0.0, -0.0, 1.00390625, 1.01171875]   # exact ties: round to even
    want = torch.from_numpy(x).float().to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.round_bf16(x), want)


# ---------------------------------------------------------------- monitors: flip count, L1-norm gap
def test_flip_count_hand_examples():
    # Sec. 4.1, definition of the flip rate: the L1 distance of the two 0/1 mask vectors
    a = np.array([[0x33CC, 0xCC33], [0x5A5A, 0x33CC]], dtype=np.uint16)
    assert oracle.mask_flips(a, a) == 0
    b = a.copy()
    b[0, 0] = 0xCC33                      # the complementary pattern: all 16 cells change
    assert oracle.mask_flips(b, a) == 16
    b[1, 0] = 0x5A5A ^ 0x0003             # two more cells
    per_block = np.zeros(4, dtype=np.uint32)
    assert oracle.mask_flips(b, a, per_block) == 18
    assert per_block.tolist() == [16, 0, 2, 0]
    assert oracle.mask_flips(b, a, per_block) == 18          # the per-block counter accumulates
    assert per_block.tolist() == [32, 0, 4, 0]
    assert oracle.mask_flips(a, b) == oracle.mask_flips(b, a)


def test_flip_count_equals_numpy_on_expanded_masks():
    w0 = si.random_matrix(31, (64, 96), 0.02, "bf16")
    w1 = si.random_matrix(32, (64, 96), 0.02, "bf16")
    m0, m1 = oracle.transposable_mask(w0), oracle.transposable_mask(w1)
    want = int(np.abs(expand_mask(m0).astype(np.int64) - expand_mask(m1).astype(np.int64)).sum())
    assert oracle.mask_flips(m1, m0) == want
    assert 0 < want <= 64 * 96


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
def test_l1_gap_equals_exact_rational_enumeration(legal_blocks, dtype):
    # Sec. 4.2: g = ||m1 . w||_1 - ||m2 . w||_1 with m1, m2 the masks of largest and second largest kept norm
    W = si.random_matrix(41, (16, 24), 0.02, dtype)
    a = np.abs(f64(W))
    got = oracle.l1_norm_gap(W)
    for bi in range(4):
        for bj in range(6):
            blk = [Fraction(float(a[4 * bi + i, 4 * bj + j])) for i in range(4) for j in range(4)]
            sums = sorted((sum(blk[t] for t in range(16) if (p >> t) & 1) for p in legal_blocks), reverse=True)
            assert Fraction(float(got[bi, bj])) == sums[0] - sums[1]      # exact: the difference fits fp64


def test_l1_gap_special_cases():
    ones = np.ones((4, 4), dtype=np.float32)
    assert oracle.l1_norm_gap(ones)[0, 0] == 0.0                          # every pattern keeps 8
    w = ones.copy()
    w[0, 0] = 3.0                                                         # many patterns keep cell (0,0): still tied
    assert oracle.l1_norm_gap(w)[0, 0] == 0.0
    # a block whose best pattern is unique: heavy cells on 0x33CC, then one kept cell lowered by 0.25 --
    # the runner-up swaps one 2x2 sub-pattern, so the gap is the cost of that swap
    pat = 0x33CC
    w = np.full(16, 1.0, dtype=np.float32)
    for t in range(16):
        if (pat >> t) & 1:
            w[t] = 8.0
    g0 = oracle.l1_norm_gap(w.reshape(4, 4))[0, 0]
    assert g0 == 2 * (8.0 - 1.0)                                          # any other legal pattern drops >= 2 heavy cells
    # scaling by a power of two scales the gap exactly; the gap is never negative
    W = si.random_matrix(43, (32, 32), 0.02, "f32")
    g = oracle.l1_norm_gap(W)
    assert (g >= 0).all()
    assert np.array_equal(oracle.l1_norm_gap((W * 4.0).astype(np.float32)), 4.0 * g)


def test_l1_gap_is_consistent_with_the_mask_search():
    # best kept norm = norm kept by the oracle's own mask; with a strictly positive gap that mask is the unique optimum
    W = si.random_matrix(44, (32, 48), 0.02, "bf16")
    a = np.abs(f64(W))
    keep = expand_mask(oracle.transposable_mask(W)).astype(bool)
    g = oracle.l1_norm_gap(W)
    tab = [int(v) for v in oracle.pattern_table()]
    for bi in range(8):
        for bj in range(12):
            blk = a[4 * bi:4 * bi + 4, 4 * bj:4 * bj + 4]
            best = blk[keep[4 * bi:4 * bi + 4, 4 * bj:4 * bj + 4]].sum()
            others = sorted(sum(blk[t // 4, t % 4] for t in range(16) if (p >> t) & 1) for p in tab)
            assert abs(others[-1] - best) <= 1e-12 * best
            assert abs((others[-1] - others[-2]) - g[bi, bj]) <= 1e-12 * best


# ---------------------------------------------------------------- unbiased 2:4 pruning of the output gradient
def mvue_dense(dY, seed):
    """Oracle's compressed S_z(dY^T) decoded to a dense [r, p] float64 matrix, plus the kept-position flags."""
    vals, meta = oracle.mvue24(dY, seed)
    p, r = dY.shape
    v = f64(vals).reshape(r, p // 4, 2)
    nib = ((meta.astype(np.int64)[:, :, None] >> (4 * np.arange(4))) & 0xF).reshape(r, p // 4)
    i0, i1 = nib & 3, nib >> 2
    assert (i0 < i1).all()                                       # two distinct kept positions, ascending
    out = np.zeros((r, p // 4, 4))
    kept = np.zeros((r, p // 4, 4), dtype=bool)
    rr, gg = np.meshgrid(np.arange(r), np.arange(p // 4), indexing="ij")
    out[rr, gg, i0] = v[:, :, 0]
    out[rr, gg, i1] = v[:, :, 1]
    kept[rr, gg, i0] = True
    kept[rr, gg, i1] = True
    return out.reshape(r, p), kept.reshape(r, p)


def test_mvue_deterministic_groups():
    # Eq. 6 read as: keep two of four, unbiased, least variance.  Groups where nothing is left to chance:
    col = np.array([3.0, -5.0, 0.0, 0.0,      # two non-zeros: both kept as they are
                    0.0, 0.0, 0.0, 7.0,       # one non-zero: kept as it is (plus a zero)
                    0.0, 0.0, 0.0, 0.0,       # nothing
                    -1.5, 0.0, 2.5, 0.0], dtype=np.float32).reshape(16, 1)
    for seed in range(5):
        out, kept = mvue_dense(col, seed)
        assert np.array_equal(out[0], col[:, 0].astype(np.float64))
        assert kept.reshape(4, 4).sum(axis=1).tolist() == [2, 2, 2, 2]
    # equal magnitudes: every element kept with probability 1/2 and doubled
    col = np.array([2.0, -2.0, 2.0, 2.0] * 4, dtype=np.float32).reshape(16, 1)
    out, kept = mvue_dense(col, 3)
    assert np.array_equal(out[0][kept[0]], 2.0 * col[:, 0][kept[0]])
    assert np.all(out[0][~kept[0]] == 0)


def test_mvue_single_nonzero_survives_at_every_position():
    # a group with one non-zero element has nothing to draw: the element is kept as it is, wherever it stands
    for pos in range(4):
        for x in (7.0, -0.375):
            col = np.zeros((16, 3), dtype=np.float32)
            col[pos::4, :] = x
            for seed in range(8):
                out, kept = mvue_dense(col, seed)
                assert np.array_equal(out, col.T.astype(np.float64)), (pos, x, seed)
                assert kept.reshape(3, 4, 4).sum(axis=2).tolist() == [[2] * 4] * 3


def test_mvue_draws_differ_across_features_groups_and_seeds():
    """The same four numbers in every group of every feature: whatever differs between two outputs is the draw.
    Kept frequencies taken over features alone (one token group), over token groups alone (one feature) and over
    seeds alone (one group of one feature) must each approach the inclusion probabilities 2 |a_j| / S."""
    a = np.array([1.0, -2.0, 3.0, 4.0], dtype=np.float32)
    pi = 2 * np.abs(a) / np.abs(a).sum()
    tol = lambda n: 5 * np.sqrt(pi * (1 - pi) / n) + 1e-9
    r = 4096
    _, kept = mvue_dense(np.tile(a.reshape(4, 1), (4, r)), 21)                  # 4 groups x 4096 features
    for g in range(4):
        freq = kept[:, 4 * g:4 * g + 4].mean(axis=0)
        assert np.all(np.abs(freq - pi) <= tol(r)), ("over features", g, freq)
    assert not np.array_equal(kept[:, 0:4], kept[:, 4:8])                       # and group 1 is not a copy of group 0
    G = 4096
    _, kept = mvue_dense(np.tile(a, G).reshape(4 * G, 1), 22)                   # 4096 groups of one feature
    assert np.all(np.abs(kept[0].reshape(G, 4).mean(axis=0) - pi) <= tol(G))
    n = 1024
    seen = np.stack([mvue_dense(np.tile(a, 4).reshape(16, 1), seed)[1][0, :4] for seed in range(n)])
    assert np.all(np.abs(seen.mean(axis=0) - pi) <= tol(n)), ("over seeds", seen.mean(axis=0))


def test_mvue_neighbouring_seeds_share_no_draws_in_any_arrangement():
    """A layer takes one seed per pruned operand and step, i.e. consecutive integers.  The streams of two
    neighbouring seeds must be unrelated: not equal, and not the same draws dealt out to other token groups of the
    same feature (what a seed that is merely XORed or added into the group counter would give).  The same four
    numbers sit in every group, so the kept pair of a group is a function of its draw alone."""
    a = np.array([1.0, -2.0, 3.0, 4.0], dtype=np.float32)
    r, G = 256, 64
    dY = np.tile(a.reshape(4, 1), (G, r))
    hist = lambda kept: np.stack([np.bincount((kept.reshape(r, G, 4)[f] * (1 << np.arange(4))).sum(axis=1), minlength=16)
                                  for f in range(r)])
    for seed in (0, 6, 1000, 2 ** 31 - 2):
        k0, k1 = mvue_dense(dY, seed)[1], mvue_dense(dY, seed + 1)[1]
        same_groups = (k0.reshape(r, G, 4) == k1.reshape(r, G, 4)).all(axis=2).mean()
        # two independent draws keep the same pair with probability sum of squared pair probabilities, about 0.3
        assert same_groups < 0.45, (seed, same_groups)
        # per feature, the multiset of kept pairs over the 64 groups: equal for nearly no feature if the streams are
        # unrelated, equal for every feature if one stream is a rearrangement of the other
        same_multiset = (hist(k0) == hist(k1)).all(axis=1).mean()
        assert same_multiset < 0.05, (seed, same_multiset)
        # and the neighbour is not the same stream shifted by a few groups either
        for shift in (1, 2, 3, 4):
            moved = np.roll(k1.reshape(r, G, 4), shift, axis=1)
            assert (k0.reshape(r, G, 4) == moved).all(axis=2).mean() < 0.45, (seed, shift)


def test_mvue_reads_a_strided_operand():
    wide = si.random_matrix(54, (64, 40), 1e-2, "bf16")
    view = wide[:, 8:32]                                                         # row stride 40, 24 features
    a = oracle.mvue24(view, 9)
    b = oracle.mvue24(np.ascontiguousarray(view), 9)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("group", [(1.0, 2.0, 3.0, 4.0), (0.3, -0.2, 0.25, -0.1), (5.0, 1.0, -1.5, 0.5), (9.0, 0.0, 2.0, -1.0)])
def test_mvue_is_unbiased_with_the_least_second_moment(group):
    """65536 independent draws of one group (the same four numbers in every token group of one feature).
    Independent of the oracle's formulas: the sample mean must be the group itself, and the summed second
    moment must equal the minimum of sum_j a_j^2 / pi_j over sum pi = 2, pi <= 1, which Lagrange gives in closed
    form: S^2 / 2 without a cap, a_max^2 + R^2 with the largest element capped at probability one."""
    G = 65536
    a = np.array(group, dtype=np.float32)
    dY = np.tile(a, G).reshape(4 * G, 1)
    out, kept = mvue_dense(dY, 7)
    samples = out[0].reshape(G, 4)
    m = np.abs(a.astype(np.float64))
    S, mx = m.sum(), m.max()
    if 2 * mx <= S:
        pi = 2 * m / S
        second = S * S / 2
    else:
        R = S - mx
        pi = np.where(m == mx, 1.0, m / R)
        second = mx * mx + R * R
    var = np.where(pi > 0, m * m * (1 / np.maximum(pi, 1e-300) - 1), 0.0)
    assert np.all(np.abs(samples.mean(axis=0) - a) <= 5 * np.sqrt(var / G) + 1e-6)
    freq = kept[0].reshape(G, 4).mean(axis=0)
    assert np.all(np.abs(freq - pi) <= 5 * np.sqrt(pi * (1 - pi) / G) + 1e-6)
    got_second = (samples ** 2).sum(axis=1).mean()
    assert abs(got_second - second) <= 0.02 * second


def test_mvue_seed_and_dtype_behaviour():
    dY = si.random_matrix(51, (256, 24), 1e-2, "bf16")
    v1, m1 = oracle.mvue24(dY, 11)
    v2, m2 = oracle.mvue24(dY, 11)
    v3, m3 = oracle.mvue24(dY, 12)
    assert np.array_equal(v1, v2) and np.array_equal(m1, m2)
    assert not np.array_equal(m1, m3)
    # bf16 storage = the fp32 result rounded to nearest even; the draws do not depend on the storage type
    vf, mf = oracle.mvue24(si.to_f32(dY), 11)
    assert np.array_equal(mf, m1)
    assert np.array_equal(oracle.round_bf16(vf.astype(np.float64)), v1)


def test_mvue_weight_gradient_is_unbiased():
    # Eq. 4: the mean over seeds of S_z(dY^T) X approaches dY^T X
    dY = si.random_matrix(52, (64, 8), 1.0, "f32")
    X = si.random_matrix(53, (64, 6), 1.0, "f32")
    exact = f64(dY).T @ f64(X)
    acc = np.zeros_like(exact)
    n = 400
    for seed in range(n):
        acc += mvue_dense(dY, seed)[0] @ f64(X)
    err = np.abs(acc / n - exact)
    assert err.max() <= 6 * np.abs(exact).max() / np.sqrt(n) + 1e-3


# ---------------------------------------------------------------- binary16 (the paper's own precision, Sec. 6)
def test_f16_inputs_are_widened_exactly():
    # every one of the 65536 bit patterns, read back through a one-row column sum, against numpy's conversion
    h = np.arange(65536, dtype=np.uint16).view(np.float16).reshape(1, -1)
    got = oracle.bias_grad(h)
    want = h[0].astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])


def test_round_f16_matches_numpy_and_torch():
    rng = np.random.default_rng(17)
    x = rng.standard_normal(20000) * np.exp(rng.uniform(-22, 12, 20000))
    x[:10] = [0.0, -0.0, 1.00048828125, 1.00146484375, 65504.0, 65519.99, 65520.0, 2.0 ** -25, 1.5 * 2.0 ** -25, -1e9]
    with np.errstate(over="ignore"):
        want = x.astype(np.float32).astype(np.float16)
    got = oracle.round_f16(x)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    wt = torch.from_numpy(x).float().to(torch.float16).numpy()
    assert np.array_equal(got.view(np.uint16), wt.view(np.uint16))
    # ties to even, overflow to infinity, half the smallest subnormal to zero
    assert got[2] == 1.0 and got[3] == np.float16(1.001953125) and got[4] == 65504 and got[5] == 65504
    assert np.isinf(got[6]) and got[7] == 0 and got[8] == np.float16(2.0 ** -24) and got[9] == -np.inf


def test_mvue_f16_rounds_kept_values_to_binary16():
    dY = si.random_matrix(70, (32, 8), 0.05, "f16")
    v16, m16 = oracle.mvue24(dY, 5)
    v32, m32 = oracle.mvue24(dY.astype(np.float32), 5)
    assert v16.dtype == np.float16 and np.array_equal(m16, m32)      # same decisions: both decide in fp32
    assert np.array_equal(v16.view(np.uint16), v32.astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------- gated activation on Z = [Z1 | Z2] (Sec. 5.2 step 3)
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("gate", ["gelu", "silu"])
def test_glu_matches_library_in_both_layouts(dtype, gate):
    p, r = 12, 24
    Z = si.random_matrix(80, (p, 2 * r), 1.5, dtype)
    D = si.random_matrix(81, (p, r), 1.0, dtype)
    g = oracle.GATE_GELU_ERF if gate == "gelu" else oracle.GATE_SILU
    fn = (lambda t: torch.nn.functional.gelu(t, approximate="none")) if gate == "gelu" else torch.nn.functional.silu
    tz = torch.from_numpy(f64(Z)).requires_grad_()
    th = fn(tz[:, :r]) * tz[:, r:]
    th.backward(torch.from_numpy(f64(D)))
    H = oracle.glu_fwd(Z, g)
    np.testing.assert_allclose(H, th.detach().numpy(), rtol=1e-13, atol=1e-300)
    dZ = oracle.glu_bwd(D, Z, g)
    np.testing.assert_allclose(dZ, tz.grad.numpy(), rtol=1e-12, atol=1e-15)
    # column-major storage of the same matrices is the row-major storage of their transposes
    Zc, Dc = np.ascontiguousarray(Z.T), np.ascontiguousarray(D.T)
    assert np.array_equal(oracle.glu_fwd(Zc, g, layout=oracle.COL_MAJOR), H)
    assert np.array_equal(oracle.glu_bwd(Dc, Zc, g, layout=oracle.COL_MAJOR, layout_h=oracle.COL_MAJOR), dZ)
    assert np.array_equal(oracle.glu_bwd(D, Zc, g, layout=oracle.COL_MAJOR), dZ)
    # the gate is the FIRST half: swapping the halves changes the result
    Zs = np.concatenate([Z[:, r:], Z[:, :r]], axis=1)
    assert not np.allclose(oracle.glu_fwd(Zs, g), H)


def test_glu_special_values_and_the_swiglu_special_case():
    # GELU(1) = Phi(1), GELU(-1) = -(1 - Phi(1)), GELU(0) = 0, GELU'(0) = 1/2; Phi(1) to 16 digits
    phi1 = 0.8413447460685429
    Z = np.array([[1.0, -1.0, 0.0, 40.0, 2.0, 3.0, 5.0, 0.5]], dtype=np.float32)
    H = oracle.glu_fwd(Z, oracle.GATE_GELU_ERF)[0]
    np.testing.assert_allclose(H[:2], [2.0 * phi1, -3.0 * (1.0 - phi1)], rtol=1e-14)
    assert H[2] == 0.0 and H[3] == 20.0
    dZ = oracle.glu_bwd(np.ones((1, 4), dtype=np.float32), Z, oracle.GATE_GELU_ERF)[0]
    assert dZ[2] == 0.5 * 5.0 and dZ[6] == 0.0 and dZ[7] == 40.0 and dZ[3] == 0.5
    np.testing.assert_allclose(dZ[4], phi1, rtol=1e-14)
    # central differences of the forward function
    Zr = si.random_matrix(82, (3, 16), 1.0, "f32")
    Dr = si.random_matrix(83, (3, 8), 1.0, "f32")
    an = oracle.glu_bwd(Dr, Zr, oracle.GATE_GELU_ERF)
    eps = 2.0 ** -10
    for c in range(16):
        Zp, Zm = Zr.copy(), Zr.copy()
        Zp[:, c] += eps
        Zm[:, c] -= eps
        fd = (oracle.glu_fwd(Zp, oracle.GATE_GELU_ERF) - oracle.glu_fwd(Zm, oracle.GATE_GELU_ERF)) / (Zp[:, c] - Zm[:, c]).astype(np.float64)[:, None]
        np.testing.assert_allclose(an[:, c], (fd * f64(Dr))[:, c % 8], rtol=1e-5, atol=1e-7)
    # with the SiLU gate it is the SwiGLU of the two halves
    Zb = si.random_matrix(84, (5, 32), 2.0, "bf16")
    Db = si.random_matrix(85, (5, 16), 1.0, "bf16")
    G, U = np.ascontiguousarray(Zb[:, :16]), np.ascontiguousarray(Zb[:, 16:])
    assert np.array_equal(oracle.glu_fwd(Zb, oracle.GATE_SILU), oracle.swiglu_fwd(G, U))
    dG, dU = oracle.swiglu_bwd(Db, G, U)
    np.testing.assert_allclose(oracle.glu_bwd(Db, Zb, oracle.GATE_SILU), np.concatenate([dG, dU], axis=1), rtol=1e-14, atol=0)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_bias_gradient_is_the_column_sum_and_bias_shifts_every_row(dtype):
    dZ = si.random_matrix(86, (37, 24), 1.0, dtype)
    want = np.array([sum(Fraction(float(v)) for v in f64(dZ)[:, c]) for c in range(24)], dtype=object)
    got = oracle.bias_grad(dZ)
    assert all(abs(Fraction(float(g)) - w) <= abs(w) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 60) for g, w in zip(got, want))
    assert np.array_equal(oracle.bias_grad(np.ascontiguousarray(dZ.T), layout=oracle.COL_MAJOR), got)
    ones = np.ones((5, 8), dtype=np.float32)
    assert (oracle.bias_grad(ones) == 5.0).all()
    # Z = X W^T + d: every row moves by d, and d = 0 gives the plain product
    p, q, r = 8, 64, 16
    W = si.random_matrix(87, (r, q), 0.02, dtype)
    X = si.random_matrix(88, (p, q), 1.0, dtype)
    d = si.random_matrix(89, (r,), 0.5, dtype)
    mask = oracle.transposable_mask(W)
    vals, meta, _, _ = oracle.compress(W, mask)
    Y = oracle.spmm_fwd(X, vals, meta)
    Z = oracle.spmm_fwd_bias(X, vals, meta, d)
    np.testing.assert_allclose(Z - Y, np.broadcast_to(f64(d), (p, r)), rtol=0, atol=1e-15)
    assert np.array_equal(oracle.spmm_fwd_bias(X, vals, meta, np.zeros_like(d)), Y)
