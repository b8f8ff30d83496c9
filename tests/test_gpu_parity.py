"""GPU parity: every libs24 entry point against the CPU oracle, element by
element, on seeded inputs that span several tiles and ragged tails.  Masks,
pattern ids, compressed values and metadata must match bit for bit; GEMM and
activation outputs within the tolerance of tests/util.py."""
import numpy as np
import pytest
import torch

import oracle
import s24_inputs as si
from util import BF16_TOL, F32_TOL, assert_close, dev, dev_bf16, host_bits, host_f64, tol_for, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def s24():
    import paper_2404_01847_amd as lib
    lib.lib()   # fail loudly here if libs24.so is missing
    assert torch.cuda.is_available()
    return lib


def tdtype(dtype):
    return torch_dtype(dtype)


def tol(dtype):
    return tol_for(dtype)


def gpu_mask(s24, W, want_index=True):
    Wd = dev_bf16(W)
    r, q = W.shape
    mask = torch.zeros((r // 4, q // 4), dtype=torch.int16, device="cuda")
    index = torch.zeros((r // 4, q // 4), dtype=torch.uint8, device="cuda") if want_index else None
    s24.transposable_mask(Wd, mask, index)
    torch.cuda.synchronize()
    return host_bits(mask), (host_bits(index) if want_index else None)


def packed(vals, meta):
    """Oracle's row-major compressed operand -> the library's chunk-major storage, on the GPU."""
    vp, mp = oracle.pack(vals, meta)
    return dev_bf16(vp), dev(mp)


def gpu_compress(s24, W, mask=None):
    Wd = dev_bf16(W)
    r, q = W.shape
    dt = Wd.dtype
    vals = torch.zeros((q // 64, r, 32), dtype=dt, device="cuda")
    meta = torch.zeros((q // 64, r, 4), dtype=torch.int16, device="cuda")
    valsT = torch.zeros((r // 64, q, 32), dtype=dt, device="cuda")
    metaT = torch.zeros((r // 64, q, 4), dtype=torch.int16, device="cuda")
    mask_out = torch.zeros((r // 4, q // 4), dtype=torch.int16, device="cuda")
    s24.compress(Wd, None if mask is None else dev(mask), vals, meta, valsT, metaT, mask_out=mask_out)
    torch.cuda.synchronize()
    return vals, meta, valsT, metaT, mask_out


# ------------------------------------------------------------------ pattern table
def test_pattern_table_matches_oracle(s24):
    assert s24.pattern_table() == [int(v) for v in oracle.pattern_table()]


# ------------------------------------------------------------------ mask search
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [(4, 4), (128, 128), (260, 388), (516, 132), (64, 1024)])
def test_mask_random_bit_exact(s24, dtype, shape):
    W = si.random_matrix(100 + shape[0], shape, 0.02, dtype)
    want_m, want_i = oracle.transposable_mask(W, want_index=True)
    got_m, got_i = gpu_mask(s24, W)
    assert np.array_equal(got_m, want_m)
    assert np.array_equal(got_i, want_i)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("kind", ["few", "equal", "zeros", "tiny", "range", "subnormal", "window"])
def test_mask_ties_and_wide_ranges_bit_exact(s24, dtype, kind):
    W = si.tie_matrix(77, 192, 320, dtype, kind)
    want_m, want_i = oracle.transposable_mask(W, want_index=True)
    got_m, got_i = gpu_mask(s24, W)
    assert np.array_equal(got_m, want_m), kind
    assert np.array_equal(got_i, want_i), kind


@pytest.mark.parametrize("dtype,big_exp", [("f32", 30), ("f32", 100), ("bf16", 47), ("bf16", 100)])
def test_mask_margin_below_fp64_resolution(s24, dtype, big_exp, legal_blocks):
    """Blocks whose best pattern wins by one unit in the last place of 1 beside six cells of 2^big_exp (sums of fp64
    terms cannot tell it from an earlier pattern): the search alone and fused with compress."""
    from util import absorbed_margin_blocks
    W, want = absorbed_margin_blocks(legal_blocks, dtype, big_exp)
    W = np.ascontiguousarray(np.tile(W[:, :320], (16, 1)))        # [64, 320]: 16 x 80 blocks
    want_m, want_i = oracle.transposable_mask(W, want_index=True)
    assert [int(v) for v in want_m[0]] == want[:80]
    got_m, got_i = gpu_mask(s24, W)
    assert np.array_equal(got_m, want_m)
    assert np.array_equal(got_i, want_i)
    fused = gpu_compress(s24, W, None)
    assert np.array_equal(host_bits(fused[4]), want_m)


def test_mask_strided_weight_and_empty(s24):
    W = si.random_matrix(5, (64, 256), 0.02, "bf16")
    Wd = dev_bf16(W)
    view = Wd[:, 64:192]                       # ldw = 256 > q = 128
    mask = torch.zeros((16, 32), dtype=torch.int16, device="cuda")
    s24.transposable_mask(view, mask, None)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(mask), oracle.transposable_mask(np.ascontiguousarray(W[:, 64:192])))
    empty = torch.zeros((0, 128), dtype=torch.bfloat16, device="cuda")
    s24.transposable_mask(empty, torch.zeros((0, 32), dtype=torch.int16, device="cuda"), None)


# ------------------------------------------------------------------ compress
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [(64, 64), (128, 128), (320, 448), (576, 192)])
@pytest.mark.parametrize("fused", [False, True])
def test_compress_bit_exact(s24, dtype, shape, fused):
    W = si.random_matrix(200 + shape[1], shape, 0.02, dtype)
    W[0:4, 0:8] = 0
    mask = oracle.transposable_mask(W)
    c = oracle.compress(W, mask)
    want = oracle.pack(c[0], c[1]) + oracle.pack(c[2], c[3])
    vals, meta, valsT, metaT, mask_out = gpu_compress(s24, W, None if fused else mask)
    if fused:
        assert np.array_equal(host_bits(mask_out), mask)
    for got, ref, name in zip((vals, meta, valsT, metaT), want, ("vals", "meta", "valsT", "metaT")):
        g = host_bits(got)
        assert np.array_equal(g.view(ref.dtype) if g.dtype != ref.dtype else g, ref), name


def test_compress_tie_matrix_fused(s24):
    W = si.tie_matrix(3, 128, 256, "bf16", "few")
    mask = oracle.transposable_mask(W)
    c = oracle.compress(W, mask)
    want = oracle.pack(c[0], c[1]) + oracle.pack(c[2], c[3])
    got = gpu_compress(s24, W, None)
    assert np.array_equal(host_bits(got[4]), mask)
    for g, ref in zip(got[:4], want):
        assert np.array_equal(host_bits(g), ref)


# ------------------------------------------------------------------ sparse GEMMs
def compressed(W):
    mask = oracle.transposable_mask(W)
    return (mask,) + oracle.compress(W, mask)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("pqr", [(1, 64, 16), (128, 128, 128), (300, 256, 208), (77, 192, 400), (513, 64, 144)])
def test_spmm_fwd(s24, dtype, pqr):
    p, q, r = pqr
    W = si.random_matrix(300 + r, (r, q), 0.02, dtype)
    X = si.random_matrix(301 + p, (p, q), 1.0, dtype)
    mask, vals, meta, valsT, metaT = compressed(W)
    Y = torch.full((p, r), 7.0, dtype=tdtype(dtype), device="cuda")
    s24.spmm_fwd(dev_bf16(X), *packed(vals, meta), Y)
    torch.cuda.synchronize()
    assert_close(host_f64(Y), oracle.spmm_fwd(X, vals, meta), tol(dtype), f"spmm_fwd {pqr}")


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("pqr", [(1, 16, 64), (128, 128, 128), (300, 208, 256), (77, 400, 192)])
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_spmm_bwd_dx(s24, dtype, pqr, beta):
    p, q, r = pqr
    W = si.random_matrix(310 + r, (r, q), 0.02, dtype)
    dY = si.random_matrix(311 + p, (p, r), 1e-2, dtype)
    dX0 = si.random_matrix(312, (p, q), 1e-3, dtype)
    mask, vals, meta, valsT, metaT = compressed(W)
    dX = dev_bf16(dX0).clone()
    s24.spmm_bwd_dx(dev_bf16(dY), *packed(valsT, metaT), dX, beta=beta)
    torch.cuda.synchronize()
    ref = oracle.spmm_bwd_dx(dY, valsT, metaT, beta=beta, dX0=si.to_f32(dX0).astype(np.float64))
    assert_close(host_f64(dX), ref, tol(dtype), f"spmm_bwd_dx {pqr} beta={beta}")


@pytest.mark.parametrize("k", [64, 128, 192, 256, 320, 448])
def test_spmm_large_tile_path(s24, k):
    """Shapes with at least 192 tiles of 256 x 256 take the large-tile kernel: ragged token and
    feature tails, every residue of the chunk count modulo the three-stage ring."""
    p, r = 6100, 2000
    W = si.random_matrix(330 + k, (r, k), 0.02, "bf16")
    X = si.random_matrix(331 + k, (p, k), 1.0, "bf16")
    mask, vals, meta, valsT, metaT = compressed(W)
    rows = np.unique(np.concatenate([[0, 255, 256, p - 1], np.random.default_rng(k).integers(0, p, 40)])).astype(np.int64)
    ridx = torch.from_numpy(rows).cuda()
    Y = torch.full((p, r), 3.0, dtype=torch.bfloat16, device="cuda")
    s24.spmm_fwd(dev_bf16(X), *packed(vals, meta), Y)
    torch.cuda.synchronize()
    assert_close(host_f64(Y[ridx]), oracle.spmm_fwd(X, vals, meta, rows=rows), BF16_TOL, f"large spmm_fwd k={k}")
    # the same operands as an input-gradient GEMM: dX[p][r'] with r' = 2000 features, contraction k
    # (valsT of a [k x 2000] weight is a [2000 x k/2] operand, which is what `vals` already is)
    dX0 = si.random_matrix(332, (p, r), 1e-2, "bf16")
    dX = dev_bf16(dX0).clone()
    s24.spmm_bwd_dx(dev_bf16(X), *packed(vals, meta), dX, beta=1.0)
    torch.cuda.synchronize()
    ref = oracle.spmm_bwd_dx(X, vals, meta, beta=1.0, dX0=si.to_f32(dX0[rows]).astype(np.float64), rows=rows)
    assert_close(host_f64(dX[ridx]), ref, BF16_TOL, f"large spmm_bwd_dx k={k}")


def test_spmm_large_tiles_with_a_small_tile_strip(s24):
    """296 large tiles are a whole round over 256 compute units plus a mostly empty one: the first 8192 tokens run in
    large tiles and the last 1064 as small tiles in a second launch.  Rows on both sides of the cut, a ragged
    tail, a bias, and beta = 1."""
    p, r, k = 9256, 2000, 192
    W = si.random_matrix(340, (r, k), 0.02, "bf16")
    X = si.random_matrix(341, (p, k), 1.0, "bf16")
    bias = si.random_matrix(342, (r,), 0.3, "bf16")
    mask, vals, meta, valsT, metaT = compressed(W)
    rows = np.unique(np.concatenate([[0, 8063, 8064, 8191, 8192, 8193, 8319, 8320, p - 129, p - 1],
                                     np.random.default_rng(9).integers(0, p, 40)])).astype(np.int64)
    ridx = torch.from_numpy(rows).cuda()
    Y = torch.full((p, r), 3.0, dtype=torch.bfloat16, device="cuda")
    s24.spmm_fwd(dev_bf16(X), *packed(vals, meta), Y)
    torch.cuda.synchronize()
    assert_close(host_f64(Y[ridx]), oracle.spmm_fwd(X, vals, meta, rows=rows), BF16_TOL, "strip spmm_fwd")
    Y.fill_(3.0)
    s24.spmm_fwd_bias(dev_bf16(X), *packed(vals, meta), dev_bf16(bias), Y)
    torch.cuda.synchronize()
    assert_close(host_f64(Y[ridx]), oracle.spmm_fwd_bias(X, vals, meta, bias, rows=rows), BF16_TOL, "strip spmm_fwd_bias")
    dX0 = si.random_matrix(343, (p, r), 1e-2, "bf16")
    dX = dev_bf16(dX0).clone()
    s24.spmm_bwd_dx(dev_bf16(X), *packed(vals, meta), dX, beta=1.0)
    torch.cuda.synchronize()
    ref = oracle.spmm_bwd_dx(X, vals, meta, beta=1.0, dX0=si.to_f32(dX0[rows]).astype(np.float64), rows=rows)
    assert_close(host_f64(dX[ridx]), ref, BF16_TOL, "strip spmm_bwd_dx")
    # every token outside the sample: finite, and not the fill value in all of a row
    assert torch.isfinite(dX.float()).all() and (Y.float() != 3.0).any(dim=1).all()


def test_spmm_one_hot_reproduces_masked_weight_exactly(s24):
    q, r = 128, 144
    W = si.random_matrix(320, (r, q), 0.02, "bf16")
    mask, vals, meta, valsT, metaT = compressed(W)
    eye = dev_bf16(si.f32_to_bf16_bits(torch.eye(q)))
    Y = torch.zeros((q, r), dtype=torch.bfloat16, device="cuda")
    s24.spmm_fwd(eye, *packed(vals, meta), Y)
    torch.cuda.synchronize()
    ref = oracle.spmm_fwd(si.f32_to_bf16_bits(torch.eye(q)), vals, meta)
    assert np.array_equal(host_f64(Y), ref)       # products with 1 and sums with 0 are exact


# ------------------------------------------------------------------ gated forward in one pass
@pytest.mark.parametrize("case", [
    # (p, q, f): the fallback (two kernels) and the fused epilogue (>= 192 tiles of 256 tokens x 128 features),
    # the latter with a ragged last token tile and a ragged last feature tile
    (96, 64, 48), (300, 128, 272), (1000, 128, 6272), (777, 192, 6224)])
def test_spmm_fwd_swiglu_equals_the_two_calls_and_the_oracle(s24, case):
    p, q, f = case
    X = si.random_matrix(900 + p, (p, q), 1.0, "bf16")
    W = si.random_matrix(901 + p, (2 * f, q), 0.02, "bf16")        # stacked [W_gate; W_up]
    mask = oracle.transposable_mask(W)
    vals, meta, _, _ = oracle.compress(W, mask)
    vp, mp = oracle.pack(vals, meta)
    d_X, d_v, d_m = dev_bf16(X), dev_bf16(vp), dev(mp)
    GU = torch.full((p, 2 * f), 7.0, dtype=torch.bfloat16, device="cuda")
    H = torch.full((p, f), 7.0, dtype=torch.bfloat16, device="cuda")
    s24.spmm_fwd_swiglu(d_X, d_v, d_m, GU, H)
    GU2 = torch.empty_like(GU)
    H2 = torch.empty_like(H)
    s24.spmm_fwd(d_X, d_v, d_m, GU2)
    s24.swiglu_fwd(GU2[:, :f], GU2[:, f:], H2)
    torch.cuda.synchronize()
    assert torch.equal(GU.view(torch.int16), GU2.view(torch.int16))            # same bits as the two calls
    assert torch.equal(H.view(torch.int16), H2.view(torch.int16))
    rows = np.unique(np.concatenate([[0, p - 1], np.random.default_rng(p).integers(0, p, 12)])).astype(np.int64)
    Z = oracle.spmm_fwd(X, vals, meta, rows=rows)
    assert_close(host_f64(GU[torch.from_numpy(rows).cuda()]), Z, BF16_TOL, f"GU {case}")
    Zb = oracle.round_bf16(Z)
    Href = oracle.swiglu_fwd(np.ascontiguousarray(Zb[:, :f]), np.ascontiguousarray(Zb[:, f:]))
    assert_close(host_f64(H[torch.from_numpy(rows).cuda()]), Href, (2e-2, 5e-3), f"H {case}")


@pytest.mark.parametrize("case", [(2000, 6272, 128), (1800, 6224, 192)])    # (p, f, r): >= 192 tiles of 256 x 256
def test_spmm_bwd_dx_swiglu_equals_the_two_calls_and_the_oracle(s24, case):
    p, f, r = case
    dY = si.random_matrix(910 + p, (p, r), 1e-2, "bf16")
    Wd = si.random_matrix(911 + p, (r, f), 0.02, "bf16")
    GU = si.random_matrix(912 + p, (p, 2 * f), 1.0, "bf16")
    mask = oracle.transposable_mask(Wd)
    _, _, valsT, metaT = oracle.compress(Wd, mask)
    vtp, mtp = oracle.pack(valsT, metaT)
    d_dY, d_v, d_m, d_GU = dev_bf16(dY), dev_bf16(vtp), dev(mtp), dev_bf16(GU)
    dGU = torch.full((p, 2 * f), 7.0, dtype=torch.bfloat16, device="cuda")
    s24.spmm_bwd_dx_swiglu(d_dY, d_v, d_m, d_GU, dGU)
    dH = torch.empty((p, f), dtype=torch.bfloat16, device="cuda")
    dGU2 = torch.empty_like(dGU)
    s24.spmm_bwd_dx(d_dY, d_v, d_m, dH)
    s24.swiglu_bwd(dH, d_GU[:, :f], d_GU[:, f:], dGU2[:, :f], dGU2[:, f:])
    torch.cuda.synchronize()
    assert torch.equal(dGU.view(torch.int16), dGU2.view(torch.int16))          # same bits as the two calls
    rows = np.unique(np.concatenate([[0, p - 1], np.random.default_rng(p).integers(0, p, 12)])).astype(np.int64)
    dHr = oracle.round_bf16(oracle.spmm_bwd_dx(dY, valsT, metaT, rows=rows))
    G, U = np.ascontiguousarray(GU[rows][:, :f]), np.ascontiguousarray(GU[rows][:, f:])
    dG, dU = oracle.swiglu_bwd(dHr, G, U)
    got = host_f64(dGU[torch.from_numpy(rows).cuda()])
    assert_close(got[:, :f], dG, (2e-2, 5e-3), f"dG {case}")
    assert_close(got[:, f:], dU, (2e-2, 5e-3), f"dU {case}")


def test_spmm_bwd_dx_swiglu_declines_small_shapes(s24):
    p, f, r = 64, 64, 64
    z = torch.zeros((p, 2 * f), dtype=torch.bfloat16, device="cuda")
    before = z.clone()
    v = torch.zeros((1, f, 32), dtype=torch.bfloat16, device="cuda")
    m = torch.zeros((1, f, 4), dtype=torch.int16, device="cuda")
    with pytest.raises(s24.S24Error) as e:
        s24.spmm_bwd_dx_swiglu(torch.zeros((p, r), dtype=torch.bfloat16, device="cuda"), v, m, z, z)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert torch.equal(z, before)


# ------------------------------------------------------------------ dense GEMMs
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("pqr", [(1, 16, 16), (64, 128, 128), (300, 208, 272), (1000, 144, 400)])
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_dense_dw(s24, dtype, pqr, beta):
    p, q, r = pqr
    dY = si.random_matrix(400 + p, (p, r), 1e-2, dtype)
    X = si.random_matrix(401 + q, (p, q), 1.0, dtype)
    dW0 = si.random_matrix(402, (r, q), 1e-2, "f32")
    dW = dev(dW0).clone()
    s24.dense_dw(dev_bf16(dY), dev_bf16(X), dW, beta=beta)
    torch.cuda.synchronize()
    ref = oracle.dense_dw(dY, X, beta=beta, dW0=dW0.astype(np.float64))
    # fp32 output: only accumulation-order noise, whatever the input dtype
    assert_close(host_f64(dW), ref, F32_TOL, f"dense_dw {pqr} beta={beta}")


@pytest.mark.parametrize("p", [1, 64, 130, 200])
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_dense_dw_large_tile_path(s24, p, beta):
    """At least 192 tiles of 256 x 256 take the large-tile kernel: ragged feature tails and token counts."""
    q, r = 6096, 2000
    dY = si.random_matrix(430 + p, (p, r), 1e-2, "bf16")
    X = si.random_matrix(431 + p, (p, q), 1.0, "bf16")
    dW0 = si.random_matrix(432, (r, q), 1e-2, "f32")
    dW = dev(dW0).clone()
    s24.dense_dw(dev_bf16(dY), dev_bf16(X), dW, beta=beta)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, r - 1], np.random.default_rng(p).integers(0, r, 24)])).astype(np.int64)
    ref = oracle.dense_dw(dY, X, beta=beta, dW0=dW0[rows].astype(np.float64), rows=rows)
    assert_close(host_f64(dW[torch.from_numpy(rows).cuda()]), ref, F32_TOL, f"large dense_dw p={p} beta={beta}")


@pytest.mark.parametrize("p", [33, 150])
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_dense_dw_many_small_tiles_path(s24, p, beta):
    """More 128x128 tiles than compute units, fewer 256x256 tiles than fill the chip: the two-workgroups-per-CU
    variant (32 tokens per ring stage, ragged last chunk, ragged last tile row and column)."""
    q, r = 2192, 2160
    dY = si.random_matrix(470 + p, (p, r), 1e-2, "bf16")
    X = si.random_matrix(471 + p, (p, q), 1.0, "bf16")
    dW0 = si.random_matrix(472, (r, q), 1e-3, "f32")
    dW = dev(dW0).clone()
    s24.dense_dw(dev_bf16(dY), dev_bf16(X), dW, beta=beta)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 127, 128, r - 1], np.random.default_rng(p).integers(0, r, 24)])).astype(np.int64)
    ref = oracle.dense_dw(dY, X, beta=beta, dW0=dW0[rows].astype(np.float64), rows=rows)
    assert_close(host_f64(dW[torch.from_numpy(rows).cuda()]), ref, F32_TOL, f"dense_dw small tiles p={p} beta={beta}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("rq", [(4096, 4336), (4240, 4096)])     # 16 x 17 and 17 x 16 large tiles, ragged strip
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_dense_dw_round_exact_slab_plus_small_tile_strip(s24, dtype, rq, beta):
    """Tile grids that are not a whole number of rounds over the compute units are cut into a slab of whole rounds
    (large tiles) and a strip (small tiles), along either axis: rows and columns on both sides of the cut, the
    ragged edge, accumulation and the decay term against the oracle, and the same bits as the unfused route."""
    r, q = rq
    p, lam = 150, 2e-4
    dY = si.random_matrix(480 + r, (p, r), 1e-2, dtype)
    X = si.random_matrix(481 + q, (p, q), 1.0, dtype)
    W = si.random_matrix(482, (r, q), 0.02, dtype)
    dW0 = si.random_matrix(483, (r, q), 1e-3, "f32")
    mask = oracle.transposable_mask(W)
    d_dY, d_X, d_W, d_mask = dev_bf16(dY), dev_bf16(X), dev_bf16(W), dev(mask)
    fused = dev(dW0).clone()
    s24.dense_dw_decay(d_dY, d_X, fused, d_W, d_mask, lam, beta=beta)
    two = dev(dW0).clone()
    s24.dense_dw(d_dY, d_X, two, beta=beta)
    s24.masked_decay_grad(two, d_W, d_mask, lam)
    torch.cuda.synchronize()
    assert torch.equal(fused.view(torch.int32), two.view(torch.int32))
    rows = np.unique(np.concatenate([[0, 4095, r - 1, r - 2, 2048, 4000], np.random.default_rng(r).integers(0, r, 16)])).astype(np.int64)
    g = oracle.dense_dw(dY, X, beta=beta, dW0=dW0[rows].astype(np.float64), rows=rows)
    g = g + oracle.masked_decay(np.zeros((r, q), np.float32), W, mask, lam)[rows]
    assert_close(host_f64(fused[torch.from_numpy(rows).cuda()]), g, F32_TOL, f"dense_dw slab+strip {rq} beta={beta}")


@pytest.mark.parametrize("case", [
    # (dtype, p, [(r, q), ...], decay on each, beta)
    ("bf16", 130, [(22016, 4096), (4096, 11008)], [True, True], 0.0),    # c4's pair: 2064 tiles, one tile row cut off
    ("f16", 70, [(4096, 4352), (4096, 4096), (4112, 4096)], [True, True, True], 1.0),   # 272+256+272 = 800: 32 over, two columns cut
    ("bf16", 90, [(4096, 4096), (4096, 8192)], [False, False], 0.0),     # whole rounds: nothing to cut
    ("bf16", 64, [(4096, 4096), (528, 272)], [True, True], 0.0),         # a small problem: one after the other
    ("bf16", 200, [(3072, 768), (768, 3072)], [True, True], 0.0),        # c2's pair: 144 + 144 small tiles in one grid
    ("f16", 96, [(528, 272), (272, 528), (144, 1040)], [False, False, False], 1.0),   # 15 + 15 + 18 small tiles, ragged
    ("bf16", 64, [(4096, 4096), (4096, 4096)], [True, False], 1.0),      # decay on one only: one after the other
    ("f32", 40, [(64, 48), (32, 96)], [True, False], 0.0)])
def test_dense_dw_batch_equals_the_single_calls_and_the_oracle(s24, case):
    dtype, p, shapes, decays, beta = case
    lam = 3e-4
    probs, singles, host = [], [], []
    for k, ((r, q), dec) in enumerate(zip(shapes, decays)):
        dY = si.random_matrix(3000 + 10 * k, (p, r), 1e-2, dtype)
        X = si.random_matrix(3001 + 10 * k, (p, q), 1.0, dtype)
        W = si.random_matrix(3002 + 10 * k, (r, q), 0.02, dtype)
        dW0 = si.random_matrix(3003 + 10 * k, (r, q), 1e-3, "f32")
        mask = oracle.transposable_mask(W)
        d = (dev_bf16(dY), dev_bf16(X), dev(dW0).clone(), dev_bf16(W) if dec else None, dev(mask) if dec else None, lam)
        probs.append(d)
        one = dev(dW0).clone()
        if dec:
            s24.dense_dw_decay(d[0], d[1], one, d[3], d[4], lam, beta=beta)
        else:
            s24.dense_dw(d[0], d[1], one, beta=beta)
        singles.append(one)
        host.append((dY, X, W, dW0, mask))
    s24.dense_dw_batch(probs, beta=beta)
    torch.cuda.synchronize()
    for k, ((r, q), dec) in enumerate(zip(shapes, decays)):
        assert torch.equal(probs[k][2].view(torch.int32), singles[k].view(torch.int32)), f"problem {k}"
        dY, X, W, dW0, mask = host[k]
        rows = np.unique(np.concatenate([[0, r - 1, r - 2, r // 2], np.random.default_rng(k).integers(0, r, 6)])).astype(np.int64)
        g = oracle.dense_dw(dY, X, beta=beta, dW0=dW0[rows].astype(np.float64), rows=rows)
        if dec:
            g = g + oracle.masked_decay(np.zeros((r, q), np.float32), W, mask, lam)[rows]
        assert_close(host_f64(probs[k][2][torch.from_numpy(rows).cuda()]), g, F32_TOL, f"dense_dw_batch {case[:2]} problem {k}")


def test_dense_dw_no_tokens(s24):
    dW = torch.full((64, 128), 5.0, dtype=torch.float32, device="cuda")
    # with no tokens the operand pointers are never read: any aligned non-null value will do
    assert s24.lib().s24_dense_dw(0x1000, 0x1000, dW.data_ptr(), 0, 128, 64, 1.0, s24.BF16, None) == 0
    torch.cuda.synchronize()
    assert (dW == 5.0).all()                       # beta = 1 keeps the gradient
    assert s24.lib().s24_dense_dw(0x1000, 0x1000, dW.data_ptr(), 0, 128, 64, 0.0, s24.BF16, None) == 0
    torch.cuda.synchronize()
    assert (dW == 0.0).all()                       # beta = 0 clears it


def test_dense_dw_rank_one_is_exact(s24):
    dY = si.random_matrix(410, (1, 144), 1.0, "bf16")
    X = si.random_matrix(411, (1, 208), 1.0, "bf16")
    dW = torch.zeros((144, 208), dtype=torch.float32, device="cuda")
    s24.dense_dw(dev_bf16(dY), dev_bf16(X), dW)
    torch.cuda.synchronize()
    assert np.array_equal(host_f64(dW), oracle.dense_dw(dY, X))    # bf16 x bf16 fits fp32 exactly


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("pqr", [(1, 64, 16), (128, 128, 128), (300, 256, 208)])
def test_dense_gemm(s24, dtype, pqr):
    p, q, r = pqr
    X = si.random_matrix(420 + p, (p, q), 1.0, dtype)
    W = si.random_matrix(421 + r, (r, q), 0.02, dtype)
    Y = torch.zeros((p, r), dtype=tdtype(dtype), device="cuda")
    s24.dense_gemm(dev_bf16(X), dev_bf16(W), Y)
    torch.cuda.synchronize()
    assert_close(host_f64(Y), oracle.dense_gemm(X, W), tol(dtype), f"dense_gemm {pqr}")


@pytest.mark.parametrize("k", [64, 128, 192, 320])
def test_dense_gemm_large_tile_path(s24, k):
    p, r = 6100, 2000
    X = si.random_matrix(440 + k, (p, k), 1.0, "bf16")
    W = si.random_matrix(441 + k, (r, k), 0.02, "bf16")
    Y = torch.full((p, r), 3.0, dtype=torch.bfloat16, device="cuda")
    s24.dense_gemm(dev_bf16(X), dev_bf16(W), Y)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, p - 1], np.random.default_rng(k).integers(0, p, 40)])).astype(np.int64)
    assert_close(host_f64(Y[torch.from_numpy(rows).cuda()]), oracle.dense_gemm(X, W, rows=rows), BF16_TOL,
                 f"large dense_gemm k={k}")


# ------------------------------------------------------------------ masked decay
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [(16, 16), (260, 400), (128, 1024)])
def test_masked_decay(s24, dtype, shape):
    lam = 2e-4
    W = si.random_matrix(500 + shape[0], shape, 0.02, dtype)
    dW = si.random_matrix(501, shape, 1e-3, "f32")
    mask = oracle.transposable_mask(W)
    G = dev(dW).clone()
    s24.masked_decay_grad(G, dev_bf16(W), dev(mask), lam)
    torch.cuda.synchronize()
    got = host_bits(G)
    ref = oracle.masked_decay(dW, W, mask, lam)
    keep = np.zeros(shape, dtype=bool)
    for i in range(4):
        for j in range(4):
            keep[i::4, j::4] = ((mask >> (4 * i + j)) & 1).astype(bool)
    assert np.array_equal(got[keep], dW[keep])                       # kept cells bit-identical
    np.testing.assert_allclose(got.astype(np.float64), ref, rtol=3e-7, atol=0)


# ------------------------------------------------------------------ weight gradient + masked decay in one call
@pytest.mark.parametrize("case", [
    # (p, q, r, dtype, beta): small tiles, fp32 route, and enough 256x256 tiles for the fused epilogue
    (300, 256, 208, "bf16", 0.0), (96, 64, 48, "f32", 1.0),
    (1000, 3600, 3408, "bf16", 0.0), (777, 3600, 3408, "bf16", 1.0), (90, 2192, 2160, "bf16", 1.0)])
def test_dense_dw_decay_equals_the_two_calls_and_the_oracle(s24, case):
    p, q, r, dtype, beta = case
    lam = 2e-4
    dY = si.random_matrix(600 + p, (p, r), 1e-2, dtype)
    X = si.random_matrix(601 + p, (p, q), 1.0, dtype)
    W = si.random_matrix(602 + p, (r, q), 0.02, dtype)
    dW0 = si.random_matrix(603 + p, (r, q), 1e-3, "f32")
    mask = oracle.transposable_mask(W)
    d_dY, d_X, d_W, d_mask = dev_bf16(dY), dev_bf16(X), dev_bf16(W), dev(mask)
    fused = dev(dW0).clone()
    s24.dense_dw_decay(d_dY, d_X, fused, d_W, d_mask, lam, beta=beta)
    two = dev(dW0).clone()
    s24.dense_dw(d_dY, d_X, two, beta=beta)
    s24.masked_decay_grad(two, d_W, d_mask, lam)
    torch.cuda.synchronize()
    assert torch.equal(fused.view(torch.int32), two.view(torch.int32))          # same bits by construction
    rows = np.unique(np.concatenate([[0, 3, 4, r - 1], np.random.default_rng(p).integers(0, r, 20)])).astype(np.int64)
    g = oracle.dense_dw(dY, X, beta=beta, dW0=dW0[rows].astype(np.float64), rows=rows)
    # the decay term of the sampled rows, from the oracle's own decay on a zero gradient
    g = g + oracle.masked_decay(np.zeros((r, q), np.float32), W, mask, lam)[rows]
    assert_close(host_f64(fused[torch.from_numpy(rows).cuda()]), g, tol("f32") if dtype == "f32" else F32_TOL,
                 f"dense_dw_decay {case}")


# ------------------------------------------------------------------ unbiased 2:4 pruning of dY and the sparse weight gradient
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [(64, 16), (128, 80), (448, 272), (1024, 1040)])
def test_mvue24_matches_the_oracle_bit_for_bit(s24, dtype, shape):
    p, r = shape
    dY = si.random_matrix(800 + p, (p, r), 1e-2, dtype)
    dY[:8, : r // 2] = 0                                  # all-zero and half-zero groups
    dY[8:16:2, :] = 0
    vals = torch.zeros((p // 64, r, 32), dtype=tdtype(dtype), device="cuda")
    meta = torch.zeros((p // 64, r, 4), dtype=torch.int16, device="cuda")
    s24.mvue24(dev_bf16(dY), 20240401, vals, meta)
    torch.cuda.synchronize()
    want_v, want_m = oracle.pack(*oracle.mvue24(dY, 20240401))
    assert np.array_equal(host_bits(meta), want_m)
    word = np.uint32 if dtype == "f32" else np.uint16
    assert np.array_equal(host_bits(vals).view(word), want_v.view(word))
    # another seed gives another draw
    s24.mvue24(dev_bf16(dY), 7, vals, meta)
    torch.cuda.synchronize()
    want_v2, want_m2 = oracle.pack(*oracle.mvue24(dY, 7))
    assert np.array_equal(host_bits(meta), want_m2) and not np.array_equal(want_m2, want_m)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_mvue24_degenerate_and_repeated_groups(s24, dtype):
    """Groups with one non-zero at each position, the same four numbers in every group of every feature (only the draw
    differs), equal magnitudes, and a dominant element (capped probability): bit for bit as the oracle."""
    p, r = 128, 80
    x = np.zeros((p, r), dtype=np.float32)
    for pos in range(4):
        x[16 * pos + pos:16 * pos + 16:4, :] = (-1.0) ** pos * (0.375 + pos)     # tokens 0..63: single non-zeros
    x[64:96] = np.tile(np.array([1.0, -2.0, 3.0, 4.0], dtype=np.float32), 8)[:, None]
    x[96:112] = np.tile(np.array([2.0, -2.0, 2.0, 2.0], dtype=np.float32), 4)[:, None]
    x[112:128] = np.tile(np.array([9.0, 0.0, 2.0, -1.0], dtype=np.float32), 4)[:, None]
    dY = x if dtype == "f32" else si.f32_to_bf16_bits(torch.from_numpy(x))
    vals = torch.zeros((p // 64, r, 32), dtype=tdtype(dtype), device="cuda")
    meta = torch.zeros((p // 64, r, 4), dtype=torch.int16, device="cuda")
    for seed in (1, 2, 3):
        s24.mvue24(dev_bf16(dY), seed, vals, meta)
        torch.cuda.synchronize()
        want_v, want_m = oracle.pack(*oracle.mvue24(dY, seed))
        word = np.uint32 if dtype == "f32" else np.uint16
        assert np.array_equal(host_bits(meta), want_m), seed
        assert np.array_equal(host_bits(vals).view(word), want_v.view(word)), seed


def test_mvue24_strided_input(s24):
    p, r = 128, 96
    full = si.random_matrix(810, (p, 2 * r), 1e-2, "bf16")
    d = dev_bf16(full)
    vals = torch.zeros((p // 64, r, 32), dtype=torch.bfloat16, device="cuda")
    meta = torch.zeros((p // 64, r, 4), dtype=torch.int16, device="cuda")
    s24.mvue24(d[:, r:], 5, vals, meta)                   # the right half of a [p, 2r] buffer
    torch.cuda.synchronize()
    want_v, want_m = oracle.pack(*oracle.mvue24(np.ascontiguousarray(full[:, r:]), 5))
    assert np.array_equal(host_bits(meta), want_m) and np.array_equal(host_bits(vals), want_v)


def gpu_mvue_dense(s24, dY, seed):
    """The kernel's own compressed S_z(dY^T), decoded on the host (no oracle code involved) to a dense [r, p] float64
    matrix plus the kept-position flags."""
    p, r = dY.shape
    vals = torch.zeros((p // 64, r, 32), dtype=torch.float32, device="cuda")
    meta = torch.zeros((p // 64, r, 4), dtype=torch.int16, device="cuda")
    s24.mvue24(dev(dY), seed, vals, meta)
    torch.cuda.synchronize()
    v = host_bits(vals).transpose(1, 0, 2).reshape(r, p // 4, 2).astype(np.float64)        # chunk-major -> per feature
    m = host_bits(meta).transpose(1, 0, 2).reshape(r, p // 16).astype(np.int64)
    nib = ((m[:, :, None] >> (4 * np.arange(4))) & 0xF).reshape(r, p // 4)
    i0, i1 = nib & 3, nib >> 2
    assert (i0 < i1).all()
    out = np.zeros((r, p // 4, 4))
    kept = np.zeros((r, p // 4, 4), dtype=bool)
    rr, gg = np.meshgrid(np.arange(r), np.arange(p // 4), indexing="ij")
    out[rr, gg, i0], out[rr, gg, i1] = v[:, :, 0], v[:, :, 1]
    kept[rr, gg, i0] = kept[rr, gg, i1] = True
    return out, kept


@pytest.mark.parametrize("group", [(1.0, 2.0, 3.0, 4.0), (0.3, -0.2, 0.25, -0.1), (5.0, 1.0, -1.5, 0.5), (9.0, 0.0, 2.0, -1.0)])
def test_mvue24_kernel_output_is_unbiased_with_the_least_second_moment(s24, group):
    """Statistics of the KERNEL's draws, against what Eq. 6's name fixes and no code of ours: 65536 draws of one
    group (the same four numbers in every token group of 64 features x 1024 groups).  Sample mean = the group;
    inclusion frequencies = min(1, |a_j| / tau) with sum 2; summed second moment = the Lagrange minimum of
    sum a_j^2 / pi_j (S^2/2 uncapped, max^2 + R^2 capped); every kept value = a_j / pi_j from the plain fp64
    definition to a few fp32 ulp; frequencies also hold along features alone and along token groups alone."""
    a = np.array(group, dtype=np.float32)
    r, G = 64, 1024
    dY = np.tile(a.reshape(4, 1), (G, r))
    out, kept = gpu_mvue_dense(s24, dY, 7)
    n = r * G
    samples, flags = out.reshape(n, 4), kept.reshape(n, 4)
    m = np.abs(a.astype(np.float64))
    S, mx = m.sum(), m.max()
    if 2 * mx <= S:
        pi, second = 2 * m / S, S * S / 2
    else:
        R = S - mx
        pi, second = np.where(m == mx, 1.0, m / R), mx * mx + R * R
    assert (flags.sum(axis=1) == 2).all()
    var = np.where(pi > 0, m * m * (1 / np.maximum(pi, 1e-300) - 1), 0.0)
    assert np.all(np.abs(samples.mean(axis=0) - a) <= 5 * np.sqrt(var / n) + 1e-6)
    assert np.all(np.abs(flags.mean(axis=0) - pi) <= 5 * np.sqrt(pi * (1 - pi) / n) + 1e-6)
    assert abs((samples ** 2).sum(axis=1).mean() - second) <= 0.02 * second
    # kept values from the definition a_j / pi_j in fp64 (zero-probability cells are kept only as exact zeros)
    want = np.where(pi > 0, a.astype(np.float64) / np.maximum(pi, 1e-300), 0.0)
    for j in range(4):
        got = samples[flags[:, j], j]
        assert np.all(np.abs(got - want[j]) <= 4 * 2.0 ** -23 * abs(want[j])), (j, want[j], got[:4])
    assert (samples[~flags] == 0).all()
    # the draws differ along each axis alone
    tol = lambda k: 5 * np.sqrt(pi * (1 - pi) / k) + 1e-9
    assert np.all(np.abs(kept[:, 0, :].mean(axis=0) - pi) <= tol(r) + 0.05)          # 64 features of one group
    assert np.all(np.abs(kept[0].mean(axis=0) - pi) <= tol(G))                        # 1024 groups of one feature


def test_mvue24_kernel_probabilities_follow_the_definition_on_random_groups(s24):
    """Random groups, 512 seeds: each element's inclusion frequency over the seeds against pi_j = min(1, |a_j|/tau)
    computed in fp64 from the plain definition (the largest element capped at one when it exceeds the others' sum),
    each kept value against a_j / pi_j, and the mean of the estimates against the input (unbiasedness)."""
    p, r, seeds = 64, 64, 512
    dY = si.random_matrix(830, (p, r), 1.0, "f32")
    dY[0:4, :8] *= np.array([8.0, 1.0, 1.0, 1.0], dtype=np.float32)[:, None]          # some capped groups
    a = dY.T.reshape(r, p // 4, 4).astype(np.float64)
    m = np.abs(a)
    S, mx = m.sum(axis=2, keepdims=True), m.max(axis=2, keepdims=True)
    capped = 2 * mx > S
    pi = np.where(capped, np.where(m == mx, 1.0, m / (S - mx)), 2 * m / S)
    want = a / pi
    freq = np.zeros_like(pi)
    mean = np.zeros_like(pi)
    for seed in range(seeds):
        out, kept = gpu_mvue_dense(s24, dY, 3000 + seed)
        out, kept = out.reshape(r, p // 4, 4), kept.reshape(r, p // 4, 4)
        assert np.all(np.abs(out[kept] - want[kept]) <= 8 * 2.0 ** -23 * np.abs(want[kept]))
        freq += kept
        mean += out
    freq /= seeds
    mean /= seeds
    assert np.all(np.abs(freq - pi) <= 5.5 * np.sqrt(pi * (1 - pi) / seeds) + 1e-9)
    sd = np.sqrt(m * m * (1 / pi - 1) / seeds)
    assert np.all(np.abs(mean - a) <= 5.5 * sd + 1e-6 * m)


def test_mvue24_kernel_neighbouring_seeds_give_unrelated_draws(s24):
    """Consecutive seeds (what a layer passes from one operand and step to the next) on the kernel itself: the kept
    pairs of seed s + 1 are neither those of seed s nor a rearrangement of them over the token groups of a feature."""
    a = np.array([1.0, -2.0, 3.0, 4.0], dtype=np.float32)
    r, G = 256, 64
    dY = np.tile(a.reshape(4, 1), (G, r))
    code = lambda kept: (kept.reshape(r, G, 4) * (1 << np.arange(4))).sum(axis=2)
    k0, k1 = code(gpu_mvue_dense(s24, dY, 1000)[1]), code(gpu_mvue_dense(s24, dY, 1001)[1])
    assert (k0 == k1).mean() < 0.45
    hist = lambda c: np.stack([np.bincount(row, minlength=16) for row in c])
    assert (hist(k0) == hist(k1)).all(axis=1).mean() < 0.05


@pytest.mark.parametrize("case", [
    # (p, q, r, dtype, beta, decay)
    (64, 16, 16, "bf16", 0.0, False), (192, 272, 144, "bf16", 1.0, False), (128, 64, 48, "f32", 1.0, True),
    (448, 1040, 528, "bf16", 0.0, True), (1024, 3600, 3408, "bf16", 1.0, True),
    # two and five 64-token chunks: the remaining residues of the chunk count modulo the three-stage ring
    (128, 272, 144, "bf16", 0.0, True), (320, 528, 272, "f16", 1.0, False)])
def test_spmm_dw_on_the_pruned_gradient(s24, case):
    """S_z(dY^T) X from the oracle's own pruned operand: the GEMM is checked on its own (its input is
    the oracle's compressed operand, not the GPU's), with and without accumulation and the decay term."""
    p, q, r, dtype, beta, decay = case
    lam = 2e-4
    dY = si.random_matrix(820 + p, (p, r), 1e-2, dtype)
    X = si.random_matrix(821 + p, (p, q), 1.0, dtype)
    W = si.random_matrix(822 + p, (r, q), 0.02, dtype)
    dW0 = si.random_matrix(823 + p, (r, q), 1e-3, "f32")
    mask = oracle.transposable_mask(W)
    vz, mz = oracle.mvue24(dY, 99)
    vp, mp = oracle.pack(vz, mz)
    dW = dev(dW0).clone()
    s24.spmm_dw(dev_bf16(vp), dev(mp), dev_bf16(X), dW, beta=beta,
                W=dev_bf16(W) if decay else None, mask=dev(mask) if decay else None, lam=lam if decay else 0.0)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 3, r - 1], np.random.default_rng(p).integers(0, r, 20)])).astype(np.int64)
    # dW^T = X^T . S^T: the oracle's sparse forward GEMM with X^T as the dense operand and S_z(dY^T) as the weight
    Xt = np.ascontiguousarray(X.T)
    ref = oracle.spmm_fwd(Xt, vz, mz).T[rows] + beta * dW0[rows].astype(np.float64)
    if decay:
        ref = ref + oracle.masked_decay(np.zeros((r, q), np.float32), W, mask, lam)[rows]
    assert_close(host_f64(dW[torch.from_numpy(rows).cuda()]), ref, F32_TOL, f"spmm_dw {case}")


# ------------------------------------------------------------------ monitors
@pytest.mark.parametrize("shape", [(4, 4), (64, 96), (260, 1000), (1024, 1028)])
def test_mask_flips(s24, shape):
    w0 = si.random_matrix(700 + shape[0], shape, 0.02, "bf16")
    w1 = si.random_matrix(701 + shape[0], shape, 0.02, "bf16")
    # half of the blocks keep their weights, so some masks do not change at all
    w1[: shape[0] // 8 * 4] = w0[: shape[0] // 8 * 4]
    m0, m1 = oracle.transposable_mask(w0), oracle.transposable_mask(w1)
    flips = torch.full((1,), 12345, dtype=torch.int64, device="cuda")
    per = np.arange(m0.size, dtype=np.uint32)                      # non-zero start: the counter accumulates
    d_per = torch.from_numpy(per.view(np.int32).copy()).cuda()
    # a 16-byte aligned pair of device masks (4x4 alone is 2 bytes: pad the allocation)
    d0 = torch.zeros(m0.size + 8, dtype=torch.int16, device="cuda")
    d1 = torch.zeros(m0.size + 8, dtype=torch.int16, device="cuda")
    d0[: m0.size] = dev(m0).reshape(-1)
    d1[: m0.size] = dev(m1).reshape(-1)
    s24.lib()
    rc = s24.lib().s24_mask_flips(d1.data_ptr(), d0.data_ptr(), m0.size, d_per.data_ptr(), flips.data_ptr(), None)
    assert rc == 0
    torch.cuda.synchronize()
    want_per = per.copy()
    want = oracle.mask_flips(m1, m0, want_per)
    assert int(flips.item()) == want
    assert np.array_equal(d_per.cpu().numpy().view(np.uint32), want_per)
    # without the per-block counter, and with no blocks at all
    s24.lib().s24_mask_flips(d1.data_ptr(), d0.data_ptr(), m0.size, None, flips.data_ptr(), None)
    torch.cuda.synchronize()
    assert int(flips.item()) == want
    assert s24.lib().s24_mask_flips(None, None, 0, None, flips.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert int(flips.item()) == 0


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [(4, 4), (64, 96), (260, 1000)])
def test_l1_norm_gap_matches_the_oracle_bit_for_bit(s24, dtype, shape):
    W = si.random_matrix(720 + shape[0], shape, 0.02, dtype)
    gap = torch.full((shape[0] // 4, shape[1] // 4), -1.0, dtype=torch.float64, device="cuda")
    s24.l1_norm_gap(dev_bf16(W), gap)
    torch.cuda.synchronize()
    ref = oracle.l1_norm_gap(W)
    # N(0, 0.02) blocks stay far inside the exponent window in which fp64 sums are exact
    assert np.array_equal(gap.cpu().numpy(), ref)


@pytest.mark.parametrize("kind", ["few", "equal", "zeros", "range"])
def test_l1_norm_gap_on_tied_and_wide_range_blocks(s24, kind):
    W = si.tie_matrix(730, 64, 64, "bf16", kind)
    gap = torch.empty((16, 16), dtype=torch.float64, device="cuda")
    s24.l1_norm_gap(dev_bf16(W), gap)
    torch.cuda.synchronize()
    got, ref = gap.cpu().numpy(), oracle.l1_norm_gap(W)
    a = np.abs(si.to_f32(W).astype(np.float64))
    scale = a.reshape(16, 4, 16, 4).sum(axis=(1, 3))          # an upper bound of every kept norm of the block
    assert (got >= 0).all()
    assert np.all(np.abs(got - ref) <= 2.0 ** -50 * scale)     # fp64 rounding of sums of eight terms at most
    if kind in ("few", "equal", "zeros"):
        assert np.array_equal(got, ref)


# ------------------------------------------------------------------ activations
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("pf", [(1, 8), (37, 264), (256, 1000)])
def test_swiglu_fwd_bwd(s24, dtype, pf):
    p, f = pf
    g = si.random_matrix(600 + p, (p, f), 2.0, dtype)
    u = si.random_matrix(601 + f, (p, f), 1.0, dtype)
    d = si.random_matrix(602, (p, f), 1e-2, dtype)
    G, U, D = dev_bf16(g), dev_bf16(u), dev_bf16(d)
    H = torch.zeros_like(G)
    dG, dU = torch.zeros_like(G), torch.zeros_like(G)
    s24.swiglu_fwd(G, U, H)
    s24.swiglu_bwd(D, G, U, dG, dU)
    torch.cuda.synchronize()
    assert_close(host_f64(H), oracle.swiglu_fwd(g, u), tol(dtype), "swiglu_fwd")
    rg, ru = oracle.swiglu_bwd(d, g, u)
    assert_close(host_f64(dG), rg, tol(dtype), "swiglu_bwd dG")
    assert_close(host_f64(dU), ru, tol(dtype), "swiglu_bwd dU")


def test_swiglu_halves_of_one_buffer_and_extremes(s24):
    p, f = 19, 136
    gu = si.random_matrix(610, (p, 2 * f), 1.5, "bf16")
    gu[0, :8] = si.f32_to_bf16_bits(torch.tensor([0.0, -0.0, 88.0, -88.0, 3e38, -3e38, 1e-30, -1e-30]))
    d = si.random_matrix(611, (p, f), 1.0, "bf16")
    GU = dev_bf16(gu)
    G, U = GU[:, :f], GU[:, f:]
    H = torch.zeros((p, f), dtype=torch.bfloat16, device="cuda")
    dGU = torch.zeros_like(GU)
    s24.swiglu_fwd(G, U, H)
    s24.swiglu_bwd(dev_bf16(d), G, U, dGU[:, :f], dGU[:, f:])
    torch.cuda.synchronize()
    g, u = np.ascontiguousarray(gu[:, :f]), np.ascontiguousarray(gu[:, f:])
    h = host_f64(H)
    assert np.isfinite(h).all()
    assert_close(h, oracle.swiglu_fwd(g, u), BF16_TOL, "swiglu_fwd halves")
    rg, ru = oracle.swiglu_bwd(d, g, u)
    out = host_f64(dGU)
    assert_close(out[:, :f], rg, BF16_TOL, "swiglu_bwd dG halves")
    assert_close(out[:, f:], ru, BF16_TOL, "swiglu_bwd dU halves")


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("act", ["relu", "gelu"])
def test_act_fwd_bwd(s24, dtype, act):
    code = {"relu": (s24.ACT_RELU, oracle.ACT_RELU), "gelu": (s24.ACT_GELU_ERF, oracle.ACT_GELU_ERF)}[act]
    z = si.random_matrix(620, (33, 264), 1.5, dtype)
    z.reshape(-1)[:5] = 0
    d = si.random_matrix(621, (33, 264), 1e-2, dtype)
    Z, D = dev_bf16(z), dev_bf16(d)
    H, dZ = torch.zeros_like(Z), torch.zeros_like(Z)
    s24.act_fwd(Z, H, code[0])
    s24.act_bwd(D, Z, dZ, code[0])
    torch.cuda.synchronize()
    assert_close(host_f64(H), oracle.act_fwd(z, code[1]), tol(dtype), f"{act} fwd")
    assert_close(host_f64(dZ), oracle.act_bwd(d, z, code[1]), tol(dtype), f"{act} bwd")


# ------------------------------------------------------------------ instrumentation
def test_probe_copy_copies_and_matrix_rate_probe_runs(s24):
    src = torch.arange(0, 3 * 1000 * 4 + 4, dtype=torch.int32, device="cuda")          # ragged: not a whole run
    dst = torch.zeros_like(src)
    s24.probe_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    sink = torch.full((4 * 512,), float("nan"), dtype=torch.float32, device="cuda")
    for sparse in (0, 1):
        s24.probe_matrix_rate(sparse, 4, 8, sink)
        torch.cuda.synchronize()
        assert torch.isfinite(sink).all()
    # four accumulators of 32 x 32 x (16 * 8) products of values below 1/2: a loose bound that a wrong loop breaks
    assert float(sink.abs().max()) < 4 * 16 * 8 * 32 * 0.25 * 64
