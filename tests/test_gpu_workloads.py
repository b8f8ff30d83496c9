"""GPU parity on the five benchmark workloads.

c1 (fp32, ReLU) runs the whole FFN step and is compared stage by stage with an
oracle chain.  c2..c5 are checked at full size, in the launch configuration the
benchmark times: masks, compressed values and metadata bit-exactly over every
weight; GEMM outputs on randomly sampled output rows (the oracle computes each
sampled row in full); elementwise kernels on sampled row bands."""
import numpy as np
import pytest
import torch

import oracle
import s24_inputs as si
from util import BF16_TOL, F32_TOL, assert_close, dev, dev_bf16, host_bits, host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def s24():
    import paper_2404_01847_amd as lib
    lib.lib()
    assert torch.cuda.is_available()
    return lib


def keep_of(mask):
    r4, q4 = mask.shape
    keep = np.zeros((4 * r4, 4 * q4), dtype=bool)
    for i in range(4):
        for j in range(4):
            keep[i::4, j::4] = ((mask >> (4 * i + j)) & 1).astype(bool)
    return keep


# ------------------------------------------------------------------ whole step, oracle chain
def oracle_chain(wl, t, rnd):
    """Reference FFN step.  `rnd` rounds a stage output to the storage dtype the
    GPU pipeline uses between kernels, so both sides round at the same points."""
    out = {}
    comp = {}
    for n in wl.weight_names:
        m = oracle.transposable_mask(t[n])
        comp[n] = (m,) + oracle.compress(t[n], m)
        out["mask_" + n] = m
    X, dY = t["X"], t["dY"]
    if wl.gated:
        G = rnd(oracle.spmm_fwd(X, comp["Wg"][1], comp["Wg"][2]))
        U = rnd(oracle.spmm_fwd(X, comp["Wu"][1], comp["Wu"][2]))
        H = rnd(oracle.swiglu_fwd(G, U))
        Y = oracle.spmm_fwd(H, comp["Wd"][1], comp["Wd"][2])
        dH = rnd(oracle.spmm_bwd_dx(dY, comp["Wd"][3], comp["Wd"][4]))
        dG64, dU64 = oracle.swiglu_bwd(dH, G, U)
        dG, dU = rnd(dG64), rnd(dU64)
        dX1 = oracle.spmm_bwd_dx(dG, comp["Wg"][3], comp["Wg"][4])
        dX = oracle.spmm_bwd_dx(dU, comp["Wu"][3], comp["Wu"][4], beta=1.0, dX0=si.to_f32(rnd(dX1)).astype(np.float64))
        grads = {"Wd": oracle.dense_dw(dY, H), "Wg": oracle.dense_dw(dG, X), "Wu": oracle.dense_dw(dU, X)}
        out.update(G=G, U=U, H=H, dH=dH, dG=dG, dU=dU)
    else:
        act = oracle.ACT_RELU if wl.act == "relu" else oracle.ACT_GELU_ERF
        Z = rnd(oracle.spmm_fwd(X, comp["W1"][1], comp["W1"][2]))
        H = rnd(oracle.act_fwd(Z, act))
        Y = oracle.spmm_fwd(H, comp["W2"][1], comp["W2"][2])
        dH = rnd(oracle.spmm_bwd_dx(dY, comp["W2"][3], comp["W2"][4]))
        dZ = rnd(oracle.act_bwd(dH, Z, act))
        dX = oracle.spmm_bwd_dx(dZ, comp["W1"][3], comp["W1"][4])
        grads = {"W2": oracle.dense_dw(dY, H), "W1": oracle.dense_dw(dZ, X)}
        out.update(Z=Z, H=H, dH=dH, dZ=dZ)
    out.update(Y=Y, dX=dX)
    for n in wl.weight_names:
        out["grad_" + n] = oracle.masked_decay(grads[n].astype(np.float32), t[n], comp[n][0], wl.lam)
    return out


def run_chain(s24, wl, t, tol_act, tol_grad):
    from paper_2404_01847_amd.ffn import SparseFFN
    rnd = lambda a: oracle.round_like(a, t["X"])
    ref = oracle_chain(wl, t, rnd)
    ffn = SparseFFN({n: dev_bf16(t[n]) for n in wl.weight_names}, t["X"].shape[0], wl.act, wl.lam)
    X, dY = dev_bf16(t["X"]), dev_bf16(t["dY"])
    ffn.step(X, dY)
    torch.cuda.synchronize()
    for n in wl.weight_names:
        assert np.array_equal(host_bits(ffn.w[n].mask), ref["mask_" + n]), n
    names = ("G", "U", "H", "Y", "dH", "dG", "dU", "dX") if wl.gated else ("Z", "H", "Y", "dH", "dZ", "dX")
    if not wl.gated and ffn.fuse_gate_bwd:
        # the second projection's input-gradient GEMM applied act'(Z) in its epilogue: dH never reached memory.  The
        # plain GEMM gives it here, so that the chain is still checked stage by stage.
        s24.spmm_bwd_dx(dY, ffn.w["W2"].valsT, ffn.w["W2"].metaT, ffn.dH)
        torch.cuda.synchronize()
    for k in names:
        want = ref[k]
        want = si.to_f32(want).astype(np.float64) if want.dtype != np.float64 else want
        assert_close(host_f64(getattr(ffn, k)), want, tol_act, f"{wl.name} {k}")
    # Weight gradients are sums over tokens in which a rounding that flipped upstream shows at full size in the
    # near-cancelled elements: they are checked against the oracle applied to what the GPU itself stored for the
    # operands of each weight-gradient GEMM (the stage values above already tie those operands to the oracle).
    ops = ({"Wd": ("dY", "H"), "Wg": ("dG", "X"), "Wu": ("dU", "X")} if wl.gated else {"W2": ("dY", "H"), "W1": ("dZ", "X")})
    stored = {"X": t["X"], "dY": t["dY"]}
    for n in wl.weight_names:
        a, b = (stored[k] if k in stored else host_bits(getattr(ffn, k)) for k in ops[n])
        want = oracle.masked_decay(oracle.dense_dw(a, b).astype(np.float32), t[n], ref["mask_" + n], wl.lam)
        assert_close(host_f64(ffn.w[n].grad), want, tol_grad, f"{wl.name} grad {n}")


def test_c1_whole_step_fp32(s24):
    wl = si.WORKLOADS["c1"]
    run_chain(s24, wl, si.make(wl), F32_TOL, F32_TOL)


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_reduced_bf16_whole_step(s24, act):
    # a small layer of the same structure as c2/c3 (ungated) and c4/c5 (gated); ragged token count
    wl = si.Workload("mini_" + act, 200, 128, 448, act, "bf16", 17)
    # the chain compounds bf16 roundings: a 1-ulp flip upstream moves a downstream value by up to its own
    # rounding step, so the element bound is doubled here; the normwise bound stays
    run_chain(s24, wl, si.make(wl), (2e-2, 5e-3), F32_TOL)


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_reduced_binary16_whole_step(s24, act):
    # the same small layers in IEEE binary16, the paper's own precision: three more significant bits than bf16, so
    # the normwise bound is five times tighter; the element bound is the doubled one of the bf16 chain for the
    # same reason (a flipped rounding upstream moves a near-cancelled element downstream by its own rounding step)
    # Output gradients of unit scale: binary16 training scales the loss precisely so that the gradients of a layer
    # like this one (1e-5 .. 1e-4 at the workloads' 1e-2) do not fall among the subnormals, where they keep
    # only a few bits.
    wl = si.Workload("mini16_" + act, 200, 128, 448, act, "f16", 18, std_dy=1.0)
    run_chain(s24, wl, si.make(wl), (2e-2, 1e-3), F32_TOL)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_geglu_layer_with_biases_whole_step(s24, dtype):
    """Sec. 5.2 as written: concatenated gate/up weight and bias, Z = X W^T + d, GELU(Z_1) .* Z_2, and the
    backward of all of it including the bias gradients, against an oracle chain that rounds where the kernels do."""
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.Workload("mini_geglu", 200, 128, 448, "geglu", dtype, 19, std_dy=1.0 if dtype == "f16" else 1e-2)
    t = si.make(wl)
    p, d, f = 200, wl.d_model, wl.d_ff
    Wgu = np.concatenate([t["Wg"], t["Wu"]], axis=0)
    bgu = si.random_matrix(191, (2 * f,), 0.3, dtype)
    bd = si.random_matrix(192, (d,), 0.3, dtype)
    rnd = lambda a: oracle.round_like(a, t["X"])
    mgu, md = oracle.transposable_mask(Wgu), oracle.transposable_mask(t["Wd"])
    cgu, cd = oracle.compress(Wgu, mgu), oracle.compress(t["Wd"], md)
    X, dY = t["X"], t["dY"]
    Z = rnd(oracle.spmm_fwd_bias(X, cgu[0], cgu[1], bgu))
    H = rnd(oracle.glu_fwd(Z, oracle.GATE_GELU_ERF))
    Y = oracle.spmm_fwd_bias(H, cd[0], cd[1], bd)
    dH = rnd(oracle.spmm_bwd_dx(dY, cd[2], cd[3]))
    dZ = rnd(oracle.glu_bwd(dH, Z, oracle.GATE_GELU_ERF))
    dX = oracle.spmm_bwd_dx(dZ, cgu[2], cgu[3])

    ffn = SparseFFN({n: dev_bf16(t[n]) for n in wl.weight_names}, p, "geglu", wl.lam, concat_gate_up=True,
                    biases={"Wgu": dev_bf16(bgu), "Wd": dev_bf16(bd)})
    ffn.step(dev_bf16(X), dev_bf16(dY))
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(ffn.w["Wgu"].mask), mgu) and np.array_equal(host_bits(ffn.w["Wd"].mask), md)
    tol = (2e-2, 5e-3) if dtype == "bf16" else (2e-2, 1e-3)
    widen = lambda a: a if a.dtype == np.float64 else si.to_f32(a).astype(np.float64)
    for name, want in (("GU", Z), ("H", H), ("Y", Y), ("dGU", dZ), ("dX", dX)):
        assert_close(host_f64(getattr(ffn, name)), widen(want), tol, f"geglu {dtype} {name}")
    # Weight and bias gradients: sums over tokens in which a rounding flipped upstream shows at full size in the
    # near-cancelled elements, so they are checked against the oracle applied to the kernels' own inputs (what
    # the GPU stored for dZ and H); the chain values above already tie those inputs to the oracle.
    dZ_gpu, H_gpu = host_bits(ffn.dGU), host_bits(ffn.H)
    g_gu = oracle.masked_decay(oracle.dense_dw(dZ_gpu, X).astype(np.float32), Wgu, mgu, wl.lam)
    g_d = oracle.masked_decay(oracle.dense_dw(dY, H_gpu).astype(np.float32), t["Wd"], md, wl.lam)
    assert_close(host_f64(ffn.w["Wgu"].grad), g_gu, F32_TOL, "geglu grad Wgu")
    assert_close(host_f64(ffn.w["Wd"].grad), g_d, F32_TOL, "geglu grad Wd")
    assert_close(host_f64(ffn.bias_grad["Wgu"]), oracle.bias_grad(dZ_gpu), F32_TOL, "geglu bias grad gu")
    assert_close(host_f64(ffn.bias_grad["Wd"]), oracle.bias_grad(dY), F32_TOL, "geglu bias grad d")


# ------------------------------------------------------------------ full-size workloads
def sample_rows(n, k, seed):
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=k)]))
    return rows.astype(np.int64)


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_workload_full_size(s24, name):
    wl = si.WORKLOADS[name]
    t = si.make(wl)
    p, d, f = wl.p, wl.d_model, wl.d_ff
    X, dY = t["X"], t["dY"]
    Xd, dYd = dev_bf16(X), dev_bf16(dY)
    up = wl.weight_names[0]
    down = wl.weight_names[-1]
    comp = {}
    # --- mask + compress over every weight, bit-exact
    for n in wl.weight_names:
        W = t[n]
        r, q = W.shape
        Wd = dev_bf16(W)
        vals = torch.zeros((q // 64, r, 32), dtype=torch.bfloat16, device="cuda")
        meta = torch.zeros((q // 64, r, 4), dtype=torch.int16, device="cuda")
        valsT = torch.zeros((r // 64, q, 32), dtype=torch.bfloat16, device="cuda")
        metaT = torch.zeros((r // 64, q, 4), dtype=torch.int16, device="cuda")
        mask = torch.zeros((r // 4, q // 4), dtype=torch.int16, device="cuda")
        mask2 = torch.zeros_like(mask)
        s24.compress(Wd, None, vals, meta, valsT, metaT, mask_out=mask)
        s24.transposable_mask(Wd, mask2, None)
        torch.cuda.synchronize()
        want_mask = oracle.transposable_mask(W)
        assert np.array_equal(host_bits(mask), want_mask), f"{name} {n} fused mask"
        assert np.array_equal(host_bits(mask2), want_mask), f"{name} {n} mask"
        want = oracle.compress(W, want_mask)
        want_packed = oracle.pack(want[0], want[1]) + oracle.pack(want[2], want[3])
        for got, ref, what in zip((vals, meta, valsT, metaT), want_packed, ("vals", "meta", "valsT", "metaT")):
            assert np.array_equal(host_bits(got), ref), f"{name} {n} {what}"
        del want_packed
        # masked decay on a sampled band of rows (the kernel runs over the whole matrix)
        G = torch.zeros((r, q), dtype=torch.float32, device="cuda")
        s24.masked_decay_grad(G, Wd, mask, wl.lam)
        torch.cuda.synchronize()
        r0 = (r // 3) // 4 * 4
        band = slice(r0, r0 + 64)
        ref = oracle.masked_decay(np.zeros((64, q), np.float32), np.ascontiguousarray(W[band]),
                                  np.ascontiguousarray(want_mask[r0 // 4:r0 // 4 + 16]), wl.lam)
        got = host_bits(G[band])
        np.testing.assert_allclose(got.astype(np.float64), ref, rtol=3e-7, atol=0)
        assert (got[keep_of(want_mask[r0 // 4:r0 // 4 + 16])] == 0).all()
        comp[n] = (want, (vals, meta, valsT, metaT))
        del Wd, G
    # --- forward sparse GEMM, up projection: sampled token rows
    rows = sample_rows(p, 24, 1)
    (ovals, ometa, ovalsT, ometaT), (vals, meta, valsT, metaT) = comp[up]
    Z = torch.zeros((p, f), dtype=torch.bfloat16, device="cuda")
    s24.spmm_fwd(Xd, vals, meta, Z)
    torch.cuda.synchronize()
    assert_close(host_f64(Z[torch.from_numpy(rows).cuda()]), oracle.spmm_fwd(X, ovals, ometa, rows=rows), BF16_TOL,
                 f"{name} spmm_fwd")
    # --- backward sparse GEMM through the up projection: dX = dZ . W, synthetic dZ
    dZ = si.random_matrix(900 + wl.seed, (p, f), 1e-2, "bf16")
    dZd = dev_bf16(dZ)
    dX = torch.zeros((p, d), dtype=torch.bfloat16, device="cuda")
    s24.spmm_bwd_dx(dZd, valsT, metaT, dX)
    torch.cuda.synchronize()
    assert_close(host_f64(dX[torch.from_numpy(rows).cuda()]), oracle.spmm_bwd_dx(dZ, ovalsT, ometaT, rows=rows),
                 BF16_TOL, f"{name} spmm_bwd_dx")
    # --- dense weight gradient dW = dZ^T X and dense comparison GEMM: sampled output rows
    orow = sample_rows(f, 6, 2)
    dW = torch.zeros((f, d), dtype=torch.float32, device="cuda")
    s24.dense_dw(dZd, Xd, dW)
    torch.cuda.synchronize()
    assert_close(host_f64(dW[torch.from_numpy(orow).cuda()]), oracle.dense_dw(dZ, X, rows=orow), F32_TOL,
                 f"{name} dense_dw")
    del dW
    s24.dense_gemm(Xd, dev_bf16(t[up]), Z)
    torch.cuda.synchronize()
    assert_close(host_f64(Z[torch.from_numpy(rows).cuda()]), oracle.dense_gemm(X, t[up], rows=rows), BF16_TOL,
                 f"{name} dense_gemm")
    # --- down projection forward (contraction over d_ff) on synthetic H
    Hh = si.random_matrix(901 + wl.seed, (p, f), 0.5, "bf16")
    (ovals, ometa, _, _), (vals, meta, _, _) = comp[down]
    Y = torch.zeros((p, d), dtype=torch.bfloat16, device="cuda")
    Hd = dev_bf16(Hh)
    s24.spmm_fwd(Hd, vals, meta, Y)
    torch.cuda.synchronize()
    assert_close(host_f64(Y[torch.from_numpy(rows).cuda()]), oracle.spmm_fwd(Hh, ovals, ometa, rows=rows), BF16_TOL,
                 f"{name} spmm_fwd down")
    # --- activation on the full buffers, compared on sampled rows
    band = sample_rows(p, 48, 3)
    bidx = torch.from_numpy(band).cuda()
    if wl.gated:
        Uh = si.random_matrix(902 + wl.seed, (p, f), 1.0, "bf16")
        Ud = dev_bf16(Uh)
        out, dG, dU = torch.zeros_like(Hd), torch.zeros_like(Hd), torch.zeros_like(Hd)
        s24.swiglu_fwd(Hd, Ud, out)
        s24.swiglu_bwd(dZd, Hd, Ud, dG, dU)
        torch.cuda.synchronize()
        g, u, dd = Hh[band], Uh[band], dZ[band]
        assert_close(host_f64(out[bidx]), oracle.swiglu_fwd(g, u), BF16_TOL, f"{name} swiglu_fwd")
        rg, ru = oracle.swiglu_bwd(dd, g, u)
        assert_close(host_f64(dG[bidx]), rg, BF16_TOL, f"{name} swiglu_bwd dG")
        assert_close(host_f64(dU[bidx]), ru, BF16_TOL, f"{name} swiglu_bwd dU")
    else:
        out, dz = torch.zeros_like(Hd), torch.zeros_like(Hd)
        s24.act_fwd(Hd, out, s24.ACT_GELU_ERF)
        s24.act_bwd(dZd, Hd, dz, s24.ACT_GELU_ERF)
        torch.cuda.synchronize()
        assert_close(host_f64(out[bidx]), oracle.act_fwd(Hh[band], oracle.ACT_GELU_ERF), BF16_TOL, f"{name} gelu fwd")
        assert_close(host_f64(dz[bidx]), oracle.act_bwd(dZ[band], Hh[band], oracle.ACT_GELU_ERF), BF16_TOL,
                     f"{name} gelu bwd")


def aligned_row_groups(n, k, seed):
    """Rows of k + 2 aligned groups of four (the first, the last and k random ones): the mask is per 4x4 block."""
    rng = np.random.default_rng(seed)
    g = np.unique(np.concatenate([[0, n // 4 - 1], rng.integers(0, n // 4, size=k)]))
    return (4 * g[:, None] + np.arange(4)[None, :]).reshape(-1).astype(np.int64)


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_default_step_full_size_against_the_oracle_chain(s24, name):
    """The step exactly as bench.py times it -- gate and up projection as one stacked weight, the activation and its
    backward inside the GEMM epilogues, all weight gradients in one batched pass with the decay in its epilogue -- at
    the workload's full size.  Every stage but the weight gradient is local to a token, so the oracle runs the whole
    chain (Eq. 2, Sec. 5.2, Eq. 3) on sampled token rows, rounding to the storage type where the kernels do, and each
    stage is also checked against the oracle applied to what the GPU itself stored as that stage's input (the bar of
    a single kernel).  Weight gradients (Eq. 1 + Eq. 10): sampled output rows from the GPU-stored operands."""
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.WORKLOADS[name]
    t = si.make(wl)
    p, d, f = wl.p, wl.d_model, wl.d_ff
    X, dY = t["X"], t["dY"]
    ffn = SparseFFN({n: dev_bf16(t[n]) for n in wl.weight_names}, p, wl.act, wl.lam, concat_gate_up=True)
    assert ffn.concat == wl.gated and ffn.fuse_swiglu and ffn.fuse_decay and ffn.batch_dw     # bench.py's defaults
    Xd, dYd = dev_bf16(X), dev_bf16(dY)
    ffn.step(Xd, dYd)
    torch.cuda.synchronize()
    if wl.gated:
        assert ffn.fuse_gate_bwd is True, "the large layers must take the fused backward epilogue"
        host_w = {"Wgu": np.concatenate([t["Wg"], t["Wu"]], axis=0), "Wd": t["Wd"]}
        up, down = "Wgu", "Wd"
    else:
        host_w = {"W1": t["W1"], "W2": t["W2"]}
        up, down = "W1", "W2"
    comp, masks = {}, {}
    for n, W in host_w.items():
        masks[n] = oracle.transposable_mask(W)
        assert np.array_equal(host_bits(ffn.w[n].mask), masks[n]), f"{name} {n} mask"
        comp[n] = oracle.compress(W, masks[n])
        packed = oracle.pack(comp[n][0], comp[n][1]) + oracle.pack(comp[n][2], comp[n][3])
        for got, ref, what in zip((ffn.w[n].vals, ffn.w[n].meta, ffn.w[n].valsT, ffn.w[n].metaT), packed,
                                  ("vals", "meta", "valsT", "metaT")):
            assert np.array_equal(host_bits(got), ref), f"{name} {n} {what}"
        del packed
    rows = sample_rows(p, 24, 5)
    ridx = torch.from_numpy(rows).cuda()
    Xs, dYs = np.ascontiguousarray(X[rows]), np.ascontiguousarray(dY[rows])
    rnd = lambda a: oracle.round_like(a, X)
    wide = lambda a: si.to_f32(a).astype(np.float64)
    got = lambda tens: host_f64(tens[ridx])
    gbits = lambda tens: host_bits(tens[ridx].contiguous())
    def assert_chain(gotv, ref, what):
        """The chained comparison.  A bf16 rounding that falls the other way upstream (GPU fp32 accumulation against
        the oracle's fp64) moves that operand by 2^-8 of itself, and a contraction over thousands of such operands
        then moves every output by some 1e-3 of the output's rms, whatever the output's own size: the element
        bound of a chain is taken relative to max(|ref|, rms) (a single kernel's bar, relative to max(|ref|,
        1e-2 rms), is applied below to each stage on the GPU's own stored input).  The normwise bound is the bar's."""
        gotv, ref = np.asarray(gotv, dtype=np.float64), np.asarray(ref, dtype=np.float64)
        assert np.isfinite(gotv).all(), what
        rms = np.sqrt(np.mean(ref * ref))
        e_max = (np.abs(gotv - ref) / np.maximum(np.abs(ref), rms)).max()
        e_nrm = np.linalg.norm(gotv - ref) / np.linalg.norm(ref)
        assert e_max <= 2e-2 and e_nrm <= BF16_TOL[1], f"{what}: max {e_max:.3e} of max(|ref|, rms), normwise {e_nrm:.3e}"
    if wl.gated:
        gate = oracle.GATE_SILU
        Z = rnd(oracle.spmm_fwd(Xs, comp[up][0], comp[up][1]))
        H = rnd(oracle.glu_fwd(Z, gate))
        Y = oracle.spmm_fwd(H, comp[down][0], comp[down][1])
        dH = rnd(oracle.spmm_bwd_dx(dYs, comp[down][2], comp[down][3]))
        dZ = rnd(oracle.glu_bwd(dH, Z, gate))
        dXr = oracle.spmm_bwd_dx(dZ, comp[up][2], comp[up][3])
        assert_close(got(ffn.GU), wide(Z), BF16_TOL, f"{name} GU")            # first stage: single-kernel bar
        assert_chain(got(ffn.H), wide(H), f"{name} H (chain)")
        assert_chain(got(ffn.Y), Y, f"{name} Y (chain)")
        assert_chain(got(ffn.dGU), wide(dZ), f"{name} dGU (chain)")
        assert_chain(got(ffn.dX), dXr, f"{name} dX (chain)")
        # each later stage on the GPU's own stored input
        GUg, Hg, dGUg = gbits(ffn.GU), gbits(ffn.H), gbits(ffn.dGU)
        assert_close(got(ffn.H), oracle.glu_fwd(GUg, gate), BF16_TOL, f"{name} H")
        assert_close(got(ffn.Y), oracle.spmm_fwd(Hg, comp[down][0], comp[down][1]), BF16_TOL, f"{name} Y")
        # the fused backward epilogue never stores dH: the plain input-gradient GEMM (whose bits the fused kernel
        # reproduces) gives the GPU's own dH for the single-kernel bar of the activation backward
        s24.spmm_bwd_dx(dYd, ffn.w[down].valsT, ffn.w[down].metaT, ffn.dH)
        torch.cuda.synchronize()
        assert_close(got(ffn.dH), wide(dH), BF16_TOL, f"{name} dH")
        assert_close(got(ffn.dGU), oracle.glu_bwd(gbits(ffn.dH), GUg, gate), BF16_TOL, f"{name} dGU")
        assert_close(got(ffn.dX), oracle.spmm_bwd_dx(dGUg, comp[up][2], comp[up][3]), BF16_TOL, f"{name} dX")
        ops = {"Wd": (dY, host_bits(ffn.H), dYd, ffn.H), "Wgu": (host_bits(ffn.dGU), X, ffn.dGU, Xd)}
    else:
        act = oracle.ACT_GELU_ERF
        Z = rnd(oracle.spmm_fwd(Xs, comp[up][0], comp[up][1]))
        H = rnd(oracle.act_fwd(Z, act))
        Y = oracle.spmm_fwd(H, comp[down][0], comp[down][1])
        dH = rnd(oracle.spmm_bwd_dx(dYs, comp[down][2], comp[down][3]))
        dZ = rnd(oracle.act_bwd(dH, Z, act))
        dXr = oracle.spmm_bwd_dx(dZ, comp[up][2], comp[up][3])
        assert_close(got(ffn.Z), wide(Z), BF16_TOL, f"{name} Z")
        assert_chain(got(ffn.H), wide(H), f"{name} H (chain)")
        assert_chain(got(ffn.Y), Y, f"{name} Y (chain)")
        assert_chain(got(ffn.dZ), wide(dZ), f"{name} dZ (chain)")
        assert_chain(got(ffn.dX), dXr, f"{name} dX (chain)")
        Zg, Hg, dZg = gbits(ffn.Z), gbits(ffn.H), gbits(ffn.dZ)
        assert_close(got(ffn.H), oracle.act_fwd(Zg, act), BF16_TOL, f"{name} H")
        assert_close(got(ffn.Y), oracle.spmm_fwd(Hg, comp[down][0], comp[down][1]), BF16_TOL, f"{name} Y")
        s24.spmm_bwd_dx(dYd, ffn.w[down].valsT, ffn.w[down].metaT, ffn.dH)
        torch.cuda.synchronize()
        assert_close(got(ffn.dH), wide(dH), BF16_TOL, f"{name} dH")
        assert_close(got(ffn.dZ), oracle.act_bwd(gbits(ffn.dH), Zg, act), BF16_TOL, f"{name} dZ")
        assert_close(got(ffn.dX), oracle.spmm_bwd_dx(dZg, comp[up][2], comp[up][3]), BF16_TOL, f"{name} dX")
        ops = {"W2": (dY, host_bits(ffn.H), dYd, ffn.H), "W1": (host_bits(ffn.dZ), X, ffn.dZ, Xd)}
    del comp
    # Weight gradients with the decay term (Eq. 1 + Eq. 10) on aligned groups of output rows.  At these sizes the decay
    # term (lambda |w| of some 4e-6) is smaller than the fp32 accumulation noise of a sum over thousands of tokens, so a
    # tolerance comparison alone would not see it: the batched, decay-fused result is compared (a) with the oracle's
    # dense_dw + masked_decay of the GPU-stored operands within the fp32 tolerance and (b) cell by cell with the
    # oracle's Eq. 10 applied to the plain weight-gradient GEMM's own output for the same operands (kept cells bit
    # for bit, pruned cells to an fp32 rounding), that GEMM in turn being held to the oracle's.
    for n, (a, b, a_dev, b_dev) in ops.items():
        W, r = host_w[n], host_w[n].shape[0]
        orow = aligned_row_groups(r, 6, 11 + len(n))
        oidx = torch.from_numpy(orow).cuda()
        dWr = oracle.dense_dw(a, b, rows=orow)
        Wrows, mrows = np.ascontiguousarray(W[orow]), np.ascontiguousarray(masks[n][orow[::4] // 4])
        want = oracle.masked_decay(dWr.astype(np.float32), Wrows, mrows, wl.lam)
        gotg = host_bits(ffn.w[n].grad[oidx])
        assert_close(gotg.astype(np.float64), want, F32_TOL, f"{name} grad {n}")
        plain = torch.empty_like(ffn.w[n].grad)
        s24.dense_dw(a_dev, b_dev, plain)
        torch.cuda.synchronize()
        plain_rows = host_bits(plain[oidx])
        del plain
        assert_close(plain_rows.astype(np.float64), dWr, F32_TOL, f"{name} plain dW {n}")
        cell = oracle.masked_decay(plain_rows, Wrows, mrows, wl.lam)
        keep = keep_of(mrows)
        assert np.array_equal(gotg[keep], plain_rows[keep]), f"{name} grad {n}: kept cells"
        np.testing.assert_allclose(gotg[~keep].astype(np.float64), cell[~keep], rtol=3e-7, atol=0)
        assert (gotg[~keep] != plain_rows[~keep]).mean() > 0.5, f"{name} grad {n}: the decay term is missing"


def test_step_replayed_from_a_hip_graph_matches_eager_launches():
    """The captured step is replayed several times with eager work and synchronisations in between;
    every replay must reproduce the eager results bit for bit (the kernels are deterministic)."""
    import torch
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.Workload("g", 768, 256, 512, "swiglu", "bf16", 11)
    host = si.make(wl)
    d = {k: dev_bf16(v) for k, v in host.items()}
    ffn = SparseFFN({n: d[n] for n in wl.weight_names}, wl.p, wl.act, wl.lam)
    X, dY = d["X"], d["dY"]

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (ffn.Y, ffn.dX, ffn.H, *(w.grad for w in ffn.w.values()),
                                    *(w.mask for w in ffn.w.values()), *(w.valsT for w in ffn.w.values()))]

    ffn.step(X, dY)
    want = snapshot()
    graph = ffn.capture(X, dY)
    for replay in range(3):
        for t in (ffn.Y, ffn.dX, ffn.H, *(w.grad for w in ffn.w.values())):
            t.zero_()                      # eager work between replays; also proves the replay rewrites everything
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(want, got):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b), f"replay {replay} differs"
        ffn.step(X, dY)                    # an eager step between replays


def test_mask_interval_keeps_the_mask_and_recompresses_the_new_weights():
    """Between two mask searches the stored mask is applied to the updated weights (prune + compress every
    step, search every l-th step): checked against the oracle's compress of the new weights under the old mask."""
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.Workload("i", 256, 128, 256, "gelu", "bf16", 12)
    host = si.make(wl)
    d = {k: dev_bf16(v) for k, v in host.items()}
    ffn = SparseFFN({n: d[n] for n in wl.weight_names}, wl.p, wl.act, wl.lam, mask_interval=3)
    ffn.step(d["X"], d["dY"])
    torch.cuda.synchronize()
    mask0 = {n: host_bits(w.mask).copy() for n, w in ffn.w.items()}
    for n in wl.weight_names:
        assert np.array_equal(mask0[n], oracle.transposable_mask(host[n]))
    # new weights (another seed), same buffers
    new = {n: si.random_matrix(900 + i, host[n].shape, 0.02, "bf16") for i, n in enumerate(wl.weight_names)}
    for n in wl.weight_names:
        ffn.w[n].W.copy_(dev_bf16(new[n]))
    ffn.step(d["X"], d["dY"])          # step 1: no search
    torch.cuda.synchronize()
    for n, w in ffn.w.items():
        assert np.array_equal(host_bits(w.mask), mask0[n])
        vals, meta, valsT, metaT = oracle.compress(new[n], mask0[n])
        vp, mp = oracle.pack(vals, meta)
        vtp, mtp = oracle.pack(valsT, metaT)
        assert np.array_equal(host_bits(w.vals), vp) and np.array_equal(host_bits(w.meta), mp)
        assert np.array_equal(host_bits(w.valsT), vtp) and np.array_equal(host_bits(w.metaT), mtp)
    ffn.step(d["X"], d["dY"])          # step 2: no search
    ffn.step(d["X"], d["dY"])          # step 3: search again, now on the new weights
    torch.cuda.synchronize()
    for n, w in ffn.w.items():
        assert np.array_equal(host_bits(w.mask), oracle.transposable_mask(new[n]))


def test_captured_step_keeps_the_mask_schedule():
    """A captured layer with mask_interval = 3 must search on the same steps as the eager layer does: two layers on
    copies of the same weights, one stepped eagerly and one replayed, the weights rewritten before every step; masks,
    compressed operands and outputs agree bit for bit after each of seven steps (replays 3 and 6 search)."""
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.Workload("s", 256, 128, 256, "swiglu", "bf16", 21)
    host = si.make(wl)
    d = {k: dev_bf16(v) for k, v in host.items()}
    mk = lambda: SparseFFN({n: d[n].clone() for n in wl.weight_names}, wl.p, wl.act, wl.lam, mask_interval=3,
                           concat_gate_up=True)
    eager, replayed = mk(), mk()
    X, dY = d["X"], d["dY"]
    graph = replayed.capture(X, dY)          # runs step 0 (with the search) for real
    eager.step(X, dY)
    searched = []
    for step in range(1, 8):
        new = {n: dev_bf16(si.random_matrix(2100 + 10 * step + i, tuple(w.W.shape), 0.02, "bf16"))
               for i, (n, w) in enumerate(eager.w.items())}
        before = {n: w.mask.clone() for n, w in replayed.w.items()}
        for ffn in (eager, replayed):
            for n, w in ffn.w.items():
                w.W.copy_(new[n])
        eager.step(X, dY)
        graph.replay()
        torch.cuda.synchronize()
        searched.append(any(not torch.equal(before[n], w.mask) for n, w in replayed.w.items()))
        for n in eager.w:
            a, b = eager.w[n], replayed.w[n]
            assert torch.equal(a.mask, b.mask), (step, n)
            assert torch.equal(a.vals.view(torch.int16), b.vals.view(torch.int16)) and torch.equal(a.metaT, b.metaT), (step, n)
            assert torch.equal(a.grad, b.grad), (step, n)
        assert torch.equal(eager.Y.view(torch.int16), replayed.Y.view(torch.int16)), step
        assert torch.equal(eager.dX.view(torch.int16), replayed.dX.view(torch.int16)), step
    assert searched == [False, False, True, False, False, True, False]
    assert eager.steps_done == replayed.steps_done == 8


def test_gate_and_up_as_one_weight_matches_the_separate_weights():
    """One [2*d_ff, d_model] weight: forward results and weight gradients are bit-identical to the three-weight
    layout (same per-output arithmetic); dX sums the 2*d_ff contraction in one GEMM, so it agrees to tolerance."""
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.Workload("c", 640, 256, 448, "swiglu", "bf16", 13)
    host = si.make(wl)
    d = {k: dev_bf16(v) for k, v in host.items()}
    a = SparseFFN({n: d[n] for n in wl.weight_names}, wl.p, wl.act, wl.lam)
    b = SparseFFN({n: d[n] for n in wl.weight_names}, wl.p, wl.act, wl.lam, concat_gate_up=True)
    a.step(d["X"], d["dY"])
    b.step(d["X"], d["dY"])
    torch.cuda.synchronize()
    f = wl.d_ff
    bits = lambda t: t.contiguous().view(torch.int16)
    for x, y in ((a.G, b.G), (a.U, b.U), (a.H, b.H), (a.Y, b.Y), (a.dH, b.dH), (a.dG, b.dG), (a.dU, b.dU)):
        assert torch.equal(bits(x), bits(y))
    assert torch.equal(a.w["Wg"].grad, b.w["Wgu"].grad[:f]) and torch.equal(a.w["Wu"].grad, b.w["Wgu"].grad[f:])
    assert torch.equal(a.w["Wd"].grad, b.w["Wd"].grad)
    assert torch.equal(a.w["Wg"].mask, b.w["Wgu"].mask[:f // 4]) and torch.equal(a.w["Wu"].mask, b.w["Wgu"].mask[f // 4:])
    # both routes round to bf16 (the two-GEMM route twice), so they differ by bf16 roundings of partial sums:
    # normwise agreement, and no element further apart than a few bf16 steps at the scale of the larger sums
    x, y = host_f64(a.dX), host_f64(b.dX)
    assert np.linalg.norm(x - y) <= BF16_TOL[1] * np.linalg.norm(x)
    assert np.abs(x - y).max() <= 2.0 ** -6 * np.abs(x).max()


def test_step_with_the_sparse_weight_gradient():
    """Eq. 4 mode of the layer: every weight gradient is S_z(dY^T) X (+ decay) for the draw the layer made.
    The GPU's pruned operand is compared bit for bit with the oracle's for the same seed, on an input that
    comes from the seeded generator (dY of the down projection), and its gradient with the oracle's GEMM."""
    from paper_2404_01847_amd.ffn import SparseFFN
    wl = si.Workload("m", 256, 128, 256, "gelu", "bf16", 14)
    host = si.make(wl)
    d = {k: dev_bf16(v) for k, v in host.items()}
    ffn = SparseFFN({n: d[n] for n in wl.weight_names}, wl.p, wl.act, wl.lam, mvue=True, seed=1000)
    ffn.step(d["X"], d["dY"])
    torch.cuda.synchronize()
    # first pruned operand of the step: dY for W2 (seed + 1)
    w2 = ffn.w["W2"]
    vz, mz = oracle.mvue24(host["dY"], 1001)
    vp, mp = oracle.pack(vz, mz)
    assert np.array_equal(host_bits(w2.zmeta), mp) and np.array_equal(host_bits(w2.zvals), vp)
    # its gradient: S_z(dY^T) H + decay, with H as the GPU computed it upstream fed to nothing but the comparison of
    # shapes; the oracle side uses its own chain for H
    mask1 = oracle.transposable_mask(host["W1"])
    c1 = oracle.compress(host["W1"], mask1)
    Z = oracle.round_bf16(oracle.spmm_fwd(host["X"], c1[0], c1[1]))
    H = oracle.round_bf16(oracle.act_fwd(Z, oracle.ACT_GELU_ERF))
    mask2 = oracle.transposable_mask(host["W2"])
    ref = oracle.spmm_fwd(np.ascontiguousarray(H.T), vz, mz).T
    ref = ref + oracle.masked_decay(np.zeros(host["W2"].shape, np.float32), host["W2"], mask2, wl.lam)
    assert_close(host_f64(w2.grad), ref, (2e-2, 5e-3), "W2 gradient from the pruned dY")
    with pytest.raises(RuntimeError):
        ffn.capture(d["X"], d["dY"])
