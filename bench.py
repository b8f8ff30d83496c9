#!/usr/bin/env python3
"""Benchmark of the 2:4-sparse FFN training step on one MI355X.

One step = the whole hot path once on one batch of synthetic input already
resident in HBM: per weight the transposable mask search fused with
prune/compress, the sparse forward GEMMs, the activation, the sparse
input-gradient GEMMs, the dense weight-gradient GEMMs and the masked decay.

    python bench.py [--workload c5] [--also c1,c2,c3,c4] [--steps K] [--warmup W]

Prints ONE JSON line.  `value` is the dense-equivalent GEMM TFLOP/s of the whole
step (all 6 or 9 GEMMs' 2*p*d*d_ff FLOPs divided by the wall time of the step,
mask/compress/activation/decay included).  `roofline` describes the kernel that
takes the largest share of the step; `kernels` lists every kernel with its own
roofline fraction; `cpu_baseline` is the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_DENSE_BF16 = 2500.0      # TFLOP/s, dense bf16 MFMA
PEAK_SPARSE_BF16 = 5000.0     # TFLOP/s, 2:4 structured-sparse bf16 (dense-equivalent FLOPs)
PEAK_HBM = 8000.0             # GB/s

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.md")


def measured_traffic(workload, kernel):
    """HBM-side bytes (read + written) per call of the entry point in the default configuration of `workload`, from the
    tracked summary of the rocprofv3 PMC runs of this file (FETCH_SIZE and WRITE_SIZE, each scaled by what the same
    counter reads for a device copy of known size): the rows `| workload | kernel | read bytes | written bytes |` of
    profiles/hbm_traffic_pmc.md.  None when the table has no such row (nothing is assumed)."""
    try:
        with open(TRAFFIC_TABLE) as fh:
            for line in fh:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 4 and cells[0] == workload and cells[1] == kernel:
                    return float(cells[2]) + float(cells[3])
    except (OSError, ValueError):
        pass
    return None


def kernel_model(wl):
    """Algorithmic work of each kernel over one whole step: (kind, amount per step, peak, unit).  Per step and not
    per launch because the launches of one kernel differ in size when gate and up projection are one weight."""
    p, d, f = wl.p, wl.d_model, wl.d_ff
    es = 4 if wl.dtype == "f32" else 2
    nw = len(wl.weight_names)
    blocks = nw * d * f / 16
    gemm = nw * 2.0 * p * d * f
    m = {
        "spmm_fwd": ("mfma", gemm, PEAK_SPARSE_BF16, "TFLOP/s"),
        "spmm_bwd_dx": ("mfma", gemm, PEAK_SPARSE_BF16, "TFLOP/s"),
        "dense_dw": ("mfma", gemm, PEAK_DENSE_BF16, "TFLOP/s"),
        # Eq. 4 mode: the pruned output gradients (p x d_ff for every up-type weight, p x d for the down one):
        # read es per element, write es/2 + 1/8; then the weight gradient as a sparse GEMM
        "mvue24": ("hbm", ((nw - 1) * p * f + p * d) * (es + es / 2 + 0.125), PEAK_HBM, "GB/s"),
        "spmm_dw": ("mfma", gemm, PEAK_SPARSE_BF16, "TFLOP/s"),
        # per 4x4 block: read 16 weights; write mask 2, vals 16*es/2, meta 2, valsT 16*es/2, metaT 2
        "mask_compress": ("hbm", blocks * (16 * es + 2 + 8 * es + 2 + 8 * es + 2), PEAK_HBM, "GB/s"),
        # with a given mask: read 16 weights + mask 2; write vals, meta, valsT, metaT
        "compress": ("hbm", blocks * (16 * es + 2 + 8 * es + 2 + 8 * es + 2), PEAK_HBM, "GB/s"),
        # per element: read dW 4 + W es + mask 1/8, write 4
        "masked_decay": ("hbm", nw * d * f * (8 + es + 0.125), PEAK_HBM, "GB/s"),
        "swiglu_fwd": ("hbm", p * f * 3 * es, PEAK_HBM, "GB/s"),
        "swiglu_bwd": ("hbm", p * f * 5 * es, PEAK_HBM, "GB/s"),
        "act_fwd": ("hbm", p * f * 2 * es, PEAK_HBM, "GB/s"),
        "act_bwd": ("hbm", p * f * 3 * es, PEAK_HBM, "GB/s"),
        # bias gradients (only with --geglu-bias): every output gradient read once
        "bias_grad": ("hbm", ((nw - 1) * p * f + p * d) * es, PEAK_HBM, "GB/s"),
    }
    return m


def cpu_baseline(wl, tensors_host, budget_tokens=None):
    """The oracle, as it stands, on a bounded sample of the same workload: every weight-side stage (mask, compress,
    decay) at full size, every token-side stage (GEMMs, activation) on the first `budget_tokens` tokens against the
    full weights, extrapolated linearly in the token count.  Returns dense-equivalent TFLOP/s of the whole step."""
    import numpy as np
    import oracle
    t = tensors_host
    if budget_tokens is None:
        # some 5 s of oracle GEMM work on 16 host threads (6 d d_ff FLOPs per token and weight, about 40 GFLOP/s in
        # fp64): the token sample shrinks with the layer's size
        budget_tokens = max(16, min(wl.p, int(2.0e11 / (6.0 * len(wl.weight_names) * wl.d_model * wl.d_ff))))
    n = min(budget_tokens, wl.p)
    X, dY = np.ascontiguousarray(t["X"][:n]), np.ascontiguousarray(t["dY"][:n])
    t0 = time.perf_counter()
    comp = {}
    for name in wl.weight_names:
        m = oracle.transposable_mask(t[name])
        comp[name] = (m,) + oracle.compress(t[name], m)
    for name in wl.weight_names:
        r, q = t[name].shape
        oracle.masked_decay(np.zeros((r, q), np.float32), t[name], comp[name][0], wl.lam)
    t_weights = time.perf_counter() - t0
    rnd = lambda a: oracle.round_like(a, X)
    t0 = time.perf_counter()
    if wl.gated:
        G = rnd(oracle.spmm_fwd(X, comp["Wg"][1], comp["Wg"][2]))
        U = rnd(oracle.spmm_fwd(X, comp["Wu"][1], comp["Wu"][2]))
        gate = oracle.GATE_GELU_ERF if wl.act == "geglu" else oracle.GATE_SILU
        Z = np.concatenate([G, U], axis=1)
        H = rnd(oracle.glu_fwd(Z, gate))
        oracle.spmm_fwd(H, comp["Wd"][1], comp["Wd"][2])
        dH = rnd(oracle.spmm_bwd_dx(dY, comp["Wd"][3], comp["Wd"][4]))
        dZ = rnd(oracle.glu_bwd(dH, Z, gate))
        dG, dU = np.ascontiguousarray(dZ[:, :wl.d_ff]), np.ascontiguousarray(dZ[:, wl.d_ff:])
        oracle.spmm_bwd_dx(dG, comp["Wg"][3], comp["Wg"][4])
        oracle.spmm_bwd_dx(dU, comp["Wu"][3], comp["Wu"][4])
        oracle.dense_dw(dY, H)
        oracle.dense_dw(dG, X)
        oracle.dense_dw(dU, X)
    else:
        act = oracle.ACT_RELU if wl.act == "relu" else oracle.ACT_GELU_ERF
        Z = rnd(oracle.spmm_fwd(X, comp["W1"][1], comp["W1"][2]))
        H = rnd(oracle.act_fwd(Z, act))
        oracle.spmm_fwd(H, comp["W2"][1], comp["W2"][2])
        dH = rnd(oracle.spmm_bwd_dx(dY, comp["W2"][3], comp["W2"][4]))
        dZ = rnd(oracle.act_bwd(dH, Z, act))
        oracle.spmm_bwd_dx(dZ, comp["W1"][3], comp["W1"][4])
        oracle.dense_dw(dY, H)
        oracle.dense_dw(dZ, X)
    t_tokens = time.perf_counter() - t0
    est = t_weights + t_tokens * (wl.p / n)
    return {
        "value": wl.gemm_flops / est / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": (f"mask+compress+decay of all {len(wl.weight_names)} weights at full size ({t_weights:.1f} s); GEMMs and "
                   f"activation on the first {n} of {wl.p} tokens ({t_tokens:.1f} s), extrapolated linearly in tokens "
                   f"to {est:.0f} s per step"),
    }


def _time_ms(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


INFINITY_CACHE_BYTES = 256e6   # the memory-side cache in front of HBM


def _rotation(working_set_bytes):
    """How many distinct sets of buffers a repeated measurement of an HBM-bound kernel cycles through so that a
    set has left the Infinity Cache before its turn comes again (the sets together are over twice its size)."""
    return int(2 * INFINITY_CACHE_BYTES // working_set_bytes) + 2


def _in_turn(calls):
    """A function that makes the next of `calls` each time it is called."""
    state = {"i": 0}

    def fn():
        calls[state["i"] % len(calls)]()
        state["i"] += 1
    return fn


def _clock_mhz(torch, s24, fn, reps=6):
    """Core clock the chip holds under `fn` (a large-tile GEMM launch): the library's clock probe makes
    workgroup 0 of the last launch report core cycles and 100 MHz reference ticks over its lifetime."""
    buf = torch.zeros(2, dtype=torch.int64, device="cuda")
    s24.set_clock_probe(buf)
    try:
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
    finally:
        s24.set_clock_probe(None)
        torch.cuda.synchronize()
    cycles, ticks = (int(v) for v in buf.tolist())
    return round(100.0 * cycles / ticks, 0) if ticks > 0 else None


def _capture(torch, fn):
    """fn (kernel launches on the current stream only, no allocation) recorded into a HIP graph."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    return graph


def c3_mask_sweep(torch, s24, wl):
    """The mask search over all weights of a GPT-2-large-sized model (36 layers x 2 matrices of the c3 layer's shapes,
    944 MB: more than the 256 MB Infinity Cache holds, so the rate is an HBM rate), one launch per matrix and stacked
    by shape into two launches."""
    import s24_inputs as si
    import numpy as np
    # the 72 matrices, stacked by shape the way a model can hold its layers' weights: [36*d_ff][d] and [36*d][d_ff]
    stacks = []
    for which in range(2):
        a = np.concatenate([si.sweep_weight(layer, which, wl) for layer in range(36)], axis=0)
        t = torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) if a.dtype == np.uint16 else torch.from_numpy(a).cuda()
        stacks.append((t, torch.empty((t.shape[0] // 4, t.shape[1] // 4), dtype=torch.int16, device="cuda")))
    rows = [wl.d_ff, wl.d_model]

    def sweep_per_matrix():
        for (t, m), r in zip(stacks, rows):
            for layer in range(36):
                s24.transposable_mask(t[layer * r:(layer + 1) * r], m[layer * r // 4:(layer + 1) * r // 4], None)

    def sweep_stacked():
        for t, m in stacks:
            s24.transposable_mask(t, m, None)

    ms72 = _time_ms(torch, sweep_per_matrix, 5)
    ms2 = _time_ms(torch, sweep_stacked, 5)
    nb72 = sum(t.numel() / 16 * 34 for t, _ in stacks)
    result = {
        "matrices": 72, "MB": round(sum(t.numel() * 2 for t, _ in stacks) / 1e6, 1),
        "one_launch_per_matrix": {"ms_per_sweep": round(ms72, 4), "GB/s": round(nb72 / ms72 / 1e6, 1),
                                  "frac_of_hbm_peak": round(nb72 / ms72 / 1e6 / PEAK_HBM, 4)},
        "one_launch_per_shape": {"ms_per_sweep": round(ms2, 4), "GB/s": round(nb72 / ms2 / 1e6, 1),
                                 "frac_of_hbm_peak": round(nb72 / ms2 / 1e6 / PEAK_HBM, 4)},
        "note": "13 MB matrices are 400 workgroups each, 1.6 per compute unit: a launch per matrix is bound by "
                "launch-to-launch latency, not by HBM; the same bytes in two launches show the kernel's rate"}
    del stacks
    return result


def side_measurements(torch, s24, wl, ffn, X, dY, weights):
    """Outside the timed step:
    (1) the mask search alone, over all weights of the layer in turn (34 algorithmic bytes per 4x4 bf16
        block: 32 read, 2 written); for c3 also over 72 distinct matrices of the layer's shape (36 layers x 2,
        944 MB, more than the 256 MB Infinity Cache holds) so that the rate is an HBM rate;
    (2) the dense-MFMA GEMM of the library next to the sparse GEMM at the layer's GEMM shapes (all three
        for c5, the up-projection otherwise);
    (3) the core clock under each large-tile GEMM kernel, and the clock-scaled matrix-core peak;
    (4) the step replayed from a HIP graph;
    (5) the step with the mask searched every 40th step only;
    (6) the flip-count and L1-norm-gap monitors;
    (7) the step with the sparse weight gradient on the MVUE-pruned output gradient."""
    import s24_inputs as si
    out = {}
    es = 4 if wl.dtype == "f32" else 2
    from paper_2404_01847_amd.ffn import SparseWeight
    # the layer's weights one by one (also where the timed step holds gate and up projection as one weight)
    named = {}
    for n in wl.weight_names:
        named[n] = SparseWeight(weights[n])
        named[n].refresh()
    ws = list(named.values())
    masks = [torch.empty_like(w.mask) for w in ws]

    def sweep():
        for w, m in zip(ws, masks):
            s24.transposable_mask(w.W, m, None)

    ms = _time_ms(torch, sweep, 10)
    nbytes = sum(w.W.numel() / 16 * (16 * es + 2) for w in ws)
    out["mask_search_only"] = {"ms_per_sweep": round(ms, 4), "matrices": len(ws), "GB/s": round(nbytes / ms / 1e6, 1),
                               "frac_of_hbm_peak": round(nbytes / ms / 1e6 / PEAK_HBM, 4),
                               "working_set_MB": round(nbytes / 1e6, 1),
                               "cache_resident": bool(nbytes < 2 * INFINITY_CACHE_BYTES)}
    if wl.name == "c3":
        out["mask_search_only_72_matrices"] = c3_mask_sweep(torch, s24, wl)
    # (6) the monitors of Sec. 4.1 / 4.2 on the first weight: flip count between two masks (4 bytes read per block,
    # one uint64 written) and L1-norm gap (32 bytes read + 8 written per bf16 block, 90 fp64 sums per block)
    w0 = ws[0]
    other = torch.roll(w0.mask, 1, 0).contiguous()
    flips = torch.zeros(1, dtype=torch.int64, device="cuda")
    ms_f = _time_ms(torch, lambda: s24.mask_flips(w0.mask, other, flips), 10)
    gap = torch.empty(w0.mask.shape, dtype=torch.float64, device="cuda")
    ms_g = _time_ms(torch, lambda: s24.l1_norm_gap(w0.W, gap), 5)
    nb = w0.mask.numel()
    out["monitors"] = {"buffers": "one weight, repeated: cache-resident when its bytes fit the 256 MB Infinity Cache",
                       "mask_flips": {"ms": round(ms_f, 4), "GB/s": round(nb * 4 / ms_f / 1e6, 1),
                                      "cache_resident": bool(nb * 4 < INFINITY_CACHE_BYTES)},
                       "l1_norm_gap": {"ms": round(ms_g, 4), "GB/s": round(nb * (16 * es + 8) / ms_g / 1e6, 1),
                                       "bound": "alu (90 x 16 fp64 select-adds per block)"}}
    # (7) the step with the weight gradient taken from the unbiasedly pruned output gradient (Eq. 4, Eq. 6)
    if not ffn.mvue:
        ffn.mvue = True
        ffn.timings = {}
        ms_m = _time_ms(torch, lambda: ffn.step(X, dY), 10)
        tm, ffn.timings, ffn.mvue = ffn.timings, None, False
        per = {k: round(sum(a.elapsed_time(b) for a, b in v) / 11, 4) for k, v in tm.items() if k in ("mvue24", "spmm_dw")}
        out["step_with_mvue_sparse_weight_gradient"] = {"ms_per_step": round(ms_m, 4), "TFLOP/s": round(wl.gemm_flops / ms_m / 1e9, 1),
                                                        "ms_per_step_by_kernel": per}
    # (4) the whole step replayed from one HIP graph: what the step costs once launch overhead is gone
    if not ffn.mvue:
        graph = ffn.capture(X, dY)
        ms_g = _time_ms(torch, graph.replay, 20)
        out["step_as_hip_graph"] = {"ms_per_step": round(ms_g, 4), "TFLOP/s": round(wl.gemm_flops / ms_g / 1e9, 1)}
        del graph
    # (5) the paper's schedule: the mask searched every 40th step, prune + compress with the stored mask on the
    # others (Sec. 5.1); 40 consecutive steps, one of them with the search
    ffn.mask_interval, ffn.steps_done = 40, 0
    ms_40 = _time_ms(torch, lambda: ffn.step(X, dY), 40)
    ffn.mask_interval, ffn.steps_done = 1, 0
    out["step_with_mask_every_40_steps"] = {"ms_per_step": round(ms_40, 4), "TFLOP/s": round(wl.gemm_flops / ms_40 / 1e9, 1)}
    out["gated_activation_sec_5_2"] = gated_activation_measurements(torch, s24)
    if wl.dtype != "f32":
        names = list(named) if wl.name == "c5" else list(named)[:1]
        cmp_ = []
        for name in names:
            w = named[name]
            r, q = w.W.shape
            A = X if q == X.shape[1] else torch.empty((wl.p, q), dtype=X.dtype, device=X.device).normal_()
            Yd = torch.empty((wl.p, r), dtype=X.dtype, device=X.device)
            flops = 2.0 * wl.p * q * r
            t_dense = _time_ms(torch, lambda: s24.dense_gemm(A, w.W, Yd), 5)
            t_sparse = _time_ms(torch, lambda: s24.spmm_fwd(A, w.vals, w.meta, Yd), 5)
            # context, not this library's code: the same dense GEMM through PyTorch's matmul (the vendor's GEMM library)
            t_vendor = _time_ms(torch, lambda: torch.matmul(A, w.W.t(), out=Yd), 5)
            cmp_.append({"weight": name, "shape_p_q_r": [wl.p, q, r],
                         "vendor_library_dense_ms": round(t_vendor, 4),
                         "vendor_library_dense_TFLOP/s": round(flops / t_vendor / 1e9, 1),
                         "speedup_over_vendor_library_dense": round(t_vendor / t_sparse, 3),
                         "dense_mfma_ms": round(t_dense, 4), "dense_mfma_TFLOP/s": round(flops / t_dense / 1e9, 1),
                         "sparse_smfmac_ms": round(t_sparse, 4),
                         "sparse_dense_equiv_TFLOP/s": round(flops / t_sparse / 1e9, 1),
                         "speedup": round(t_dense / t_sparse, 3)})
        out["dense_vs_sparse"] = cmp_
        up = ws[0]
        r, q = up.W.shape
        Yd = torch.empty((wl.p, r), dtype=X.dtype, device=X.device)
        dYr = torch.empty((wl.p, r), dtype=X.dtype, device=X.device).normal_()
        # the weight gradient next to the vendor library's dY^T X (bf16 output there, fp32 here)
        t_dw = _time_ms(torch, lambda: s24.dense_dw(dYr, X, up.grad, 0.0), 5)
        dWv = torch.empty((r, q), dtype=X.dtype, device=X.device)
        t_dwv = _time_ms(torch, lambda: torch.matmul(dYr.t(), X, out=dWv), 5)
        fl = 2.0 * wl.p * q * r
        out["weight_gradient_vs_vendor_library"] = {
            "shape_p_q_r": [wl.p, q, r], "s24_dense_dw_ms": round(t_dw, 4), "s24_TFLOP/s": round(fl / t_dw / 1e9, 1),
            "vendor_library_ms": round(t_dwv, 4), "vendor_library_TFLOP/s": round(fl / t_dwv / 1e9, 1)}
        del dWv
        clocks = {
            "spmm_fwd": _clock_mhz(torch, s24, lambda: s24.spmm_fwd(X, up.vals, up.meta, Yd)),
            "dense_dw": _clock_mhz(torch, s24, lambda: s24.dense_dw(dYr, X, up.grad, 0.0)),
            "dense_gemm": _clock_mhz(torch, s24, lambda: s24.dense_gemm(X, up.W, Yd)),
        }
        # per clock: 256 CUs x 4 matrix cores x 1024 dense bf16 FLOP (2048 dense-equivalent for 2:4 sparse)
        out["core_clock_under_load"] = {
            "MHz": clocks, "nominal_MHz": 2400,
            "clock_scaled_peak_TFLOP/s": {k: (round(256 * 4 * (2048 if k == "spmm_fwd" else 1024) * v * 1e6 / 1e12, 0)
                                              if v else None) for k, v in clocks.items()},
            "note": "the large-tile GEMMs run (only when the tile count fills the chip); the chip lowers its clock "
                    "under matrix-core + LDS + copy load, so the fraction of the published peak understates how "
                    "busy the matrix cores are"}
    return out


def gated_activation_measurements(torch, s24):
    """Sec. 5.2 / Table 4: GEGLU on the paper's inputs, 32 x 512 tokens by d features (so f = d/2 gated features) in
    binary16, stored column-major as the paper's sparse GEMMs leave them.  Three routes: column-major in and out
    (the paper's kernel), column-major in and row-major out (the layout this library's GEMMs consume; the change of
    layout rides on the same pass through 64 x 64 LDS tiles), row-major in and out.  GB/s counts the algorithmic
    bytes: Z read once, H written once (3 f p elements).  Also the backward kernel and the bias gradient at the
    widest input.  The smaller inputs would fit the Infinity Cache, so each measurement goes round several distinct
    sets of buffers."""
    out = {"input": "32 x 512 x d, binary16", "rows": [],
           "buffers": "every measurement cycles through distinct buffer sets of over 512 MB together, so no call finds "
                      "its operands in the 256 MB Infinity Cache: the rates are HBM rates"}
    p = 32 * 512
    half = lambda *shape: torch.empty(shape, dtype=torch.float16, device="cuda")
    for d in (768, 1024, 1280, 1600, 2048, 4096, 8192):
        f = d // 2
        nbytes = 3.0 * f * p * 2
        n = _rotation(nbytes)
        sets = [(half(d, p).normal_(), half(p, d).normal_(), half(f, p), half(p, f)) for _ in range(n)]
        row = {"d": d, "buffer_sets": n}
        for tag, zi, hi, lz, lh in (("col_to_col", 0, 2, 1, 1), ("col_to_row", 0, 3, 1, 0), ("row_to_row", 1, 3, 0, 0)):
            calls = [lambda z=b[zi], h=b[hi]: s24.glu_fwd(z, h, s24.GATE_GELU_ERF, layout_z=lz, layout_h=lh) for b in sets]
            ms = _time_ms(torch, _in_turn(calls), 20)
            row[tag] = {"ms": round(ms, 4), "GB/s": round(nbytes / ms / 1e6, 1)}
        out["rows"].append(row)
        if d != 8192:
            del sets
    # backward and bias gradient at d = 8192 (dH read, Z read, dZ written: 5 f p elements; bias gradient: 2 f p read)
    bsets = [(half(f, p).normal_(), half(p, f).normal_(), half(d, p), half(p, d)) for _ in range(len(sets))]
    bwd = lambda hi, zi, oi, lh, lz: _in_turn([lambda dh=b[hi], z=a[zi], dz=b[oi]: s24.glu_bwd(
        dh, z, dz, s24.GATE_GELU_ERF, layout_h=lh, layout_z=lz) for a, b in zip(sets, bsets)])
    ms_c = _time_ms(torch, bwd(0, 0, 2, 1, 1), 20)
    ms_r = _time_ms(torch, bwd(1, 1, 3, 0, 0), 20)
    ms_x = _time_ms(torch, bwd(1, 0, 2, 0, 1), 20)
    out["backward_d8192"] = {k: {"ms": round(ms, 4), "GB/s": round(5.0 * f * p * 2 / ms / 1e6, 1)}
                             for k, ms in (("col", ms_c), ("row", ms_r), ("row_dH_col_Z", ms_x))}
    db = torch.empty(d, dtype=torch.float32, device="cuda")
    ms_br = _time_ms(torch, _in_turn([lambda z=a[1]: s24.bias_grad(z, db) for a in sets]), 20)
    ms_bc = _time_ms(torch, _in_turn([lambda z=a[0]: s24.bias_grad(z, db, layout=s24.COL_MAJOR) for a in sets]), 20)
    out["bias_grad_d8192"] = {"row_major": {"ms": round(ms_br, 4), "GB/s": round(2.0 * d * p / ms_br / 1e6, 1)},
                              "col_major": {"ms": round(ms_bc, 4), "GB/s": round(2.0 * d * p / ms_bc / 1e6, 1)}}
    return out


def _rotating(torch, make_set, call, nbytes, min_reps=10):
    """Time `call(set)` over enough distinct buffer sets (made by make_set) that no call finds its operands in the
    Infinity Cache; returns (ms per call, number of sets)."""
    n = _rotation(nbytes)
    sets = [make_set() for _ in range(n)]
    ms = _time_ms(torch, _in_turn([lambda b=b: call(b) for b in sets]), max(min_reps, 2 * n))
    del sets
    return ms, n


def standalone_hbm_kernels(torch, s24, wl, ffn, X):
    """The HBM-bound kernels of the path each on its own (the default step runs the activation and the decay inside
    GEMM epilogues, so the step's own kernel list has no entry for them): gated / ungated activation forward and
    backward at the layer's [tokens][d_ff] size, masked decay, mask search alone, compress with a given mask and
    the fused search + compress on every weight of the layer as the step holds it.  Each measurement cycles through
    distinct buffer sets of over 512 MB together (two sets when one call already moves that much), so the rates
    are HBM rates.  GB/s counts the algorithmic bytes of the call."""
    out = {"buffers": "every measurement cycles through distinct buffer sets of over 512 MB together: HBM rates, "
                      "cache_resident false throughout"}
    es = 4 if wl.dtype == "f32" else 2
    p, f = wl.p, wl.d_ff
    dt, dev = X.dtype, X.device
    new = lambda *shape: torch.empty(shape, dtype=dt, device=dev)
    rnd = lambda *shape: torch.empty(shape, dtype=dt, device=dev).normal_()

    def entry(ms, nbytes, n):
        return {"ms": round(ms, 4), "bytes_per_call": int(nbytes), "GB/s": round(nbytes / ms / 1e6, 1),
                "frac_of_hbm_peak": round(nbytes / ms / 1e6 / PEAK_HBM, 4), "buffer_sets": n, "cache_resident": False}

    if wl.gated:
        nb = 3.0 * p * f * es
        ms, n = _rotating(torch, lambda: (rnd(p, f), rnd(p, f), new(p, f)), lambda b: s24.swiglu_fwd(b[0], b[1], b[2]), nb)
        out["swiglu_fwd"] = entry(ms, nb, n)
        nb = 5.0 * p * f * es
        ms, n = _rotating(torch, lambda: (rnd(p, f), rnd(p, f), rnd(p, f), new(p, f), new(p, f)),
                          lambda b: s24.swiglu_bwd(b[0], b[1], b[2], b[3], b[4]), nb)
        out["swiglu_bwd"] = entry(ms, nb, n)
        # the same on the halves of one [p][2 d_ff] buffer, the layout the stacked gate+up GEMM leaves
        nb = 3.0 * p * f * es
        ms, n = _rotating(torch, lambda: (rnd(p, 2 * f), new(p, f)), lambda b: s24.glu_fwd(b[0], b[1], s24.GATE_SILU), nb)
        out["swiglu_fwd_on_stacked_GU"] = entry(ms, nb, n)
    else:
        act = s24.ACT_RELU if wl.act == "relu" else s24.ACT_GELU_ERF
        nb = 2.0 * p * f * es
        ms, n = _rotating(torch, lambda: (rnd(p, f), new(p, f)), lambda b: s24.act_fwd(b[0], b[1], act), nb)
        out["act_fwd"] = entry(ms, nb, n)
        nb = 3.0 * p * f * es
        ms, n = _rotating(torch, lambda: (rnd(p, f), rnd(p, f), new(p, f)), lambda b: s24.act_bwd(b[0], b[1], b[2], act), nb)
        out["act_bwd"] = entry(ms, nb, n)
    from paper_2404_01847_amd.ffn import SparseWeight
    for name, w in ffn.w.items():
        r, q = w.W.shape
        blocks = r * q / 16
        per = {}

        def make():
            sw = SparseWeight(w.W.clone())
            sw.mask.copy_(w.mask)
            sw.grad.zero_()
            return sw

        nb = r * q * (8 + es + 0.125)
        ms, n = _rotating(torch, make, lambda b: s24.masked_decay_grad(b.grad, b.W, b.mask, wl.lam), nb)
        per["masked_decay_grad"] = entry(ms, nb, n)
        nb = blocks * (16 * es + 2)
        ms, n = _rotating(torch, make, lambda b: s24.transposable_mask(b.W, b.mask, None), nb)
        per["mask_search_only"] = entry(ms, nb, n)
        nb = blocks * (16 * es + 2 + 2 * (8 * es + 2))
        ms, n = _rotating(torch, make, lambda b: s24.compress(b.W, b.mask, b.vals, b.meta, b.valsT, b.metaT), nb)
        per["compress_given_mask"] = entry(ms, nb, n)
        ms, n = _rotating(torch, make, lambda b: s24.compress(b.W, None, b.vals, b.meta, b.valsT, b.metaT, mask_out=b.mask), nb)
        per["mask_search_and_compress"] = entry(ms, nb, n)
        out[f"weight {name} [{r} x {q}]"] = per
    return out


def measured_ceilings(torch, s24):
    """Ceilings measured on this device, next to the published ones: a register-only loop of matrix-core
    instructions (dense MFMA and 2:4-sparse SMFMAC, bf16; no LDS, no memory traffic) and a plain device copy."""
    out = {"label": "measured on this device in this run (the published peaks are 2500 / 5000 TFLOP/s and 8000 GB/s)"}
    wgs, iters = 1024, 8000
    sink = torch.empty(wgs * 512, dtype=torch.float32, device="cuda")
    for sparse, key, flop in ((0, "dense_mfma_32x32x16_bf16", 32768.0), (1, "sparse_smfmac_32x32x32_bf16_dense_equivalent", 65536.0)):
        ms = min(_time_ms(torch, lambda: s24.probe_matrix_rate(sparse, wgs, iters, sink), 2) for _ in range(3))
        out[key + "_TFLOP/s"] = round(wgs * 8 * 4.0 * iters * flop / ms / 1e9, 1)
    out["matrix_rate_probe"] = f"{wgs} workgroups x 8 waves x {4 * iters} instructions on registers only, 4 independent accumulators per wave"
    n = 1 << 28
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ms = min(_time_ms(torch, lambda: s24.probe_copy(src, dst), 5) for _ in range(2))
    out["device_copy_GB/s_read_plus_written"] = round(2.0 * n * 4 / ms / 1e6, 1)
    out["device_copy"] = "1 GiB read + 1 GiB written per call, 16-byte accesses"
    del src, dst, sink
    return out


def operand_value_dependence(torch, s24, wl):
    """The GEMM kernels of the step on one weight's shape, once on the workload's kind of data (normal random) and once
    on operands that are all zero: the same instruction stream, the same schedule and the same bytes moved, but no
    bits toggling in the matrix cores and on the data paths.  What the zero run gains is what the chip's power
    management, not the kernel's schedule, takes from the run on real data."""
    if wl.dtype == "f32":
        return None
    p, q, r = wl.p, wl.d_model, wl.d_ff
    dt = torch.float16 if wl.dtype == "f16" else torch.bfloat16
    fl = 2.0 * p * q * r
    out = {"shape_p_q_r": [p, q, r]}
    for label, xs, ws in (("random_operands", 1.0, 0.02), ("zero_operands", 0.0, 0.0)):
        g = torch.Generator(device="cuda").manual_seed(5)
        X = (torch.randn(p, q, device="cuda", generator=g) * xs).to(dt)
        W = (torch.randn(r, q, device="cuda", generator=g) * ws).to(dt)
        dYr = (torch.randn(p, r, device="cuda", generator=g) * 1e-2 * xs).to(dt)
        vals = torch.empty((q // 64, r, 32), dtype=dt, device="cuda")
        meta = torch.empty((q // 64, r, 4), dtype=torch.int16, device="cuda")
        valsT = torch.empty((r // 64, q, 32), dtype=dt, device="cuda")
        metaT = torch.empty((r // 64, q, 4), dtype=torch.int16, device="cuda")
        s24.compress(W, None, vals, meta, valsT, metaT)
        Y = torch.empty(p, r, dtype=dt, device="cuda")
        dW = torch.empty(r, q, dtype=torch.float32, device="cuda")
        row = {}
        for key, fn in (("spmm_fwd", lambda: s24.spmm_fwd(X, vals, meta, Y)), ("dense_dw", lambda: s24.dense_dw(dYr, X, dW)),
                        ("dense_gemm", lambda: s24.dense_gemm(X, W, Y))):
            ms = _time_ms(torch, fn, 5)
            row[key] = {"ms": round(ms, 4), "TFLOP/s": round(fl / ms / 1e9, 1), "core_clock_MHz": _clock_mhz(torch, s24, fn, 3)}
        out[label] = row
        del X, W, dYr, vals, meta, valsT, metaT, Y, dW
    out["zero_over_random"] = {k: round(out["zero_operands"][k]["TFLOP/s"] / out["random_operands"][k]["TFLOP/s"], 3)
                               for k in out["zero_operands"]}
    return out


def block_level_measurements(torch, s24, wl, ffn, X, dY, weights):
    """The paper's block-level comparison (Sec. 6, speed-up of a single FFN layer and of a single transformer block,
    forward + backward): the 2:4 FFN step of this library next to the same layer run densely through the library's own
    dense GEMMs, and both next to the rest of the block (two layer norms, QKV and output projections, causal attention),
    which is dense in either case and is run here by PyTorch's stock operators, since attention is not part of this
    library.  Reported: the three times and the two speed-ups they imply."""
    F = torch.nn.functional
    p, d, f = wl.p, wl.d_model, wl.d_ff
    dt = X.dtype
    reps = 10
    ms_sparse = _time_ms(torch, lambda: ffn.step(X, dY), reps)
    # the dense layer: same call sequence with s24_dense_gemm in place of the sparse GEMMs (the input-gradient GEMMs
    # read transposed copies of the weights, made once), no mask search, no compress, no decay
    if wl.gated:
        Wup = torch.cat([weights["Wg"], weights["Wu"]], dim=0).contiguous()
        Wdn = weights["Wd"]
    else:
        Wup, Wdn = weights["W1"], weights["W2"]
    WupT, WdnT = Wup.t().contiguous(), Wdn.t().contiguous()
    nz = Wup.shape[0]
    new = lambda *shape: torch.empty(shape, dtype=dt, device=X.device)
    Z, H, Y, dH, dZ, dX = new(p, nz), new(p, f), new(p, d), new(p, f), new(p, nz), new(p, d)
    gUp = torch.empty(Wup.shape, dtype=torch.float32, device=X.device)
    gDn = torch.empty(Wdn.shape, dtype=torch.float32, device=X.device)
    gate = s24.GATE_GELU_ERF if wl.act == "geglu" else s24.GATE_SILU
    act = s24.ACT_RELU if wl.act == "relu" else s24.ACT_GELU_ERF

    def dense_step():
        s24.dense_gemm(X, Wup, Z)
        if wl.gated:
            s24.glu_fwd(Z, H, gate)
        else:
            s24.act_fwd(Z, H, act)
        s24.dense_gemm(H, Wdn, Y)
        s24.dense_gemm(dY, WdnT, dH)
        s24.dense_dw(dY, H, gDn)
        if wl.gated:
            s24.glu_bwd(dH, Z, dZ, gate)
        else:
            s24.act_bwd(dH, Z, dZ, act)
        s24.dense_gemm(dZ, WupT, dX)
        s24.dense_dw(dZ, X, gUp)

    ms_dense = _time_ms(torch, dense_step, reps)
    out = {"ffn_sparse_ms": round(ms_sparse, 4), "ffn_dense_ms": round(ms_dense, 4),
           "ffn_speedup": round(ms_dense / ms_sparse, 3),
           "ffn_dense_note": "the same layer through s24_dense_gemm / s24_dense_dw (dense MFMA kernels of this library, "
                             "transposed weight copies prepared outside the timed region)"}
    # the rest of the block, dense in both cases: PyTorch operators (not this library's code)
    try:
        hd = 128 if d % 128 == 0 and d >= 2048 else 64
        heads = d // hd
        seq = 2048 if p % 2048 == 0 and d >= 4096 else 1024
        batch = p // seq
        g = torch.Generator(device="cuda").manual_seed(11)
        mk = lambda *shape: (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * 0.02).to(dt).requires_grad_()
        Wqkv, Wo = mk(3 * d, d), mk(d, d)
        ln1w, ln1b, ln2w, ln2b = (torch.ones(d, device="cuda", dtype=dt).requires_grad_() for _ in range(4))
        xin = X.detach().clone().requires_grad_()
        gout = dY.detach().clone()

        def attention_part():
            h = F.layer_norm(xin, (d,), ln1w, ln1b)
            qkv = F.linear(h, Wqkv).view(batch, seq, 3, heads, hd).permute(2, 0, 3, 1, 4)
            a = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=True)
            y = xin + F.linear(a.transpose(1, 2).reshape(p, d), Wo)
            z = F.layer_norm(y, (d,), ln2w, ln2b)   # the FFN's input; its gradient arrives from the FFN
            torch.autograd.backward([z, y], [gout, gout])
            for t in (xin, Wqkv, Wo, ln1w, ln1b, ln2w, ln2b):
                t.grad = None

        ms_attn = _time_ms(torch, attention_part, 5)
        out.update({"rest_of_block_ms": round(ms_attn, 4),
                    "rest_of_block": f"PyTorch: 2 layer norms, QKV and output projections, causal attention, "
                                     f"{heads} heads x {hd}, {batch} x {seq} tokens, forward + backward",
                    "block_sparse_ms": round(ms_attn + ms_sparse, 4), "block_dense_ms": round(ms_attn + ms_dense, 4),
                    "block_speedup": round((ms_attn + ms_dense) / (ms_attn + ms_sparse), 3)})
    except Exception as e:   # the comparison above stands on its own if PyTorch's attention is unavailable here
        out["rest_of_block_error"] = f"{type(e).__name__}: {e}"[:300]
    return out


def build_layer(torch, si, SparseFFN, wl, args):
    """Seeded inputs of the workload on the device and the layer in the configuration the flags select."""
    import numpy as np
    host = si.make(wl)

    def to_dev(a):
        t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
        return t.view(torch.bfloat16) if a.dtype == np.uint16 else t

    dev = {k: to_dev(v) for k, v in host.items()}
    biases = None
    if args.geglu_bias:
        biases = {"Wgu": to_dev(si.random_matrix(7001, (2 * wl.d_ff,), 0.3, wl.dtype)),
                  "Wd": to_dev(si.random_matrix(7002, (wl.d_model,), 0.3, wl.dtype))}
    ffn = SparseFFN({n: dev[n] for n in wl.weight_names}, wl.p, wl.act, wl.lam, fuse_decay=not args.no_fuse_decay,
                    concat_gate_up=not args.separate_gate_up, mvue=args.mvue, fuse_swiglu=not args.no_fuse_swiglu,
                    biases=biases, batch_dw=not args.no_batch_dw)
    return host, dev, ffn


def timed_steps(torch, wl, ffn, X, dY, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` steps between two synchronisations; per-kernel HIP-event times
    from inside the timed region.  Returns (ms per step, per-kernel table)."""
    for _ in range(warmup):
        ffn.step(X, dY)
    torch.cuda.synchronize()
    ffn.timings = {}
    t0 = time.perf_counter()
    for _ in range(steps):
        ffn.step(X, dY)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    timings, ffn.timings = ffn.timings, None
    model = kernel_model(wl)
    kernels = {}
    for name, pairs in timings.items():
        ms = [a.elapsed_time(b) for a, b in pairs]
        per_step = sum(ms) / steps
        kind, amount, peak, unit = model[name]
        achieved = amount / (per_step * 1e-3) / (1e12 if kind == "mfma" else 1e9)
        kernels[name] = {"launches_per_step": len(ms) // steps, "ms_per_step": round(per_step, 4),
                         "avg_ms": round(sum(ms) / len(ms), 4), "median_ms": round(sorted(ms)[len(ms) // 2], 4),
                         "min_ms": round(min(ms), 4), "share_of_step": round(per_step / ms_per_step, 4), "bound": kind,
                         "achieved": round(achieved, 1), "peak": peak, "unit": unit, "frac": round(achieved / peak, 4)}
    return ms_per_step, kernels


def workload_label(wl):
    return (f"{wl.name}: FFN d_model={wl.d_model} d_ff={wl.d_ff} tokens={wl.p} act={wl.act} "
            f"{wl.dtype}, {len(wl.weight_names)} weights, mask+compress every step")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"],
                    help="the workload of the headline line (default c5, the largest single-GPU configuration)")
    ap.add_argument("--also", default="c1,c2,c3,c4",
                    help="comma-separated workloads whose step is timed as well (20 steps each) and reported under "
                         "extras.other_workloads; empty for none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the measurements outside the timed step")
    ap.add_argument("--separate-gate-up", action="store_true",
                    help="gate and up projection as two weights (three mask passes and nine GEMMs for a gated FFN) "
                         "instead of one concatenated [2*d_ff, d_model] weight")
    ap.add_argument("--mvue", action="store_true",
                    help="weight gradient from the unbiasedly 2:4-pruned output gradient as a sparse GEMM (Eq. 4, Eq. 6) "
                         "instead of the dense GEMM")
    ap.add_argument("--no-fuse-swiglu", action="store_true",
                    help="SwiGLU forward and backward as their own kernels instead of GEMM epilogues")
    ap.add_argument("--no-batch-dw", action="store_true",
                    help="one launch per weight-gradient GEMM instead of one pass over the tiles of all of them")
    ap.add_argument("--no-fuse-decay", action="store_true",
                    help="masked decay as its own kernel after the weight-gradient GEMM instead of inside its epilogue")
    ap.add_argument("--dtype", default=None, choices=["bf16", "f16"],
                    help="storage type of the 16-bit workloads (default: the workload's own, bf16); f16 is IEEE binary16, "
                         "the precision the paper trains in")
    ap.add_argument("--geglu-bias", action="store_true",
                    help="gated workloads only: the layer of Sec. 5.2 as written, GELU gate and biases on both projections "
                         "(bias add in the GEMM epilogues, bias gradients as their own kernel)")
    ap.add_argument("--no-block", action="store_true",
                    help="skip the block-level comparison (the same layer run densely, and the dense rest of a transformer "
                         "block through PyTorch attention: the FFN-level and block-level speed-ups of the paper's Sec. 6)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 1 GiB device-to-device copy five times (reference for HBM byte counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1. "
                 "Under data parallelism each rank would run exactly this step on its share of the tokens.")

    import torch
    import s24_inputs as si
    import paper_2404_01847_amd as s24
    from paper_2404_01847_amd.ffn import SparseFFN

    s24.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": 5}))
        return
    import dataclasses

    def configured(name):
        wl = si.WORKLOADS[name]
        if args.dtype and wl.dtype != "f32":
            wl = dataclasses.replace(wl, dtype=args.dtype)
        if args.geglu_bias and wl.gated:
            wl = dataclasses.replace(wl, act="geglu")
        return wl

    wl = configured(args.workload)
    if args.geglu_bias and (not wl.gated or args.separate_gate_up):
        sys.exit("bench.py: --geglu-bias needs a gated workload (c4, c5) with gate and up projection as one weight")
    host, dev, ffn = build_layer(torch, si, SparseFFN, wl, args)
    X, dY = dev["X"], dev["dY"]
    ms_per_step, kernels = timed_steps(torch, wl, ffn, X, dY, args.steps, args.warmup)
    value = wl.gemm_flops / (ms_per_step * 1e-3) / 1e12
    # the same steps once more without the per-kernel events of the timed region (two event records per launch: nothing
    # on c5, a fifth of the step on c2)
    ms_plain = _time_ms(torch, lambda: ffn.step(X, dY), args.steps)

    extras = None
    if not args.no_extras:
        weights = {n: dev[n] for n in wl.weight_names}
        extras = side_measurements(torch, s24, wl, ffn, X, dY, weights)
        extras["standalone_hbm_kernels"] = standalone_hbm_kernels(torch, s24, wl, ffn, X)
        extras["measured_ceilings"] = measured_ceilings(torch, s24)
        ovd = operand_value_dependence(torch, s24, wl)
        if ovd is not None:
            extras["operand_value_dependence"] = ovd
        if not args.no_block and wl.dtype != "f32":
            extras["block_level"] = block_level_measurements(torch, s24, wl, ffn, X, dY, weights)

    dom = max(kernels, key=lambda k: kernels[k]["share_of_step"])
    kd = kernels[dom]
    default_cfg = ffn.concat == wl.gated and ffn.fuse_decay and not args.dtype and not args.geglu_bias and not ffn.mvue
    traffic = measured_traffic(wl.name, dom) if default_cfg else None
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"], "unit": kd["unit"],
                "frac": kd["frac"], "traffic": traffic,
                "traffic_source": "profiles/hbm_traffic_pmc.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                  "command, bytes per call of the entry point)" if traffic is not None else None}
    config = {"workload": workload_label(wl),
              "gate_up_as_one_weight": ffn.concat, "decay_in_dw_epilogue": ffn.fuse_decay,
              "swiglu_in_gemm_epilogues": bool(ffn.concat and ffn.fuse_swiglu),
              "weight_gradients_in_one_pass": bool(ffn.batch_dw and not ffn.mvue),
              "weight_gradient": "sparse GEMM on the MVUE-pruned output gradient" if ffn.mvue else "dense GEMM",
              "gemm_flops_per_step": wl.gemm_flops}
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, host)

    # the other workloads' steps, after the headline's buffers are gone
    del ffn, dev, host, X, dY
    torch.cuda.empty_cache()
    if extras is not None and args.also.strip():
        others = {}
        for name in [n.strip() for n in args.also.split(",") if n.strip() and n.strip() != wl.name]:
            if name not in si.WORKLOADS:
                sys.exit(f"bench.py: unknown workload {name!r} in --also")
            w2 = configured(name)
            if args.geglu_bias and not w2.gated:
                continue
            _, d2, f2 = build_layer(torch, si, SparseFFN, w2, args)
            # two passes of 20 steps: one with the per-kernel timing events (two event records per launch, which weigh
            # on a layer whose kernels take tens of microseconds) for the kernel table, one without them for the step
            ms_i, k2 = timed_steps(torch, w2, f2, d2["X"], d2["dY"], 20, 5)
            ms2 = _time_ms(torch, lambda: f2.step(d2["X"], d2["dY"]), 20)
            others[name] = {"workload": workload_label(w2), "steps": 20, "warmup": 5, "ms_per_step": round(ms2, 4),
                            "TFLOP/s": round(w2.gemm_flops / ms2 / 1e9, 2),
                            "pct_of_sparse_mfma_peak_whole_step": round(100 * w2.gemm_flops / ms2 / 1e9 / PEAK_SPARSE_BF16, 2),
                            "ms_per_step_with_kernel_events": round(ms_i, 4),
                            "kernels": {k: {f: v[f] for f in ("launches_per_step", "ms_per_step", "achieved", "unit", "frac")}
                                        for k, v in k2.items()}}
            if not f2.mvue:   # the same step replayed from one HIP graph: what it costs without launch gaps
                graph = f2.capture(d2["X"], d2["dY"])
                ms_g = _time_ms(torch, graph.replay, 20)
                others[name]["as_hip_graph"] = {"ms_per_step": round(ms_g, 4), "TFLOP/s": round(w2.gemm_flops / ms_g / 1e9, 2)}
                del graph
            del d2, f2
            torch.cuda.empty_cache()
            if w2.dtype == "f32":
                others[name]["note"] = ("fp32 correctness workload: gfx950 has no fp32 sparse matrix instruction, the GEMMs run "
                                        "on the vector unit; fractions of the bf16 peaks are shown for form only")
            if name == "c3":
                others[name]["mask_search_only_72_matrices"] = c3_mask_sweep(torch, s24, w2)
        extras["other_workloads"] = others

    out = {
        "metric": "2:4 FFN fwd+bwd TFLOP/s (dense-equivalent GEMM FLOPs over the whole step)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_without_kernel_events": round(ms_plain, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": config,
        "pct_of_sparse_mfma_peak_whole_step": round(100 * value / PEAK_SPARSE_BF16, 2),
        "roofline": roofline,
        "kernels": kernels,
        "extras": extras,
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
