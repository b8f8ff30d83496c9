"""Host-side sequencing of one 2:4-sparse FFN training step (App. B workflow).

Only call ordering and buffer ownership live here; every arithmetic step is a
libs24 kernel.  One step = for every weight: transposable mask search fused
with prune/compress (Sec. 5.1), the sparse forward GEMMs (Eq. 2), the
activation (Sec. 5.2), the sparse input-gradient GEMMs (Eq. 3), the dense
weight-gradient GEMMs (Eq. 1) and the masked decay on gradients (Eq. 10).
"""
from __future__ import annotations

import torch

from . import binding as s24

_ACT = {"relu": s24.ACT_RELU, "gelu": s24.ACT_GELU_ERF}
_GATE = {"swiglu": s24.GATE_SILU, "geglu": s24.GATE_GELU_ERF}


class SparseWeight:
    """A weight W [r, q] with its block mask and both compressed orientations."""

    def __init__(self, W: torch.Tensor):
        r, q = W.shape
        dev, dt = W.device, W.dtype
        self.W = W
        self.mask = torch.empty((r // 4, q // 4), dtype=torch.int16, device=dev)
        # chunk-major compressed operands: 64 of the contraction axis per chunk
        self.vals = torch.empty((q // 64, r, 32), dtype=dt, device=dev)
        self.meta = torch.empty((q // 64, r, 4), dtype=torch.int16, device=dev)
        self.valsT = torch.empty((r // 64, q, 32), dtype=dt, device=dev)
        self.metaT = torch.empty((r // 64, q, 4), dtype=torch.int16, device=dev)
        self.grad = torch.empty((r, q), dtype=torch.float32, device=dev)
        self.zvals = self.zmeta = None   # compressed pruned output gradient, allocated on first use

    def pruned_grad_buffers(self, p):
        """Buffers of the unbiasedly pruned output gradient S_z(dY^T) of this weight for p tokens."""
        if self.zvals is None or self.zvals.shape[0] != p // 64:
            r = self.W.shape[0]
            self.zvals = torch.empty((p // 64, r, 32), dtype=self.W.dtype, device=self.W.device)
            self.zmeta = torch.empty((p // 64, r, 4), dtype=torch.int16, device=self.W.device)
        return self.zvals, self.zmeta

    def refresh(self, call=None, search=True):
        """Rebuild both compressed operands in one pass over W; with `search` the mask is searched in the
        same pass, otherwise the stored mask is applied as it is (the steps between two mask updates)."""
        call = call or (lambda name, fn, *a, **k: fn(*a, **k))
        if search:
            call("mask_compress", s24.compress, self.W, None, self.vals, self.meta, self.valsT, self.metaT,
                 mask_out=self.mask)
        else:
            call("compress", s24.compress, self.W, self.mask, self.vals, self.meta, self.valsT, self.metaT)


class SparseFFN:
    """Buffers and call sequence of one FFN layer.  act: 'relu' | 'gelu' | 'swiglu' | 'geglu' (the last one needs
    concat_gate_up).  `biases` maps weight names (after concatenation: 'Wgu', 'Wd'; else 'Wg', 'Wu', 'Wd' or
    'W1', 'W2') to bias vectors in the weights' dtype: Z = X W^T + d as in Sec. 5.2 step 2; their gradients are
    left in `bias_grad[name]` (fp32)."""

    def __init__(self, weights: dict, p: int, act: str, lam: float, fuse_decay: bool = True, mask_interval: int = 1,
                 concat_gate_up: bool = False, mvue: bool = False, seed: int = 0, fuse_swiglu: bool = True,
                 biases: dict | None = None, batch_dw: bool = True):
        self.act, self.lam, self.p = act, lam, p
        # all dense weight gradients of the layer in one pass: the idle tail of one GEMM's tile grid takes the next one's tiles
        self.batch_dw, self._pending_dw = batch_dw, []
        # Eq. 4 / Eq. 6: the weight gradient from an unbiasedly 2:4-pruned output gradient, as a sparse GEMM
        self.mvue, self.seed = mvue, seed
        self.fuse_swiglu = fuse_swiglu   # the activation in the epilogue of the first projection's forward GEMM
        self.fuse_gate_bwd = None        # and its backward in the epilogue of the dH GEMM where the shape allows (probed)
        self.mask_interval = mask_interval   # the mask is searched every mask_interval-th step (Sec. 5.1: l = 40)
        self.steps_done = 0
        self.draws = 0
        self.fuse_decay = fuse_decay   # masked decay inside the weight-gradient GEMM's epilogue
        self.timings = None   # when a dict: kernel name -> list of (start, end) torch.cuda.Event pairs
        self.gated = act in _GATE
        self.gate = _GATE.get(act)
        if act == "geglu" and not concat_gate_up:
            raise ValueError("the GEGLU kernels take Z = [Z_1 | Z_2] as one buffer: use concat_gate_up=True")
        # gate and up projection held as one [2*d_ff, d_model] weight (Sec. 5.2): one mask/compress pass, one
        # forward GEMM into a [p, 2*d_ff] buffer whose halves are Z_1 and Z_2, one input-gradient GEMM over
        # the 2*d_ff contraction instead of two accumulated ones, one weight-gradient GEMM
        self.concat = self.gated and concat_gate_up
        if self.concat:
            weights = {"Wgu": torch.cat([weights["Wg"], weights["Wu"]], dim=0).contiguous(), "Wd": weights["Wd"]}
            names = ("Wgu", "Wd")
        else:
            names = ("Wg", "Wu", "Wd") if self.gated else ("W1", "W2")
        self.w = {n: SparseWeight(weights[n]) for n in names}
        self.bias = {n: (biases or {}).get(n) for n in names}
        self.bias_grad = {n: torch.empty(b.numel(), dtype=torch.float32, device=b.device)
                          for n, b in self.bias.items() if b is not None}
        d = weights[names[0]].shape[1]
        f = weights[names[-1]].shape[1]
        up = self.w[names[0]].W
        dev, dt = up.device, up.dtype
        new = lambda *shape: torch.empty(shape, dtype=dt, device=dev)
        self.H, self.dH, self.Y, self.dX = new(p, f), new(p, f), new(p, d), new(p, d)
        if self.concat:
            self.GU, self.dGU = new(p, 2 * f), new(p, 2 * f)
            self.G, self.U, self.dG, self.dU = self.GU[:, :f], self.GU[:, f:], self.dGU[:, :f], self.dGU[:, f:]
        elif self.gated:
            self.G, self.U, self.dG, self.dU = new(p, f), new(p, f), new(p, f), new(p, f)
        else:
            self.Z, self.dZ = new(p, f), new(p, f)

    def _k(self, name, fn, *args, **kw):
        """Run one library call; with `timings` set, bracket it with events on the current stream."""
        if self.timings is None:
            return fn(*args, **kw)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn(*args, **kw)
        e1.record()
        self.timings.setdefault(name, []).append((e0, e1))
        return out

    def prune(self, search=True):
        for w in self.w.values():
            w.refresh(self._k, search)

    def _fwd(self, Xw, name, out):
        """out = Xw (M.*W)^T, plus the weight's bias if it has one."""
        w = self.w[name]
        if self.bias[name] is None:
            self._k('spmm_fwd', s24.spmm_fwd, Xw, w.vals, w.meta, out)
        else:
            self._k('spmm_fwd', s24.spmm_fwd_bias, Xw, w.vals, w.meta, self.bias[name], out)

    def forward(self, X):
        w = self.w
        if self.concat and self.fuse_swiglu:
            if self.gate == s24.GATE_SILU and self.bias["Wgu"] is None:
                self._k('spmm_fwd', s24.spmm_fwd_swiglu, X, w["Wgu"].vals, w["Wgu"].meta, self.GU, self.H)
            else:
                self._k('spmm_fwd', s24.spmm_fwd_glu, X, w["Wgu"].vals, w["Wgu"].meta, self.bias["Wgu"], self.GU, self.H,
                        self.gate)
            self._fwd(self.H, "Wd", self.Y)
        elif self.concat:
            self._fwd(X, "Wgu", self.GU)
            self._k('swiglu_fwd', s24.glu_fwd, self.GU, self.H, self.gate)
            self._fwd(self.H, "Wd", self.Y)
        elif self.gated:
            self._fwd(X, "Wg", self.G)
            self._fwd(X, "Wu", self.U)
            self._k('swiglu_fwd', s24.swiglu_fwd, self.G, self.U, self.H)
            self._fwd(self.H, "Wd", self.Y)
        elif self.fuse_swiglu:   # the activation in the epilogue of the first projection's GEMM
            self._k('spmm_fwd', s24.spmm_fwd_act, X, w["W1"].vals, w["W1"].meta, self.bias["W1"], self.Z, self.H,
                    _ACT[self.act])
            self._fwd(self.H, "W2", self.Y)
        else:
            self._fwd(X, "W1", self.Z)
            self._k('act_fwd', s24.act_fwd, self.Z, self.H, _ACT[self.act])
            self._fwd(self.H, "W2", self.Y)
        return self.Y

    def _dw(self, dYw, Xw, weight):
        for name, w in self.w.items():   # the bias gradient of this weight: column sums of its output gradient
            if w is weight and self.bias[name] is not None:
                self._k('bias_grad', s24.bias_grad, dYw, self.bias_grad[name])
        if self.batch_dw and not self.mvue:   # collected; backward() runs them all in one pass at its end
            self._pending_dw.append((dYw, Xw, weight.grad, weight.W if self.fuse_decay else None,
                                     weight.mask if self.fuse_decay else None, self.lam))
            return
        if self.mvue:
            zv, zm = weight.pruned_grad_buffers(dYw.shape[0])
            self.draws += 1   # a fresh draw for every pruned operand of every step
            self._k('mvue24', s24.mvue24, dYw, self.seed + self.draws, zv, zm)
            if self.fuse_decay:
                self._k('spmm_dw', s24.spmm_dw, zv, zm, Xw, weight.grad, 0.0, weight.W, weight.mask, self.lam)
            else:
                self._k('spmm_dw', s24.spmm_dw, zv, zm, Xw, weight.grad)
        elif self.fuse_decay:
            self._k('dense_dw', s24.dense_dw_decay, dYw, Xw, weight.grad, weight.W, weight.mask, self.lam)
        else:
            self._k('dense_dw', s24.dense_dw, dYw, Xw, weight.grad)

    def _flush_dw(self):
        if self._pending_dw:
            self._k('dense_dw', s24.dense_dw_batch, self._pending_dw)
            self._pending_dw = []

    def backward(self, X, dY):
        out = self._backward(X, dY)
        self._flush_dw()
        return out

    def _backward(self, X, dY):
        w = self.w
        if self.concat:
            fused = False
            if self.fuse_swiglu and self.fuse_gate_bwd is not False:
                try:
                    self._k('spmm_bwd_dx', s24.spmm_bwd_dx_glu, dY, w["Wd"].valsT, w["Wd"].metaT, self.GU, self.dGU,
                            self.gate)
                    fused = self.fuse_gate_bwd = True
                except s24.S24Error as e:
                    if e.status != -6:   # anything but "this shape takes the two-call route"
                        raise
                    self.fuse_gate_bwd = False
            if not fused:
                self._k('spmm_bwd_dx', s24.spmm_bwd_dx, dY, w["Wd"].valsT, w["Wd"].metaT, self.dH)
                self._k('swiglu_bwd', s24.glu_bwd, self.dH, self.GU, self.dGU, self.gate)
            self._dw(dY, self.H, w["Wd"])
            self._k('spmm_bwd_dx', s24.spmm_bwd_dx, self.dGU, w["Wgu"].valsT, w["Wgu"].metaT, self.dX)
            self._dw(self.dGU, X, w["Wgu"])
        elif self.gated:
            self._k('spmm_bwd_dx', s24.spmm_bwd_dx, dY, w["Wd"].valsT, w["Wd"].metaT, self.dH)
            self._dw(dY, self.H, w["Wd"])
            self._k('swiglu_bwd', s24.swiglu_bwd, self.dH, self.G, self.U, self.dG, self.dU)
            self._k('spmm_bwd_dx', s24.spmm_bwd_dx, self.dG, w["Wg"].valsT, w["Wg"].metaT, self.dX)
            self._k('spmm_bwd_dx', s24.spmm_bwd_dx, self.dU, w["Wu"].valsT, w["Wu"].metaT, self.dX, beta=1.0)
            self._dw(self.dG, X, w["Wg"])
            self._dw(self.dU, X, w["Wu"])
        else:
            fused = False
            if self.fuse_swiglu and self.fuse_gate_bwd is not False:
                try:
                    self._k('spmm_bwd_dx', s24.spmm_bwd_dx_act, dY, w["W2"].valsT, w["W2"].metaT, self.Z, self.dZ,
                            _ACT[self.act])
                    fused = self.fuse_gate_bwd = True
                except s24.S24Error as e:
                    if e.status != -6:   # anything but "this shape takes the two-call route"
                        raise
                    self.fuse_gate_bwd = False
            if not fused:
                self._k('spmm_bwd_dx', s24.spmm_bwd_dx, dY, w["W2"].valsT, w["W2"].metaT, self.dH)
                self._k('act_bwd', s24.act_bwd, self.dH, self.Z, self.dZ, _ACT[self.act])
            self._dw(dY, self.H, w["W2"])
            self._k('spmm_bwd_dx', s24.spmm_bwd_dx, self.dZ, w["W1"].valsT, w["W1"].metaT, self.dX)
            self._dw(self.dZ, X, w["W1"])
        return self.dX

    def decay(self):
        if self.fuse_decay:
            return   # already applied by backward()
        for w in self.w.values():
            self._k('masked_decay', s24.masked_decay_grad, w.grad, w.W, w.mask, self.lam)

    def step(self, X, dY, search=None):
        """Mask + compress, forward, backward, masked decay: the whole hot path once.  `search` forces (True) or
        suppresses (False) the mask search of this step; by default the step count and mask_interval decide."""
        if search is None:
            search = self.steps_done % self.mask_interval == 0
        self.prune(search=search)
        self.steps_done += 1
        self.forward(X)
        self.backward(X, dY)
        self.decay()

    def capture(self, X, dY):
        """Record the step into HIP graphs and return an object whose replay() reruns it on the same buffers.
        Possible because the step allocates nothing, never synchronises and only launches kernels on the current
        stream.  Worth it where launches, not kernels, bound the step.  With mask_interval == 1 that object is the one
        torch.cuda.CUDAGraph of the step; otherwise two graphs are recorded, the step with the mask search and the
        step that re-applies the stored mask, and replay() picks by the layer's step count exactly as step() does,
        so the schedule of Sec. 5.1 (search every l-th step) survives the capture."""
        if self.timings is not None:
            raise RuntimeError("switch the per-kernel timing hooks off before capturing")
        if self.mvue:
            raise RuntimeError("the seed of the pruning draw is a launch argument: a replayed graph would repeat the draw")
        done = self.steps_done
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step(X, dY, search=True)   # once outside the capture: library load and lazy initialisation
        torch.cuda.current_stream().wait_stream(side)
        graphs = {}
        for search in ((True,) if self.mask_interval == 1 else (True, False)):
            graphs[search] = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graphs[search]):
                self.step(X, dY, search=search)
        self.steps_done = done + 1          # the warm-up run was a real step (with a search); recording runs nothing
        if self.mask_interval == 1:
            return graphs[True]
        return _CapturedSchedule(self, graphs[True], graphs[False])


class _CapturedSchedule:
    """The captured step of a layer whose mask is searched every mask_interval-th step only."""

    def __init__(self, ffn, with_search, without_search):
        self.ffn, self.with_search, self.without_search = ffn, with_search, without_search

    def replay(self):
        ffn = self.ffn
        search = ffn.steps_done % ffn.mask_interval == 0
        (self.with_search if search else self.without_search).replay()
        ffn.steps_done += 1
