"""Seeded synthetic inputs for the 2:4-sparse FFN step.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It only draws random numbers and changes number formats; none of
the method's arithmetic (masks, compression, GEMMs, activations) lives here.

The five workloads are FFN *shapes* (GPT-2-small/-large and LLaMA-class
layers); they stand in for the language-model layers the paper trains, whose
datasets and weights are not available here.  Every tensor is drawn on the
host with torch.Generator('cpu').manual_seed(seed), as randn * std in fp32,
in the fixed order: weights (W1, W2 | Wg, Wu, Wd), X, dY; bf16 workloads then
round to bf16 (nearest-even).  bf16 tensors are returned as uint16 bit arrays,
fp16 ("f16", IEEE binary16) tensors as numpy float16 arrays.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    p: int          # tokens (batch x sequence, flattened)
    d_model: int
    d_ff: int
    act: str        # "relu" | "gelu" | "swiglu" | "geglu"
    dtype: str      # "f32" | "bf16" | "f16"
    seed: int
    std_w: float = 0.02
    std_x: float = 1.0
    std_dy: float = 1e-2
    lam: float = 2e-4   # masked-decay factor (the paper's GPT-2 350M/774M value)

    @property
    def gated(self) -> bool:
        return self.act in ("swiglu", "geglu")

    @property
    def weight_names(self):
        return ("Wg", "Wu", "Wd") if self.gated else ("W1", "W2")

    def weight_shape(self, name):
        if name in ("W1", "Wg", "Wu"):
            return (self.d_ff, self.d_model)
        return (self.d_model, self.d_ff)

    @property
    def gemm_flops(self) -> float:
        """Dense-equivalent FLOPs of all GEMMs of one fwd+bwd step (3 per weight)."""
        return 3 * len(self.weight_names) * 2.0 * self.p * self.d_model * self.d_ff


WORKLOADS = {
    "c1": Workload("c1", 512, 256, 1024, "relu", "f32", 0, std_dy=1.0),
    "c2": Workload("c2", 8192, 768, 3072, "gelu", "bf16", 1),
    "c3": Workload("c3", 16384, 1280, 5120, "gelu", "bf16", 2),
    "c4": Workload("c4", 16384, 4096, 11008, "swiglu", "bf16", 3),
    "c5": Workload("c5", 8192, 8192, 28672, "swiglu", "bf16", 4),
}


def f32_to_bf16_bits(x: torch.Tensor) -> np.ndarray:
    """fp32 tensor -> bf16 (round-to-nearest-even) -> uint16 bit array."""
    return x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 values (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def to_f32(a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a.astype(np.float32, copy=False)


def _store(t: torch.Tensor, dtype: str) -> np.ndarray:
    """fp32 tensor -> the array type of `dtype` (nearest-even where it narrows)."""
    if dtype == "bf16":
        return f32_to_bf16_bits(t)
    if dtype == "f16":
        return t.to(torch.float16).numpy()
    return t.numpy()


def _draw(gen, shape, std, dtype):
    return _store(torch.randn(shape, generator=gen, dtype=torch.float32) * std, dtype)


def make(wl: Workload, p: int | None = None, only_weights: bool = False) -> dict:
    """All tensors of a workload.  `p` truncates nothing: a smaller p draws a
    smaller X/dY (used by reduced test cases), the weights stay the same."""
    gen = torch.Generator(device="cpu").manual_seed(wl.seed)
    out = {}
    for name in wl.weight_names:
        out[name] = _draw(gen, wl.weight_shape(name), wl.std_w, wl.dtype)
    if only_weights:
        return out
    pp = wl.p if p is None else p
    out["X"] = _draw(gen, (pp, wl.d_model), wl.std_x, wl.dtype)
    out["dY"] = _draw(gen, (pp, wl.d_model), wl.std_dy, wl.dtype)
    return out


def random_matrix(seed: int, shape, std: float, dtype: str) -> np.ndarray:
    gen = torch.Generator(device="cpu").manual_seed(seed)
    return _draw(gen, shape, std, dtype)


def sweep_weight(layer: int, which: int, wl: Workload = WORKLOADS["c3"]) -> np.ndarray:
    """Weight `which` (0 = up, 1 = down) of layer `layer` of the mask-only sweep
    over a whole model's FFN weights (seed = 1000*wl.seed + layer)."""
    gen = torch.Generator(device="cpu").manual_seed(1000 * wl.seed + layer)
    shapes = [(wl.d_ff, wl.d_model), (wl.d_model, wl.d_ff)]
    w = None
    for k in range(which + 1):
        w = _draw(gen, shapes[k], wl.std_w, wl.dtype)
    return w


def tie_matrix(seed: int, r: int, q: int, dtype: str, kind: str) -> np.ndarray:
    """Matrices built to provoke exactly tied pattern scores and wide exponent
    ranges inside 4x4 blocks.

    kind "few":    entries from {+-1, +-2, +-3} * 2^e, e in {-3..0}
    kind "equal":  every entry +-c for one c (all patterns tie)
    kind "zeros":  about half the entries are +-0
    kind "tiny":   normal(0, .02) with one entry per block scaled by 2^-30
    kind "range":  entries 2^e with e uniform in [-120, 100] (far beyond any
                   fixed-point window), random signs and 1..3 leading digits
    kind "subnormal": bf16/fp32 subnormals mixed with normals
    kind "window": 8-bit significands times 2^e, the exponents of a block spread over up to 11 binades above a
                   per-block base drawn from the whole exponent range
    For "f16" the same kinds stay inside binary16: "tiny" scales by 2^-12, "range" takes
    e in [-24, 13], "subnormal" mixes multiples of 2^-24 with multiples of 2^-17.
    """
    half = dtype == "f16"
    g = torch.Generator(device="cpu").manual_seed(seed)
    sign = (torch.randint(0, 2, (r, q), generator=g) * 2 - 1).float()
    if kind == "few":
        m = torch.randint(1, 4, (r, q), generator=g).float()
        e = torch.randint(-3, 1, (r, q), generator=g).float()
        x = sign * m * torch.pow(torch.tensor(2.0), e)
    elif kind == "equal":
        x = sign * 0.4375
    elif kind == "zeros":
        z = torch.randint(0, 2, (r, q), generator=g).float()
        x = sign * z * torch.randint(0, 3, (r, q), generator=g).float() * 0.5
    elif kind == "tiny":
        x = torch.randn((r, q), generator=g) * 0.02
        pick = torch.randint(0, 16, (r // 4, q // 4), generator=g)
        for t in range(16):
            sel = (pick == t)
            blk = x[t // 4::4, t % 4::4]
            blk[sel] = blk[sel] * (2.0 ** -12 if half else 2.0 ** -30)
    elif kind == "range":
        m = torch.randint(1, 8, (r, q), generator=g).float()
        e = (torch.randint(-24, 14, (r, q), generator=g) if half else torch.randint(-120, 101, (r, q), generator=g)).double()
        x = (sign.double() * m.double() * torch.pow(torch.tensor(2.0, dtype=torch.float64), e)).float()
    elif kind == "subnormal":
        m = torch.randint(0, 128, (r, q), generator=g).double()
        e = torch.where(torch.randint(0, 4, (r, q), generator=g) == 0, -17.0 if half else -126.0, -24.0 if half else -133.0)
        x = (sign.double() * m * torch.pow(torch.tensor(2.0, dtype=torch.float64), e.double())).float()
    elif kind == "window":
        # full 8-bit significands (few distinct ones, so sums tie or differ in the last bit) times 2^e, where the
        # exponents of one block spread over 0 .. 11 binades above a per-block base anywhere in the type's range:
        # blocks on both sides of a 10-binade fixed-point window, and blocks that are tiny as a whole
        sig = torch.tensor([128.0, 129.0, 192.0, 255.0])[torch.randint(0, 4, (r, q), generator=g)]
        lo, hi = (-20, 2) if half else (-125, 100)
        base = torch.randint(lo, hi, (r // 4, q // 4), generator=g).repeat_interleave(4, 0).repeat_interleave(4, 1)
        spread = torch.randint(0, 12, (r // 4, q // 4), generator=g).repeat_interleave(4, 0).repeat_interleave(4, 1)
        e = base + (torch.rand((r, q), generator=g) * (spread + 1).float()).floor().clamp(max=11)
        x = (sign.double() * sig.double() * torch.pow(torch.tensor(2.0, dtype=torch.float64), e.double() - 7.0)).float()
    else:
        raise ValueError(kind)
    return _store(x, dtype).copy()
