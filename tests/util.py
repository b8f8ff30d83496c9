"""Helpers shared by the GPU parity tests: host<->device conversion of the
seeded inputs and the error measures of the parity bar."""
import numpy as np
import torch

import s24_inputs as si


def dev(a: np.ndarray) -> torch.Tensor:
    """numpy (float32, float16, or uint16 = bf16 bits / mask words, or uint8) -> CUDA tensor."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_bf16(a: np.ndarray) -> torch.Tensor:
    """bf16 bit array (uint16) -> CUDA bfloat16 tensor; float32 and float16 arrays pass through."""
    t = dev(a)
    return t.view(torch.bfloat16) if a.dtype == np.uint16 else t


def host_bits(t: torch.Tensor) -> np.ndarray:
    """CUDA tensor -> numpy; bfloat16 and int16 come back as uint16 bit arrays."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    a = t.numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def host_f64(t: torch.Tensor) -> np.ndarray:
    return si.to_f32(host_bits(t)).astype(np.float64)


def errors(got: np.ndarray, ref: np.ndarray):
    """(max scaled element error, normwise error).  The element error divides by
    max(|ref|, 1e-2 * rms(ref)) so that cancellations do not blow it up."""
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    rms = np.sqrt(np.mean(ref * ref)) if ref.size else 0.0
    den = np.maximum(np.abs(ref), 1e-2 * rms)
    den[den == 0] = 1.0
    d = np.abs(got - ref)
    nrm = np.linalg.norm(ref.reshape(-1))
    return float((d / den).max()) if ref.size else 0.0, float(np.linalg.norm(d.reshape(-1)) / (nrm if nrm else 1.0))


# bf16 in / fp32 accumulate: max relative error 1e-2, normwise 5e-3
BF16_TOL = (1e-2, 5e-3)
# binary16 in / fp32 accumulate: the same bar holds with room to spare (11 significant bits instead of 8); the
# tighter figures are what one rounding to binary16 of an fp32-accumulated sum allows, with some slack for
# results that land among the subnormals
F16_TOL = (4e-3, 1e-3)
# fp32 data path (small correctness workload): accumulation-order noise only
F32_TOL = (1e-3, 2e-5)


def tol_for(dtype: str):
    return {"bf16": BF16_TOL, "f16": F16_TOL, "f32": F32_TOL}[dtype]


def torch_dtype(dtype: str):
    return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]


def bits(t: torch.Tensor) -> torch.Tensor:
    """Integer view of a tensor for bit-exact comparison."""
    return t.view(torch.int32) if t.dtype == torch.float32 else t.view(torch.int16)


def assert_close(got, ref, tol, what=""):
    e_max, e_nrm = errors(got, ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert e_max <= tol[0] and e_nrm <= tol[1], f"{what}: max rel {e_max:.3e} (<= {tol[0]}), normwise {e_nrm:.3e} (<= {tol[1]})"
    return e_max, e_nrm


def absorbed_margin_blocks(legal, dtype: str, big_exp: int, every: int = 7):
    """4x4 blocks whose two best patterns differ by less than fp64 sums of eight terms can see.

    For a pair of legal patterns (a, b), a before b in the canonical order, that share six cells and differ by one
    2x2 swap (no third pattern holds all six shared cells), the shared cells hold 2^big_exp, the two cells only a has
    hold 1 and 1, the two only b has hold 1 + ulp and 1, everything else 0: b retains exactly one ulp of 1 more than
    a, so exact scoring picks b although a comes first, while 6 * 2^big_exp + 2 + ulp rounds to 6 * 2^big_exp + 2 in
    fp64 once big_exp is large enough - a scorer that adds in fp64 there sees a tie and takes a.
    `legal` is the list of the 90 encodings in canonical order (bit 4i+j = m_ij).  Returns (W [4, 4n] in the storage
    of `dtype` ("f32" or "bf16"), the n expected encodings)."""
    ulp = {"f32": 2.0 ** -23, "bf16": 2.0 ** -7}[dtype]
    blocks, want = [], []
    n = 0
    for ia, a in enumerate(legal):
        for b in legal[ia + 1:]:
            shared = a & b
            if bin(shared).count("1") != 6 or any(c not in (a, b) and (c & shared) == shared for c in legal):
                continue
            n += 1
            if n % every:
                continue
            blk = np.zeros(16, dtype=np.float64)
            for t in range(16):
                if (shared >> t) & 1:
                    blk[t] = 2.0 ** big_exp
            only_a = [t for t in range(16) if ((a & ~b) >> t) & 1]
            only_b = [t for t in range(16) if ((b & ~a) >> t) & 1]
            blk[only_a[0]], blk[only_a[1]] = 1.0, 1.0
            blk[only_b[0]], blk[only_b[1]] = 1.0 + ulp, 1.0
            sign = np.where((np.arange(16) + n) % 3 == 0, -1.0, 1.0)   # signs must not matter
            blocks.append((blk * sign).reshape(4, 4))
            want.append(b)
    W = np.concatenate(blocks, axis=1).astype(np.float32)
    if dtype == "bf16":
        W = si.f32_to_bf16_bits(torch.from_numpy(W))
    return W, want
