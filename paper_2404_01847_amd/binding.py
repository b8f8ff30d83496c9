"""ctypes binding of libs24.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (bf16 data as
torch.bfloat16, binary16 as torch.float16, masks/metadata as int16/uint16 views, pattern ids as uint8),
passes their data pointers and the current HIP stream to the C entry point of
the same name, and raises S24Error on a non-zero status.  Nothing is computed
here and nothing falls back to PyTorch.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

F32, BF16, F16 = 0, 1, 2
ACT_RELU, ACT_GELU_ERF = 0, 1
GATE_SILU, GATE_GELU_ERF = 0, 1
ROW_MAJOR, COL_MAJOR = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libs24.so")
_lib = None

_i64, _vp, _int, _f32 = C.c_int64, C.c_void_p, C.c_int, C.c_float
_SIGNATURES = {
    "s24_strerror": (C.c_char_p, [_int]),
    "s24_pattern_table": (_int, [_vp]),
    "s24_transposable_mask": (_int, [_vp, _int, _i64, _i64, _i64, _vp, _vp, _vp]),
    "s24_compress": (_int, [_vp, _int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "s24_spmm_fwd": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_spmm_fwd_bias": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_spmm_fwd_glu": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp]),
    "s24_spmm_bwd_dx_glu": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp]),
    "s24_glu_fwd": (_int, [_vp, _int, _i64, _vp, _int, _i64, _i64, _i64, _int, _int, _vp]),
    "s24_glu_bwd": (_int, [_vp, _int, _i64, _vp, _int, _i64, _vp, _i64, _i64, _int, _int, _vp]),
    "s24_bias_grad": (_int, [_vp, _int, _i64, _i64, _i64, _vp, _f32, _int, _vp]),
    "s24_spmm_fwd_act": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp]),
    "s24_spmm_bwd_dx_act": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp]),
    "s24_spmm_fwd_swiglu": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_spmm_bwd_dx": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _f32, _int, _vp]),
    "s24_spmm_bwd_dx_swiglu": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_dense_dw": (_int, [_vp, _vp, _vp, _i64, _i64, _i64, _f32, _int, _vp]),
    "s24_dense_dw_decay": (_int, [_vp, _vp, _vp, _vp, _int, _vp, _f32, _i64, _i64, _i64, _f32, _int, _vp]),
    "s24_dense_dw_batch": (_int, [_vp, _int, _f32, _int, _vp]),
    "s24_mvue24": (_int, [_vp, _int, _i64, _i64, _i64, C.c_uint32, _vp, _vp, _vp]),
    "s24_spmm_dw": (_int, [_vp, _vp, _vp, _vp, _vp, _int, _vp, _f32, _i64, _i64, _i64, _f32, _int, _vp]),
    "s24_dense_gemm": (_int, [_vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_masked_decay_grad": (_int, [_vp, _vp, _int, _vp, _f32, _i64, _i64, _vp]),
    "s24_swiglu_fwd": (_int, [_vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_swiglu_bwd": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]),
    "s24_act_fwd": (_int, [_vp, _vp, _i64, _int, _int, _vp]),
    "s24_act_bwd": (_int, [_vp, _vp, _vp, _i64, _int, _int, _vp]),
    "s24_mask_flips": (_int, [_vp, _vp, _i64, _vp, _vp, _vp]),
    "s24_l1_norm_gap": (_int, [_vp, _int, _i64, _i64, _i64, _vp, _vp]),
    "s24_set_clock_probe": (_int, [_vp]),
    "s24_probe_matrix_rate": (_int, [_int, _int, _int, _vp, _vp]),
    "s24_probe_copy": (_int, [_vp, _vp, _i64, _vp]),
}
EXPORTS = tuple(_SIGNATURES)


class S24Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library.  Raises if libs24.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2404_01847_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        handle = C.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def strerror(status: int) -> str:
    return lib().s24_strerror(status).decode()


def _check(status: int, where: str):
    if status != 0:
        raise S24Error(status, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _dense(where: str, **tensors):
    """The C signatures carry no strides for these operands: a view with gaps (a column slice of a wider buffer, a
    transposed tensor) would be read as if it were dense and give wrong numbers, so it is refused here."""
    for name, t in tensors.items():
        if t is not None and not t.is_contiguous():
            raise ValueError(f"{where}: {name} must be a contiguous tensor (shape {tuple(t.shape)}, strides {t.stride()}); "
                             "this entry point takes no leading dimension")


def _rows(where: str, **tensors):
    """Operands that travel with a leading dimension: the last axis must have unit stride."""
    for name, t in tensors.items():
        if t is not None and t.dim() >= 1 and t.stride(-1) != 1 and t.shape[-1] > 1:
            raise ValueError(f"{where}: {name} needs unit stride along its last axis (strides {t.stride()})")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"s24 supports float32, float16 and bfloat16 tensors, got {t.dtype}")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def pattern_table():
    out = (C.c_uint16 * 90)()
    _check(lib().s24_pattern_table(C.cast(out, C.c_void_p)), "s24_pattern_table")
    return list(out)


def transposable_mask(W, mask, index=None):
    _rows("s24_transposable_mask", W=W)
    _dense("s24_transposable_mask", mask=mask, index=index)
    r, q = W.shape
    _check(lib().s24_transposable_mask(_ptr(W), _dt(W), r, q, W.stride(0), _ptr(mask), _ptr(index), _stream()),
           "s24_transposable_mask")
    return mask


def compress(W, mask, vals, meta, valsT, metaT, mask_out=None):
    _rows("s24_compress", W=W)
    _dense("s24_compress", mask=mask, vals=vals, meta=meta, valsT=valsT, metaT=metaT, mask_out=mask_out)
    r, q = W.shape
    _check(lib().s24_compress(_ptr(W), _dt(W), r, q, W.stride(0), _ptr(mask), _ptr(vals), _ptr(meta), _ptr(valsT),
                              _ptr(metaT), _ptr(mask_out), _stream()), "s24_compress")


def spmm_fwd(X, vals, meta, Y):
    _dense("s24_spmm_fwd", X=X, vals=vals, meta=meta, Y=Y)
    p, q = X.shape
    r = vals.shape[1]          # vals is chunk-major: [q/64, r, 32]
    _check(lib().s24_spmm_fwd(_ptr(X), _ptr(vals), _ptr(meta), _ptr(Y), p, q, r, _dt(X), _stream()), "s24_spmm_fwd")
    return Y


def spmm_fwd_bias(X, vals, meta, bias, Y):
    """Y = X (M.*W)^T + bias; bias [r] in the dtype of X, or None."""
    _dense("s24_spmm_fwd_bias", X=X, vals=vals, meta=meta, bias=bias, Y=Y)
    p, q = X.shape
    r = vals.shape[1]
    _check(lib().s24_spmm_fwd_bias(_ptr(X), _ptr(vals), _ptr(meta), _ptr(bias), _ptr(Y), p, q, r, _dt(X), _stream()),
           "s24_spmm_fwd_bias")
    return Y


def spmm_fwd_glu(X, vals, meta, bias, GU, H, gate):
    """spmm_fwd_swiglu for either gate (GATE_SILU / GATE_GELU_ERF) and an optional stacked bias [2f]."""
    _dense("s24_spmm_fwd_glu", X=X, vals=vals, meta=meta, bias=bias, GU=GU, H=H)
    p, q = X.shape
    f = vals.shape[1] // 2
    _check(lib().s24_spmm_fwd_glu(_ptr(X), _ptr(vals), _ptr(meta), _ptr(bias), _ptr(GU), _ptr(H), p, q, f, gate, _dt(X),
                                  _stream()), "s24_spmm_fwd_glu")
    return GU, H


def spmm_bwd_dx_glu(dY, valsT, metaT, GU, dGU, gate):
    _dense("s24_spmm_bwd_dx_glu", dY=dY, valsT=valsT, metaT=metaT, GU=GU, dGU=dGU)
    p, r = dY.shape
    f = valsT.shape[1]
    _check(lib().s24_spmm_bwd_dx_glu(_ptr(dY), _ptr(valsT), _ptr(metaT), _ptr(GU), _ptr(dGU), p, f, r, gate, _dt(dY),
                                     _stream()), "s24_spmm_bwd_dx_glu")
    return dGU


def _ld(t, layout):
    """Leading dimension of a 2-D tensor that stores a logical [p][n] matrix: a column-major matrix is passed as
    the [n, p] tensor holding it, so the stride of the first axis is the leading dimension either way."""
    return t.stride(0)


def glu_fwd(Z, H, gate, layout_z=ROW_MAJOR, layout_h=ROW_MAJOR):
    """H = act(Z_1) .* Z_2.  Z: [p, 2f] tensor (row-major) or the [2f, p] tensor that holds a column-major Z;
    H likewise [p, f] or [f, p]."""
    _rows("s24_glu_fwd", Z=Z, H=H)
    p, f = (H.shape[1], H.shape[0]) if layout_h == COL_MAJOR else H.shape
    _check(lib().s24_glu_fwd(_ptr(Z), layout_z, _ld(Z, layout_z), _ptr(H), layout_h, _ld(H, layout_h), p, f, gate, _dt(Z),
                             _stream()), "s24_glu_fwd")
    return H


def glu_bwd(dH, Z, dZ, gate, layout_h=ROW_MAJOR, layout_z=ROW_MAJOR):
    """dZ (shaped and laid out like Z) from dH ([p, f], or [f, p] for a column-major dH)."""
    _rows("s24_glu_bwd", dH=dH, Z=Z, dZ=dZ)
    if dZ.stride() != Z.stride():
        raise ValueError("s24_glu_bwd: dZ must have the strides of Z")
    p, f = (dH.shape[1], dH.shape[0]) if layout_h == COL_MAJOR else dH.shape
    _check(lib().s24_glu_bwd(_ptr(dH), layout_h, _ld(dH, layout_h), _ptr(Z), layout_z, _ld(Z, layout_z), _ptr(dZ), p, f,
                             gate, _dt(Z), _stream()), "s24_glu_bwd")
    return dZ


def bias_grad(dZ, db, beta=0.0, layout=ROW_MAJOR):
    """db [n] (float32) = beta*db + column sums of the logical [p][n] matrix dZ ([n, p] tensor if column-major)."""
    _rows("s24_bias_grad", dZ=dZ)
    _dense("s24_bias_grad", db=db)
    p, n = (dZ.shape[1], dZ.shape[0]) if layout == COL_MAJOR else dZ.shape
    _check(lib().s24_bias_grad(_ptr(dZ), layout, _ld(dZ, layout), p, n, _ptr(db), beta, _dt(dZ), _stream()),
           "s24_bias_grad")
    return db


def spmm_fwd_act(X, vals, meta, bias, Z, H, act):
    """Z = X (M.*W)^T + bias (bias may be None) and H = act(Z) in one pass."""
    _dense("s24_spmm_fwd_act", X=X, vals=vals, meta=meta, bias=bias, Z=Z, H=H)
    p, q = X.shape
    r = vals.shape[1]
    _check(lib().s24_spmm_fwd_act(_ptr(X), _ptr(vals), _ptr(meta), _ptr(bias), _ptr(Z), _ptr(H), p, q, r, act, _dt(X),
                                  _stream()), "s24_spmm_fwd_act")
    return Z, H


def spmm_bwd_dx_act(dY, valsT, metaT, Z, dZ, act):
    """dZ = (dY (M.*W_2)) .* act'(Z); raises S24Error with status -6 for shapes that only the two-call route covers."""
    _dense("s24_spmm_bwd_dx_act", dY=dY, valsT=valsT, metaT=metaT, Z=Z, dZ=dZ)
    p, r = dY.shape
    f = valsT.shape[1]
    _check(lib().s24_spmm_bwd_dx_act(_ptr(dY), _ptr(valsT), _ptr(metaT), _ptr(Z), _ptr(dZ), p, f, r, act, _dt(dY),
                                     _stream()), "s24_spmm_bwd_dx_act")
    return dZ


def spmm_fwd_swiglu(X, vals, meta, GU, H):
    """vals/meta: the stacked [W_gate; W_up] compressed; GU [p, 2f] (its halves are G and U), H [p, f]."""
    _dense("s24_spmm_fwd_swiglu", X=X, vals=vals, meta=meta, GU=GU, H=H)
    p, q = X.shape
    f = vals.shape[1] // 2
    _check(lib().s24_spmm_fwd_swiglu(_ptr(X), _ptr(vals), _ptr(meta), _ptr(GU), _ptr(H), p, q, f, _dt(X), _stream()),
           "s24_spmm_fwd_swiglu")
    return GU, H


def spmm_bwd_dx(dY, valsT, metaT, dX, beta=0.0):
    _dense("s24_spmm_bwd_dx", dY=dY, valsT=valsT, metaT=metaT, dX=dX)
    p, r = dY.shape
    q = valsT.shape[1]         # valsT is chunk-major: [r/64, q, 32]
    _check(lib().s24_spmm_bwd_dx(_ptr(dY), _ptr(valsT), _ptr(metaT), _ptr(dX), p, q, r, beta, _dt(dY), _stream()),
           "s24_spmm_bwd_dx")
    return dX


def spmm_bwd_dx_swiglu(dY, valsT, metaT, GU, dGU):
    """dGU [p, 2f] from dY [p, r], the compressed transpose of the down weight and GU [p, 2f]; raises S24Error
    with status -6 (unsupported) for shapes that only the two-call route covers."""
    _dense("s24_spmm_bwd_dx_swiglu", dY=dY, valsT=valsT, metaT=metaT, GU=GU, dGU=dGU)
    p, r = dY.shape
    f = valsT.shape[1]
    _check(lib().s24_spmm_bwd_dx_swiglu(_ptr(dY), _ptr(valsT), _ptr(metaT), _ptr(GU), _ptr(dGU), p, f, r, _dt(dY),
                                        _stream()), "s24_spmm_bwd_dx_swiglu")
    return dGU


def dense_dw(dY, X, dW, beta=0.0):
    _dense("s24_dense_dw", dY=dY, X=X, dW=dW)
    p, r = dY.shape
    q = X.shape[1]
    _check(lib().s24_dense_dw(_ptr(dY), _ptr(X), _ptr(dW), p, q, r, beta, _dt(X), _stream()), "s24_dense_dw")
    return dW


def dense_dw_decay(dY, X, dW, W, mask, lam, beta=0.0):
    _dense("s24_dense_dw_decay", dY=dY, X=X, dW=dW, W=W, mask=mask)
    p, r = dY.shape
    q = X.shape[1]
    _check(lib().s24_dense_dw_decay(_ptr(dY), _ptr(X), _ptr(dW), _ptr(W), _dt(W), _ptr(mask), lam, p, q, r, beta,
                                    _dt(X), _stream()), "s24_dense_dw_decay")
    return dW


class _DwProblem(C.Structure):
    _fields_ = [("dY", _vp), ("X", _vp), ("dW", _vp), ("W", _vp), ("mask", _vp), ("p", _i64), ("q", _i64), ("r", _i64),
                ("lam", _f32)]


def dense_dw_batch(problems, beta=0.0):
    """problems: up to four tuples (dY, X, dW, W, mask, lam) with W and mask None for no decay term; the weight
    gradients of all of them in one pass (same bits as dense_dw_decay / dense_dw on each)."""
    arr = (_DwProblem * len(problems))()
    for k, (dY, X, dW, W, mask, lam) in enumerate(problems):
        p, r = dY.shape
        _dense("s24_dense_dw_batch", dY=dY, X=X, dW=dW, W=W, mask=mask)
        arr[k] = _DwProblem(_ptr(dY), _ptr(X), _ptr(dW), _ptr(W), _ptr(mask), p, X.shape[1], r, lam)
    _check(lib().s24_dense_dw_batch(C.cast(arr, C.c_void_p), len(problems), beta, _dt(problems[0][0]), _stream()),
           "s24_dense_dw_batch")


def mvue24(dY, seed, vals, meta):
    """vals [p/64, r, 32] (dtype of dY) and meta [p/64, r, 4]: the unbiasedly 2:4-pruned dY^T, compressed."""
    _rows("s24_mvue24", dY=dY)
    _dense("s24_mvue24", vals=vals, meta=meta)
    p, r = dY.shape
    _check(lib().s24_mvue24(_ptr(dY), _dt(dY), p, r, dY.stride(0), seed & 0xFFFFFFFF, _ptr(vals), _ptr(meta), _stream()),
           "s24_mvue24")
    return vals, meta


def spmm_dw(vals, meta, X, dW, beta=0.0, W=None, mask=None, lam=0.0):
    _dense("s24_spmm_dw", vals=vals, meta=meta, X=X, dW=dW, W=W, mask=mask)
    p, q = X.shape
    r = vals.shape[1]          # vals is chunk-major: [p/64, r, 32]
    _check(lib().s24_spmm_dw(_ptr(vals), _ptr(meta), _ptr(X), _ptr(dW), _ptr(W), _dt(W) if W is not None else _dt(X),
                             _ptr(mask), lam, p, q, r, beta, _dt(X), _stream()), "s24_spmm_dw")
    return dW


def dense_gemm(X, W, Y):
    _dense("s24_dense_gemm", X=X, W=W, Y=Y)
    p, q = X.shape
    r = W.shape[0]
    _check(lib().s24_dense_gemm(_ptr(X), _ptr(W), _ptr(Y), p, q, r, _dt(X), _stream()), "s24_dense_gemm")
    return Y


def masked_decay_grad(G, W, mask, lam):
    _dense("s24_masked_decay_grad", G=G, W=W, mask=mask)
    r, q = W.shape
    _check(lib().s24_masked_decay_grad(_ptr(G), _ptr(W), _dt(W), _ptr(mask), lam, r, q, _stream()),
           "s24_masked_decay_grad")
    return G


def swiglu_fwd(G, U, H):
    _rows("s24_swiglu_fwd", G=G, U=U)
    _dense("s24_swiglu_fwd", H=H)
    if U.stride(0) != G.stride(0):
        raise ValueError("s24_swiglu_fwd: G and U share one row stride (ld_gu)")
    p, f = G.shape
    _check(lib().s24_swiglu_fwd(_ptr(G), _ptr(U), _ptr(H), p, f, G.stride(0), _dt(G), _stream()), "s24_swiglu_fwd")
    return H


def swiglu_bwd(dH, G, U, dG, dU):
    _rows("s24_swiglu_bwd", G=G, U=U, dG=dG, dU=dU)
    _dense("s24_swiglu_bwd", dH=dH)
    if not (U.stride(0) == G.stride(0) == dG.stride(0) == dU.stride(0)):
        raise ValueError("s24_swiglu_bwd: G, U, dG and dU share one row stride (ld_gu)")
    p, f = G.shape
    _check(lib().s24_swiglu_bwd(_ptr(dH), _ptr(G), _ptr(U), _ptr(dG), _ptr(dU), p, f, G.stride(0), _dt(G), _stream()),
           "s24_swiglu_bwd")
    return dG, dU


def act_fwd(Z, H, act):
    _dense("s24_act_fwd", Z=Z, H=H)
    _check(lib().s24_act_fwd(_ptr(Z), _ptr(H), Z.numel(), act, _dt(Z), _stream()), "s24_act_fwd")
    return H


def act_bwd(dH, Z, dZ, act):
    _dense("s24_act_bwd", dH=dH, Z=Z, dZ=dZ)
    _check(lib().s24_act_bwd(_ptr(dH), _ptr(Z), _ptr(dZ), Z.numel(), act, _dt(Z), _stream()), "s24_act_bwd")
    return dZ


def mask_flips(mask_new, mask_old, flips, block_flips=None):
    """flips: int64 tensor of one element (overwritten); block_flips: int32 tensor, one per block (added to)."""
    _dense("s24_mask_flips", mask_new=mask_new, mask_old=mask_old, flips=flips, block_flips=block_flips)
    _check(lib().s24_mask_flips(_ptr(mask_new), _ptr(mask_old), mask_new.numel(), _ptr(block_flips), _ptr(flips),
                                _stream()), "s24_mask_flips")
    return flips


def l1_norm_gap(W, gap):
    _rows("s24_l1_norm_gap", W=W)
    _dense("s24_l1_norm_gap", gap=gap)
    r, q = W.shape
    _check(lib().s24_l1_norm_gap(_ptr(W), _dt(W), r, q, W.stride(0), _ptr(gap), _stream()), "s24_l1_norm_gap")
    return gap


def set_clock_probe(buf):
    """buf: int64 tensor of two elements on the GPU, or None to switch the probe off."""
    _check(lib().s24_set_clock_probe(_ptr(buf)), "s24_set_clock_probe")


def probe_matrix_rate(sparse, workgroups, iters, sink):
    """Register-only matrix-core loop: workgroups x 8 waves x 4*iters instructions; sink: float32 [workgroups*512]."""
    _dense("s24_probe_matrix_rate", sink=sink)
    if sink.numel() < workgroups * 512:
        raise ValueError("s24_probe_matrix_rate: sink needs workgroups * 512 floats")
    _check(lib().s24_probe_matrix_rate(int(bool(sparse)), workgroups, iters, _ptr(sink), _stream()), "s24_probe_matrix_rate")


def probe_copy(src, dst):
    """Plain device copy of src into dst (same byte size, a multiple of 16)."""
    _dense("s24_probe_copy", src=src, dst=dst)
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("s24_probe_copy: sizes differ")
    _check(lib().s24_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream()), "s24_probe_copy")
