"""ctypes binding of the CPU oracle (oracle/s24_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package.  It never imports the HIP
package and the HIP package never imports it.

bf16 tensors travel as numpy uint16 arrays (raw bit patterns); fp32 tensors as
float32 arrays.  Floating-point results come back as float64 arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

F32, BF16, F16 = 0, 1, 2
ACT_RELU, ACT_GELU_ERF = 0, 1
GATE_SILU, GATE_GELU_ERF = 0, 1
ROW_MAJOR, COL_MAJOR = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s24_oracle.c")
# S24_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (host code only), for a checking run of the CPU tests:
#   S24_ORACLE_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
#       python -m pytest tests/test_oracle_pins.py -q
_SANITIZE = os.environ.get("S24_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "liborc_san.so" if _SANITIZE else "liborc.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                               _SRC, "-o", _LIB, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        for name in ("orc_pack_chunk_major", "orc_pattern_table", "orc_transposable_mask", "orc_compress", "orc_spmm_fwd",
                     "orc_spmm_bwd_dx", "orc_dense_dw", "orc_dense_gemm", "orc_masked_decay",
                     "orc_swiglu_fwd", "orc_swiglu_bwd", "orc_act_fwd", "orc_act_bwd", "orc_num_threads",
                     "orc_mask_flips", "orc_l1_norm_gap", "orc_mvue24", "orc_glu_fwd", "orc_glu_bwd", "orc_bias_grad"):
            getattr(_lib, name).restype = C.c_int
        _lib.orc_round_bf16.restype = None
        _lib.orc_round_f16.restype = None
    return _lib


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"expected float32, float16 or uint16(bf16 bits), got {a.dtype}")


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _rows(rows):
    if rows is None:
        return None, 0
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    return rows, rows.size


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return _load().orc_num_threads()


def pattern_table() -> np.ndarray:
    out = np.zeros(128, dtype=np.uint16)
    n = _load().orc_pattern_table(_p(out), C.c_int(128))
    return out[:n].copy()


def transposable_mask(W: np.ndarray, want_index: bool = False, exact_wide: bool = False):
    """Block masks uint16 [r/4, q/4] (and pattern ids uint8) of the best transposable mask."""
    W = _c(W)
    r, q = W.shape
    mask = np.zeros((r // 4, q // 4), dtype=np.uint16)
    index = np.zeros((r // 4, q // 4), dtype=np.uint8) if want_index else None
    rc = _load().orc_transposable_mask(_p(W), _dt(W), C.c_int64(r), C.c_int64(q), C.c_int64(q),
                                       _p(mask), _p(index), C.c_int(1 if exact_wide else 0))
    _check(rc, "transposable_mask")
    return (mask, index) if want_index else mask


def mask_flips(mask_new, mask_old, block_flips=None) -> int:
    """Number of mask cells that differ (the flip rate's numerator); block_flips (uint32, in place) += per block."""
    a, b = _c(mask_new, np.uint16), _c(mask_old, np.uint16)
    if a.shape != b.shape:
        raise ValueError("mask shapes differ")
    if block_flips is not None and (block_flips.dtype != np.uint32 or not block_flips.flags.c_contiguous
                                    or block_flips.size != a.size):
        raise ValueError("block_flips must be a contiguous uint32 array with one entry per block")
    total = C.c_uint64(0)
    _check(_load().orc_mask_flips(_p(a), _p(b), C.c_int64(a.size), _p(block_flips), C.byref(total)), "mask_flips")
    return int(total.value)


def l1_norm_gap(W: np.ndarray) -> np.ndarray:
    """Per 4x4 block: best minus second-best kept L1 norm over the 90 patterns, float64 [r/4, q/4]."""
    W = _c(W)
    r, q = W.shape
    gap = np.zeros((r // 4, q // 4), dtype=np.float64)
    _check(_load().orc_l1_norm_gap(_p(W), _dt(W), C.c_int64(r), C.c_int64(q), C.c_int64(q), _p(gap)), "l1_norm_gap")
    return gap


def mvue24(dY: np.ndarray, seed: int):
    """Unbiased 2:4 pruning of dY^T along the tokens: vals[r, p/2] (dtype of dY), meta[r, p/16].
    dY may be a view of a wider row-major matrix (unit column stride): its row stride is passed on as it is."""
    if not (dY.ndim == 2 and dY.strides[1] == dY.itemsize and dY.strides[0] % dY.itemsize == 0
            and dY.strides[0] >= dY.shape[1] * dY.itemsize):
        dY = _c(dY)
    p, r = dY.shape
    ld = dY.strides[0] // dY.itemsize if p > 1 else r
    vals = np.zeros((r, p // 2), dtype=dY.dtype)
    meta = np.zeros((r, p // 16), dtype=np.uint16)
    rc = _load().orc_mvue24(C.c_void_p(dY.ctypes.data), _dt(dY), C.c_int64(p), C.c_int64(r), C.c_int64(ld),
                            C.c_uint32(seed & 0xFFFFFFFF), _p(vals), _p(meta))
    _check(rc, "mvue24")
    return vals, meta


def compress(W: np.ndarray, mask: np.ndarray):
    """Returns vals[r,q/2], meta[r,q/16], valsT[q,r/2], metaT[q,r/16]."""
    W = _c(W)
    mask = _c(mask, np.uint16)
    r, q = W.shape
    vals = np.zeros((r, q // 2), dtype=W.dtype)
    meta = np.zeros((r, q // 16), dtype=np.uint16)
    valsT = np.zeros((q, r // 2), dtype=W.dtype)
    metaT = np.zeros((q, r // 16), dtype=np.uint16)
    rc = _load().orc_compress(_p(W), _dt(W), C.c_int64(r), C.c_int64(q), C.c_int64(q), _p(mask),
                              _p(vals), _p(meta), _p(valsT), _p(metaT))
    _check(rc, "compress")
    return vals, meta, valsT, metaT


def pack(vals, meta):
    """Row-major compressed operand -> chunk-major storage: vals_p[K/64, R, 32], meta_p[K/64, R, 4]."""
    vals, meta = _c(vals), _c(meta, np.uint16)
    R, half = vals.shape
    K = 2 * half
    vals_p = np.zeros((K // 64, R, 32), dtype=vals.dtype)
    meta_p = np.zeros((K // 64, R, 4), dtype=np.uint16)
    rc = _load().orc_pack_chunk_major(_p(vals), _p(meta), _dt(vals), C.c_int64(R), C.c_int64(K), _p(vals_p), _p(meta_p))
    _check(rc, "pack_chunk_major")
    return vals_p, meta_p


def spmm_fwd(X, vals, meta, rows=None):
    """Y[rows, r] = X . (M*W)^T from the compressed form, fp64."""
    X, vals, meta = _c(X), _c(vals), _c(meta, np.uint16)
    p, q = X.shape
    r = vals.shape[0]
    rows, n = _rows(rows)
    Y = np.zeros((n if rows is not None else p, r), dtype=np.float64)
    rc = _load().orc_spmm_fwd(_p(X), _p(vals), _p(meta), _dt(X), C.c_int64(p), C.c_int64(q), C.c_int64(r),
                              _p(rows), C.c_int64(n), _p(Y))
    _check(rc, "spmm_fwd")
    return Y


def spmm_bwd_dx(dY, valsT, metaT, beta=0.0, dX0=None, rows=None):
    """dX[rows, q] = beta*dX0 + dY . (M*W) from the compressed transpose, fp64."""
    dY, valsT, metaT = _c(dY), _c(valsT), _c(metaT, np.uint16)
    p, r = dY.shape
    q = valsT.shape[0]
    rows, n = _rows(rows)
    if dX0 is not None:
        dX0 = _c(dX0, np.float64)
    dX = np.zeros((n if rows is not None else p, q), dtype=np.float64)
    rc = _load().orc_spmm_bwd_dx(_p(dY), _p(valsT), _p(metaT), _dt(dY), C.c_int64(p), C.c_int64(q), C.c_int64(r),
                                 C.c_double(beta), _p(dX0), _p(rows), C.c_int64(n), _p(dX))
    _check(rc, "spmm_bwd_dx")
    return dX


def dense_dw(dY, X, beta=0.0, dW0=None, rows=None):
    """dW[rows, q] = beta*dW0 + dY^T . X, fp64 (rows selects out-features)."""
    dY, X = _c(dY), _c(X)
    p, r = dY.shape
    q = X.shape[1]
    rows, n = _rows(rows)
    if dW0 is not None:
        dW0 = _c(dW0, np.float64)
    dW = np.zeros((n if rows is not None else r, q), dtype=np.float64)
    rc = _load().orc_dense_dw(_p(dY), _p(X), _dt(X), C.c_int64(p), C.c_int64(q), C.c_int64(r),
                              C.c_double(beta), _p(dW0), _p(rows), C.c_int64(n), _p(dW))
    _check(rc, "dense_dw")
    return dW


def dense_gemm(X, W, rows=None):
    """Y[rows, r] = X . W^T, fp64."""
    X, W = _c(X), _c(W)
    p, q = X.shape
    r = W.shape[0]
    rows, n = _rows(rows)
    Y = np.zeros((n if rows is not None else p, r), dtype=np.float64)
    rc = _load().orc_dense_gemm(_p(X), _p(W), _dt(X), C.c_int64(p), C.c_int64(q), C.c_int64(r),
                                _p(rows), C.c_int64(n), _p(Y))
    _check(rc, "dense_gemm")
    return Y


def masked_decay(dW, W, mask, lam):
    dW = _c(dW, np.float32)
    W, mask = _c(W), _c(mask, np.uint16)
    r, q = W.shape
    G = np.zeros((r, q), dtype=np.float64)
    rc = _load().orc_masked_decay(_p(dW), _p(W), _dt(W), _p(mask), C.c_float(lam), C.c_int64(r), C.c_int64(q), _p(G))
    _check(rc, "masked_decay")
    return G


def swiglu_fwd(G, U):
    G, U = _c(G), _c(U)
    p, f = G.shape
    H = np.zeros((p, f), dtype=np.float64)
    _check(_load().orc_swiglu_fwd(_p(G), _p(U), _dt(G), C.c_int64(p), C.c_int64(f), C.c_int64(f), _p(H)), "swiglu_fwd")
    return H


def swiglu_bwd(dH, G, U):
    dH, G, U = _c(dH), _c(G), _c(U)
    p, f = G.shape
    dG = np.zeros((p, f), dtype=np.float64)
    dU = np.zeros((p, f), dtype=np.float64)
    _check(_load().orc_swiglu_bwd(_p(dH), _p(G), _p(U), _dt(G), C.c_int64(p), C.c_int64(f), C.c_int64(f),
                                  _p(dG), _p(dU)), "swiglu_bwd")
    return dG, dU


def act_fwd(Z, act):
    Z = _c(Z)
    H = np.zeros(Z.shape, dtype=np.float64)
    _check(_load().orc_act_fwd(_p(Z), _dt(Z), C.c_int64(Z.size), C.c_int(act), _p(H)), "act_fwd")
    return H


def act_bwd(dH, Z, act):
    dH, Z = _c(dH), _c(Z)
    dZ = np.zeros(Z.shape, dtype=np.float64)
    _check(_load().orc_act_bwd(_p(dH), _p(Z), _dt(Z), C.c_int64(Z.size), C.c_int(act), _p(dZ)), "act_bwd")
    return dZ


def round_bf16(x) -> np.ndarray:
    """fp64 -> fp32 -> bf16 bits (round-to-nearest-even at each step)."""
    x = _c(x, np.float64)
    out = np.zeros(x.shape, dtype=np.uint16)
    _load().orc_round_bf16(_p(x), C.c_int64(x.size), _p(out))
    return out


def round_f16(x) -> np.ndarray:
    """fp64 -> fp32 -> binary16 (round-to-nearest-even at each step), returned as numpy float16."""
    x = _c(x, np.float64)
    out = np.zeros(x.shape, dtype=np.uint16)
    _load().orc_round_f16(_p(x), C.c_int64(x.size), _p(out))
    return out.view(np.float16)


def round_like(x, like: np.ndarray) -> np.ndarray:
    """fp64 -> the storage type of `like` (float32, float16, or uint16 holding bf16 bits)."""
    if like.dtype == np.float32:
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    return round_f16(x) if like.dtype == np.float16 else round_bf16(x)


def _strided(Z, layout):
    """(array, leading dimension) of a logical [p][n] matrix held row-major (layout 0) or column-major (1)."""
    Z = _c(Z)
    return Z, Z.shape[1]   # a column-major [p][n] matrix is passed as the [n][p] array that stores it: ld = p


def glu_fwd(Z, gate, layout=0):
    """Sec. 5.2 step 3.  Z is [p][2r] (layout 0) or its column-major storage given as the [2r][p] array (1)."""
    Z, ld = _strided(Z, layout)
    p, n = (Z.shape[1], Z.shape[0]) if layout == COL_MAJOR else Z.shape
    r = n // 2
    H = np.zeros((p, r), dtype=np.float64)
    _check(_load().orc_glu_fwd(_p(Z), _dt(Z), C.c_int(layout), C.c_int64(ld), C.c_int64(p), C.c_int64(r), C.c_int(gate),
                               _p(H)), "glu_fwd")
    return H


def glu_bwd(dH, Z, gate, layout=0, layout_h=0):
    """dZ as a dense row-major [p][2r] fp64 array; dH is [p][r] (layout_h 0) or given as [r][p] (layout_h 1)."""
    Z, ld = _strided(Z, layout)
    dH, ldh = _strided(dH, layout_h)
    p, n = (Z.shape[1], Z.shape[0]) if layout == COL_MAJOR else Z.shape
    r = n // 2
    dZ = np.zeros((p, n), dtype=np.float64)
    _check(_load().orc_glu_bwd(_p(dH), C.c_int(layout_h), C.c_int64(ldh), _p(Z), _dt(Z), C.c_int(layout), C.c_int64(ld),
                               C.c_int64(p), C.c_int64(r), C.c_int(gate), _p(dZ)), "glu_bwd")
    return dZ


def bias_grad(dZ, layout=0):
    """Column sums of the logical [p][n] matrix dZ (given as [n][p] when layout is 1)."""
    dZ, ld = _strided(dZ, layout)
    p, n = (dZ.shape[1], dZ.shape[0]) if layout == COL_MAJOR else dZ.shape
    db = np.zeros(n, dtype=np.float64)
    _check(_load().orc_bias_grad(_p(dZ), _dt(dZ), C.c_int(layout), C.c_int64(ld), C.c_int64(p), C.c_int64(n), _p(db)),
           "bias_grad")
    return db


def spmm_fwd_bias(X, vals, meta, bias, rows=None):
    """Sec. 5.2 step 2: Z = X (M.*W)^T + d, the bias widened exactly and added in fp64."""
    Y = spmm_fwd(X, vals, meta, rows)
    b = widen(bias)
    return Y + b[None, :]


def widen(a: np.ndarray) -> np.ndarray:
    """Exact fp64 values of a float32 / float16 / bf16-bits array (numpy's own conversions)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)
