"""CPU-side checks of the HIP library: it loads without a GPU, exports every
symbol include/s24.h declares, and rejects bad arguments on the host before
anything is launched.  No kernel runs here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2404_01847_amd as s24
    if not os.path.exists(s24.lib_path()):
        from paper_2404_01847_amd.build import build
        build(verbose=False)
    return s24.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "s24.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(s24_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), n
    from paper_2404_01847_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_pattern_table_is_the_lexicographic_enumeration(lib, legal_blocks):
    import paper_2404_01847_amd as s24
    assert s24.pattern_table() == legal_blocks


def test_strerror_covers_all_codes(lib):
    import paper_2404_01847_amd as s24
    texts = {s24.strerror(c) for c in range(0, -7, -1)}
    assert len(texts) == 7 and "ok" in texts
    assert "unknown" in s24.strerror(-99)


OK, NULL, SHAPE, DTYPE, ALIGN, UNSUP = 0, -1, -2, -3, -4, -6
P = 0x1000  # a fake, well-aligned device address: validation never dereferences it


def test_mask_argument_errors(lib):
    f = lib.s24_transposable_mask
    assert f(None, 1, 8, 8, 8, P, None, None) == NULL
    assert f(P, 1, 8, 8, 8, None, None, None) == NULL
    assert f(P, 7, 8, 8, 8, P, None, None) == DTYPE
    assert f(P, 1, 6, 8, 8, P, None, None) == SHAPE
    assert f(P, 1, 8, 10, 12, P, None, None) == SHAPE
    assert f(P, 1, -4, 8, 8, P, None, None) == SHAPE
    assert f(P, 1, 8, 8, 4, P, None, None) == SHAPE          # ldw < q
    assert f(P + 2, 1, 8, 8, 8, P, None, None) == ALIGN
    assert f(P, 1, 8, 8, 10, P, None, None) == ALIGN          # row stride not a multiple of 8 bytes
    assert f(P + 8, 0, 8, 8, 8, P, None, None) == ALIGN       # fp32 rows need 16 bytes
    assert f(P, 1, 0, 8, 8, P, None, None) == OK              # empty: nothing to do


def test_compress_argument_errors(lib):
    f = lib.s24_compress
    assert f(P, 1, 64, 64, 64, None, None, P, P, P, None, None) == NULL
    assert f(P, 1, 64, 96, 96, None, P, P, P, P, None, None) == SHAPE    # q not a multiple of 64
    assert f(P, 1, 16, 64, 64, None, P, P, P, P, None, None) == SHAPE    # r not a multiple of 64
    assert f(P, 1, 64, 64, 64, None, P + 4, P, P, P, None, None) == ALIGN
    assert f(P, 1, 0, 64, 64, None, P, P, P, P, None, None) == OK


def test_gemm_argument_errors(lib):
    assert lib.s24_spmm_fwd(P, P, P, P, 4, 96, 16, 1, None) == SHAPE          # q % 64
    assert lib.s24_spmm_fwd(P, P, P, P, 4, 64, 24, 1, None) == SHAPE          # r % 16
    assert lib.s24_spmm_fwd(P, P, None, P, 4, 64, 16, 1, None) == NULL
    assert lib.s24_spmm_fwd(P, P, P, P + 2, 4, 64, 16, 1, None) == ALIGN
    assert lib.s24_spmm_fwd(P, P, P, P, 4, 64, 16, 3, None) == DTYPE
    assert lib.s24_spmm_fwd(P, P, P, P, 0, 64, 16, 1, None) == OK
    assert lib.s24_spmm_fwd_swiglu(P, P, P, P, P, 4, 96, 16, 1, None) == SHAPE      # q % 64
    assert lib.s24_spmm_fwd_swiglu(P, P, P, P, P, 4, 64, 24, 1, None) == SHAPE      # f % 16
    assert lib.s24_spmm_fwd_swiglu(P, P, P, P, None, 4, 64, 16, 1, None) == NULL
    assert lib.s24_spmm_fwd_swiglu(P, P, P, P, P, 0, 64, 16, 1, None) == OK
    assert lib.s24_spmm_bwd_dx_swiglu(P, P, P, P, P, 4, 16, 96, 1, None) == SHAPE   # r % 64
    assert lib.s24_spmm_bwd_dx_swiglu(P, P, P, None, P, 4, 16, 64, 1, None) == NULL
    assert lib.s24_spmm_bwd_dx_swiglu(P, P, P, P, P, 4, 16, 64, 1, None) == UNSUP   # too few tiles for the fused kernel
    assert lib.s24_spmm_bwd_dx_swiglu(P, P, P, P, P, 4, 16, 64, 0, None) == UNSUP   # fp32
    assert lib.s24_spmm_bwd_dx(P, P, P, P, 4, 16, 96, 0.0, 1, None) == SHAPE  # r % 64
    assert lib.s24_spmm_bwd_dx(P, P, P, P, 4, 16, 64, 0.5, 1, None) == UNSUP  # beta must be 0 or 1
    assert lib.s24_dense_dw(P, P, P, 4, 24, 16, 0.0, 1, None) == SHAPE
    assert lib.s24_dense_dw(P, P, P, 4, 16, 16, 2.0, 1, None) == UNSUP
    assert lib.s24_dense_dw(P, None, P, 4, 16, 16, 0.0, 1, None) == NULL
    assert lib.s24_dense_dw_decay(P, P, P, P, 1, P, 1e-4, 4, 24, 16, 0.0, 1, None) == SHAPE
    assert lib.s24_dense_dw_decay(P, P, P, None, 1, P, 1e-4, 4, 16, 16, 0.0, 1, None) == NULL
    assert lib.s24_dense_dw_decay(P, P, P, P, 7, P, 1e-4, 4, 16, 16, 0.0, 1, None) == DTYPE
    assert lib.s24_dense_dw_decay(P, P, P, P, 1, P + 2, 1e-4, 4, 16, 16, 0.0, 1, None) == ALIGN
    assert lib.s24_dense_dw_decay(P, P, P, P, 1, P, 1e-4, 4, 16, 0, 0.0, 1, None) == OK
    assert lib.s24_dense_gemm(P, P, P, 4, 32, 16, 1, None) == SHAPE
    assert lib.s24_dense_gemm(P, P, P, 0, 64, 16, 1, None) == OK
    # feature extents at or beyond 2^23 (32-bit byte offsets inside a tile) and token counts at or beyond 2^31
    big = 1 << 23
    assert lib.s24_spmm_fwd(P, P, P, P, 4, big, 16, 1, None) == SHAPE
    assert lib.s24_spmm_fwd(P, P, P, P, 4, 64, big, 1, None) == SHAPE
    assert lib.s24_spmm_bwd_dx(P, P, P, P, 4, big, 64, 0.0, 1, None) == SHAPE
    assert lib.s24_dense_dw(P, P, P, 4, big, 16, 0.0, 1, None) == SHAPE
    assert lib.s24_dense_gemm(P, P, P, 1 << 31, 64, 16, 1, None) == SHAPE
    # the compressed operands' alignment is what the kernels' 16- and 8-byte stores need
    assert lib.s24_compress(P, 1, 64, 64, 64, None, P + 8, P, P, P, None, None) == ALIGN
    assert lib.s24_compress(P, 1, 64, 64, 64, None, P, P + 2, P, P, None, None) == ALIGN
    assert lib.s24_compress(P, 1, 64, 64, 64, None, P, P, P, P + 4, None, None) == ALIGN


def test_probe_argument_errors(lib):
    assert lib.s24_probe_matrix_rate(0, -1, 8, P, None) == SHAPE
    assert lib.s24_probe_matrix_rate(1, 4, 8, None, None) == NULL
    assert lib.s24_probe_matrix_rate(0, 0, 8, None, None) == OK
    assert lib.s24_probe_copy(P, P, 24, None) == SHAPE
    assert lib.s24_probe_copy(P, None, 32, None) == NULL
    assert lib.s24_probe_copy(P + 4, P, 32, None) == ALIGN
    assert lib.s24_probe_copy(None, None, 0, None) == OK


def test_mvue_argument_errors(lib):
    assert lib.s24_mvue24(P, 1, 96, 16, 16, 1, P, P, None) == SHAPE            # p % 64
    assert lib.s24_mvue24(P, 1, 64, 16, 8, 1, P, P, None) == SHAPE             # ld < r
    assert lib.s24_mvue24(P, 4, 64, 16, 16, 1, P, P, None) == DTYPE
    assert lib.s24_mvue24(P, 1, 64, 16, 16, 1, None, P, None) == NULL
    assert lib.s24_mvue24(P, 1, 64, 16, 16, 1, P + 8, P, None) == ALIGN
    assert lib.s24_mvue24(P, 1, 0, 16, 16, 1, None, None, None) == OK
    assert lib.s24_spmm_dw(P, P, P, P, None, 1, None, 0.0, 96, 16, 16, 0.0, 1, None) == SHAPE
    assert lib.s24_spmm_dw(P, P, P, P, None, 1, None, 0.0, 64, 16, 16, 0.5, 1, None) == UNSUP
    assert lib.s24_spmm_dw(P, None, P, P, None, 1, None, 0.0, 64, 16, 16, 0.0, 1, None) == NULL
    assert lib.s24_spmm_dw(P, P, P, P, P, 1, None, 1e-4, 64, 16, 16, 0.0, 1, None) == NULL    # decay without a mask
    assert lib.s24_spmm_dw(P, P, P, P, None, 1, None, 0.0, 64, 16, 0, 0.0, 1, None) == OK


def test_monitor_argument_errors(lib):
    assert lib.s24_mask_flips(P, P, -1, None, P, None) == SHAPE
    assert lib.s24_mask_flips(P, P, 16, None, None, None) == NULL
    assert lib.s24_mask_flips(P, P, 16, None, P + 4, None) == ALIGN
    assert lib.s24_l1_norm_gap(P, 1, 6, 8, 8, P, None) == SHAPE
    assert lib.s24_l1_norm_gap(P, 9, 8, 8, 8, P, None) == DTYPE
    assert lib.s24_l1_norm_gap(P, 1, 8, 8, 8, None, None) == NULL
    assert lib.s24_l1_norm_gap(P, 1, 0, 8, 8, None, None) == OK


def test_elementwise_argument_errors(lib):
    assert lib.s24_masked_decay_grad(P, P, 1, None, 1e-4, 16, 16, None) == NULL
    assert lib.s24_masked_decay_grad(P, P, 1, P, 1e-4, 16, 24, None) == SHAPE
    assert lib.s24_masked_decay_grad(P + 4, P, 1, P, 1e-4, 16, 16, None) == ALIGN
    assert lib.s24_masked_decay_grad(P, P, 5, P, 1e-4, 16, 16, None) == DTYPE
    assert lib.s24_swiglu_fwd(P, P, P, 4, 12, 16, 1, None) == SHAPE
    assert lib.s24_swiglu_fwd(P, P, P, 4, 16, 8, 1, None) == SHAPE            # ld < f
    assert lib.s24_swiglu_fwd(P, None, P, 4, 16, 16, 1, None) == NULL
    assert lib.s24_swiglu_bwd(P, P, P, P, None, 4, 16, 16, 1, None) == NULL
    assert lib.s24_swiglu_bwd(P, P, P, P, P + 8, 4, 16, 16, 1, None) == ALIGN
    assert lib.s24_act_fwd(P, P, 12, 0, 1, None) == SHAPE
    assert lib.s24_act_fwd(P, P, 16, 9, 1, None) == DTYPE
    assert lib.s24_act_bwd(P, P, None, 16, 0, 1, None) == NULL
    assert lib.s24_act_fwd(P, P, 0, 0, 1, None) == OK


def test_gated_family_argument_errors(lib):
    R, Cm = 0, 1
    # s24_glu_fwd(Z, lz, ldz, H, lh, ldh, p, f, gate, dt, stream)
    assert lib.s24_glu_fwd(P, R, 32, P, R, 16, 4, 12, 1, 2, None) == SHAPE             # f % 8
    assert lib.s24_glu_fwd(P, R, 24, P, R, 16, 4, 16, 1, 2, None) == SHAPE             # ldz < 2f
    assert lib.s24_glu_fwd(P, Cm, 8, P, R, 16, 4, 16, 1, 2, None) == SHAPE             # column-major needs p % 8
    assert lib.s24_glu_fwd(P, Cm, 4, P, Cm, 8, 8, 16, 1, 2, None) == SHAPE             # ldz < p
    assert lib.s24_glu_fwd(P, 2, 32, P, R, 16, 4, 16, 1, 2, None) == DTYPE             # layout enum
    assert lib.s24_glu_fwd(P, R, 32, P, R, 16, 4, 16, 5, 2, None) == DTYPE             # gate enum
    assert lib.s24_glu_fwd(P, R, 32, P, R, 16, 4, 16, 1, 3, None) == DTYPE
    assert lib.s24_glu_fwd(None, R, 32, P, R, 16, 4, 16, 1, 2, None) == NULL
    assert lib.s24_glu_fwd(P + 8, R, 32, P, R, 16, 4, 16, 1, 2, None) == ALIGN
    assert lib.s24_glu_fwd(None, R, 32, None, R, 16, 0, 16, 1, 2, None) == OK
    # s24_glu_bwd(dH, lh, ldh, Z, lz, ldz, dZ, p, f, gate, dt, stream)
    assert lib.s24_glu_bwd(P, R, 16, P, R, 32, None, 4, 16, 0, 1, None) == NULL
    assert lib.s24_glu_bwd(P, R, 8, P, R, 32, P, 4, 16, 0, 1, None) == SHAPE           # ldh < f
    assert lib.s24_glu_bwd(P, Cm, 8, P, R, 32, P, 4, 16, 0, 1, None) == SHAPE          # mixed layouts need p % 8
    assert lib.s24_glu_bwd(P, R, 16, P, R, 32, P + 2, 4, 16, 0, 1, None) == ALIGN
    # s24_bias_grad(dZ, layout, ld, p, n, db, beta, dt, stream)
    assert lib.s24_bias_grad(P, R, 16, 4, 12, P, 0.0, 1, None) == SHAPE                # n % 8
    assert lib.s24_bias_grad(P, R, 8, 4, 16, P, 0.0, 1, None) == SHAPE                 # ld < n
    assert lib.s24_bias_grad(P, Cm, 8, 4, 16, P, 0.0, 1, None) == SHAPE                # column-major needs p % 8
    assert lib.s24_bias_grad(P, R, 16, 4, 16, P, 0.5, 1, None) == UNSUP
    assert lib.s24_bias_grad(P, R, 16, 4, 16, None, 0.0, 1, None) == NULL
    assert lib.s24_bias_grad(P, R, 16, 4, 16, P + 2, 0.0, 1, None) == ALIGN
    assert lib.s24_bias_grad(P, R, 16, 4, 16, P, 0.0, 8, None) == DTYPE
    assert lib.s24_bias_grad(None, R, 16, 4, 0, None, 0.0, 1, None) == OK
    # s24_spmm_fwd_bias(X, vals, meta, bias, Y, p, q, r, dt, stream)
    assert lib.s24_spmm_fwd_bias(P, P, P, P, P, 4, 96, 16, 2, None) == SHAPE
    assert lib.s24_spmm_fwd_bias(P, P, P, P + 4, P, 4, 64, 16, 2, None) == ALIGN       # bias 8-byte aligned
    assert lib.s24_spmm_fwd_bias(P, P, None, None, P, 4, 64, 16, 2, None) == NULL
    assert lib.s24_spmm_fwd_bias(P, P, P, None, P, 0, 64, 16, 2, None) == OK
    # s24_spmm_fwd_glu(X, vals, meta, bias, GU, H, p, q, f, gate, dt, stream)
    assert lib.s24_spmm_fwd_glu(P, P, P, None, P, P, 4, 64, 24, 1, 2, None) == SHAPE   # f % 16
    assert lib.s24_spmm_fwd_glu(P, P, P, None, P, P, 4, 64, 16, 3, 2, None) == DTYPE   # gate
    assert lib.s24_spmm_fwd_glu(P, P, P, None, P, None, 4, 64, 16, 1, 2, None) == NULL
    assert lib.s24_spmm_fwd_glu(P, P, P, None, P, P, 0, 64, 16, 1, 2, None) == OK
    # s24_spmm_bwd_dx_glu(dY, valsT, metaT, GU, dGU, p, f, r, gate, dt, stream)
    assert lib.s24_spmm_bwd_dx_glu(P, P, P, P, P, 4, 16, 96, 1, 2, None) == SHAPE
    assert lib.s24_spmm_bwd_dx_glu(P, P, P, P, P, 4, 16, 64, 7, 2, None) == DTYPE
    assert lib.s24_spmm_bwd_dx_glu(P, P, P, P, P, 4, 16, 64, 1, 2, None) == UNSUP      # too few tiles
    assert lib.s24_spmm_bwd_dx_glu(P, P, P, P, P, 4, 16, 64, 1, 0, None) == UNSUP      # fp32
    # s24_spmm_fwd_act(X, vals, meta, bias, Z, H, p, q, r, act, dt, stream)
    assert lib.s24_spmm_fwd_act(P, P, P, None, P, P, 4, 96, 16, 1, 1, None) == SHAPE
    assert lib.s24_spmm_fwd_act(P, P, P, None, P, P, 4, 64, 16, 4, 1, None) == DTYPE   # activation enum
    assert lib.s24_spmm_fwd_act(P, P, P, None, P, None, 4, 64, 16, 1, 1, None) == NULL
    assert lib.s24_spmm_fwd_act(P, P, P, None, P, P, 0, 64, 16, 1, 1, None) == OK
    # s24_spmm_bwd_dx_act(dY, valsT, metaT, Z, dZ, p, f, r, act, dt, stream)
    assert lib.s24_spmm_bwd_dx_act(P, P, P, P, P, 4, 16, 96, 1, 1, None) == SHAPE
    assert lib.s24_spmm_bwd_dx_act(P, P, P, None, P, 4, 16, 64, 1, 1, None) == NULL
    assert lib.s24_spmm_bwd_dx_act(P, P, P, P, P, 4, 16, 64, 1, 0, None) == UNSUP     # fp32: the two-call route
    # s24_dense_dw_batch(problems, count, beta, dt, stream): a host array of problem records
    import ctypes
    from paper_2404_01847_amd.binding import _DwProblem
    good = _DwProblem(P, P, P, None, None, 4, 16, 16, 0.0)
    arr = (_DwProblem * 2)(good, good)
    ptr = ctypes.cast(arr, ctypes.c_void_p)
    assert lib.s24_dense_dw_batch(ptr, 5, 0.0, 1, None) == SHAPE                     # at most four problems
    assert lib.s24_dense_dw_batch(ptr, 2, 0.5, 1, None) == UNSUP
    assert lib.s24_dense_dw_batch(ptr, 2, 0.0, 9, None) == DTYPE
    assert lib.s24_dense_dw_batch(None, 2, 0.0, 1, None) == NULL
    assert lib.s24_dense_dw_batch(None, 0, 0.0, 1, None) == OK
    arr[1] = _DwProblem(P, P, P, None, None, 4, 24, 16, 0.0)
    assert lib.s24_dense_dw_batch(ptr, 2, 0.0, 1, None) == SHAPE                     # the second problem's q
    arr[1] = _DwProblem(P, None, P, None, None, 4, 16, 16, 0.0)
    assert lib.s24_dense_dw_batch(ptr, 2, 0.0, 1, None) == NULL
    arr[1] = _DwProblem(P, P, P, P, None, 4, 16, 16, 1e-4)
    assert lib.s24_dense_dw_batch(ptr, 2, 0.0, 1, None) == NULL                      # decay without a mask
    arr[0] = _DwProblem(P, P, P, None, None, 4, 16, 0, 0.0)
    arr[1] = _DwProblem(None, None, None, None, None, 4, 0, 16, 0.0)
    assert lib.s24_dense_dw_batch(ptr, 2, 0.0, 1, None) == OK                        # empty outputs: nothing to do
    # binary16 is a valid dtype everywhere a dtype is taken
    assert lib.s24_transposable_mask(P, 2, 6, 8, 8, P, None, None) == SHAPE
    assert lib.s24_spmm_fwd(P, P, P, P, 0, 64, 16, 2, None) == OK
    assert lib.s24_mvue24(P, 2, 0, 16, 16, 1, None, None, None) == OK


def test_binding_refuses_to_run_without_library(monkeypatch, tmp_path):
    from paper_2404_01847_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libs24.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()
