"""s24: the 2:4-sparse FFN training step of arXiv 2404.01847 for AMD MI355X.

The product is the C-ABI library libs24.so (include/s24.h); this package is a
thin ctypes binding with the same names.  Importing it loads nothing: the
library is opened on first use and a missing library is an error, never a
fallback.
"""
from .binding import (  # noqa: F401
    S24Error, lib, lib_path, strerror, pattern_table,
    transposable_mask, compress, spmm_fwd, spmm_fwd_swiglu, spmm_bwd_dx, spmm_bwd_dx_swiglu, dense_dw, dense_dw_decay, dense_dw_batch, dense_gemm, mvue24, spmm_dw,
    masked_decay_grad, swiglu_fwd, swiglu_bwd, act_fwd, act_bwd, set_clock_probe, mask_flips, l1_norm_gap,
    spmm_fwd_act, spmm_bwd_dx_act, spmm_fwd_bias, spmm_fwd_glu, spmm_bwd_dx_glu, glu_fwd, glu_bwd, bias_grad, probe_matrix_rate, probe_copy,
    F32, BF16, F16, ACT_RELU, ACT_GELU_ERF, GATE_SILU, GATE_GELU_ERF, ROW_MAJOR, COL_MAJOR,
)
