"""Unit-scaled linear / FFN forward and backward for AMD MI355X (gfx950).

The work is done by hand-written HIP kernels behind a C ABI (``include/us.h``, built into
``libus_mi355x.so``); this package is only the ctypes binding with the same names.  PyTorch is
used by callers for device memory and streams; the binding takes raw device pointers.
"""
from .binding import (  # noqa: F401
    ACT_GELU, ACT_RELU, ACT_SIGMOID, ACT_TANH, E4M3, E5M2, F16, F32, EPI_ACT_RELU, EPI_ACT_SIGMOID, EPI_ACT_TANH, EPI_GELU, EPI_GELU_GRAD, EPI_NONE, EPI_RESIDUAL, EPI_TABLES_READY, FFN_FP8, FFN_TABLES_READY, HIST_BINS, STATUS, TABLE_AREA_BYTES, UsError, act_bwd, act_fwd, cast_fp8, cast_snr, exponent_histogram, cast_fp8_batch, ffn_bwd, ffn_fwd,
    ffn_res_bwd, ffn_res_fwd, ffn_workspace_bytes, gelu_bwd, gelu_fwd, gelu_tables, layer_norm_bwd, layer_norm_fwd, layer_norm_workspace_bytes, lib, library_path, linear_bwd, linear_fwd, linear_scales,
    last_launch, linear_bwd_noalloc, noalloc_scratch_bytes, status_string, weighted_add, workspace_bytes, linear_bias_fwd, bias_grad, bias_grad_workspace_bytes, ffn_bias_fwd, ffn_bias_bwd,
    ffn_bias_workspace_bytes, softmax_fwd, softmax_bwd, softmax_xent, matmul_batched, attention_fwd, attention_bwd, sum_fwd, sum_bwd,
)
