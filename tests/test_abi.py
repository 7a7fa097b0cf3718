"""The C-ABI library loads and exports every entry point declared in include/us.h; host-side
argument checks answer before anything is launched (no GPU needed for any of this)."""
import ctypes
import os
import re

import pytest

import paper_2303_11257_amd as us

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "us.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(us_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"us_cast_fp8", "us_cast_fp8_batch", "us_linear_fwd", "us_linear_bwd", "us_gelu_fwd", "us_gelu_bwd", "us_linear_scales",
            "us_workspace_bytes", "us_status_string", "us_ffn_fwd", "us_ffn_bwd", "us_gelu_tables", "us_weighted_add",
            "us_ffn_res_fwd", "us_ffn_res_bwd", "us_act_fwd", "us_act_bwd", "us_layer_norm_fwd", "us_layer_norm_bwd",
            "us_layer_norm_workspace_bytes", "us_exponent_histogram", "us_cast_snr", "us_linear_bias_fwd", "us_bias_grad",
            "us_bias_grad_workspace_bytes", "us_ffn_bias_fwd", "us_ffn_bias_bwd", "us_ffn_bias_workspace_bytes", "us_softmax_fwd", "us_softmax_bwd", "us_softmax_xent", "us_matmul_batched",
            "us_attention_fwd", "us_attention_bwd", "us_sum_fwd", "us_sum_bwd", "us_last_launch", "us_linear_bwd_noalloc",
            "us_noalloc_scratch_bytes"} <= set(names)
    L = ctypes.CDLL(us.library_path())
    for n in names:
        assert hasattr(L, n), n


def test_scales_and_status_strings():
    assert us.linear_scales(256, 256, 1024) == (1 / 16, 1 / 32, 1 / 16)
    a, bx, bw = us.linear_scales(8192, 1024, 4096, 1)
    assert a == bx and abs(a - (1024 * 4096) ** -0.25) < 1e-9 and abs(bw - 8192 ** -0.5) < 1e-9
    with pytest.raises(us.UsError) as e:
        us.linear_scales(0, 4, 4)
    assert e.value.status == 2
    for code in range(8):
        assert us.status_string(code)


def test_workspace_rule():
    table_area = us.TABLE_AREA_BYTES
    assert table_area == 256 * 1024
    assert us.workspace_bytes(32768, 4096, 16384) == table_area     # the output alone fills the chip: no dW slices
    # 256 tiles of 128 x 128 cover the CUs once: the token reduction is shared by wave groups, no slices
    assert us.workspace_bytes(8192, 1024, 4096) == table_area
    assert us.workspace_bytes(4096, 768, 3072) == table_area        # 144 tiles: the wave groups again
    wb = us.workspace_bytes(4096, 512, 2048) - table_area           # 64 tiles: the token dimension is sliced
    assert wb > 0 and wb % (512 * 2048 * 4) == 0                    # whole FP32 slices of the output
    assert us.ffn_workspace_bytes(4096, 512, 2048) >= wb + table_area
    assert us.workspace_bytes(0, 16, 16) == 0
    assert us.bias_grad_workspace_bytes(8192, 4096) == 256 * 4096 * 4 and us.bias_grad_workspace_bytes(33, 16) == 2 * 16 * 4
    assert us.ffn_bias_workspace_bytes(8192, 1024, 4096) == table_area + 256 * 4096 * 4
    assert us.ffn_bias_workspace_bytes(4096, 512, 2048) == us.ffn_workspace_bytes(4096, 512, 2048) + 128 * 2048 * 4   # behind the dW slices
    assert us.ffn_bias_workspace_bytes(4096, 768, 3072) == table_area + 128 * 3072 * 4               # no slices: the bias partials
    assert us.layer_norm_workspace_bytes(8192, 1024) == 256 * 2 * 1024 * 4 and us.layer_norm_workspace_bytes(33, 16) == 2 * 2 * 16 * 4


def test_argument_errors_are_detected_on_the_host():
    F16, F32, E4, E5 = us.F16, us.F32, us.E4M3, us.E5M2
    cases = [
        (lambda: us.cast_fp8(16, F16, 32, F16, 4), 4),               # destination must be FP8
        (lambda: us.cast_fp8(None, F16, 32, E4, 4), 1),
        (lambda: us.cast_fp8(24, F16, 32, E4, 4), 3),
        (lambda: us.gelu_fwd(16, 32, 8, E4), 4),
        (lambda: us.gelu_bwd(16, None, 32, 8, F16), 1),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 24, F16, F16), 2),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, E4), 4),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, E4, E4, E4), 4),        # FP8 output of a matmul
        (lambda: us.linear_fwd(16, 16, None, 16, 16, 16, F16, F16), 1),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_GELU), 1),   # no aux buffer
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F32, 0.0, us.EPI_GELU, 0.0, 16), 4),
        (lambda: us.linear_bwd(16, 16, 16, 16, 16, 16, 16, 16, E4, E4, E4), 4),   # gradients are E5M2
        (lambda: us.linear_bwd(16, 16, 16, 16, 16, 4096, 512, 2048, F16, F16, F16), 5),   # workspace missing
        (lambda: us.linear_bwd(16, 16, 16, 16, None, 16, 16, 16, F16, F16, F16, F16, 0, 0, us.EPI_GELU_GRAD), 1),
        (lambda: us.linear_bwd(16, 16, 8, 16, 16, 16, 16, 16, F16, F16, F16), 3),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_RESIDUAL, 0.5), 1),          # no skip input
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_RESIDUAL, 1.5, 16), 7),     # weight > 1
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_RESIDUAL, 0.0, 16), 7),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F32, 0.0, us.EPI_RESIDUAL, 0.5, 16), 4),
        (lambda: us.linear_bwd(16, 16, 16, 16, 16, 16, 16, 16, F16, F16, F16, F16, 0, 0, us.EPI_RESIDUAL, 0.5), 1),
        (lambda: us.linear_bwd(16, 16, 16, 16, 16, 16, 16, 16, F16, F16, F16, F16, 0, 0, us.EPI_RESIDUAL, -1.0, 16), 7),
        (lambda: us.act_fwd(16, 32, 8, F16, 4), 4),                                                          # unknown activation
        (lambda: us.act_bwd(16, None, 32, 8, F16, us.ACT_RELU), 1),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_NONE | us.EPI_ACT_RELU), 4),  # kind without an activation epilogue
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_GELU | 0x40, 0.0, 16), 4),
        (lambda: us.layer_norm_fwd(16, 16, 16, 16, 4, 24), 2),                                               # n not a multiple of 16
        (lambda: us.layer_norm_fwd(16, 16, 16, 16, 4, 8192), 2),                                             # row too long
        (lambda: us.layer_norm_fwd(16, 16, None, 16, 4, 32), 1),
        (lambda: us.layer_norm_fwd(16, 16, 16, 16, 4, 32, -1.0), 7),
        (lambda: us.layer_norm_bwd(16, 16, 16, 16, 16, 16, 64, 32, 0.0, 0.0, 16, 100), 5),                   # workspace too small
        (lambda: us.exponent_histogram(16, E4, 8, 64), 4),
        (lambda: us.exponent_histogram(16, F16, 8, None), 1),
        (lambda: us.cast_snr(16, F32, 8, E4, 0.0, 64), 7),                                                   # scale must be positive
        (lambda: us.cast_snr(16, F32, 8, F16, 1.0, 64), 4),
        (lambda: us.weighted_add(16, None, 32, 8), 1),
        (lambda: us.weighted_add(16, 16, 32, 8, E4), 4),
        (lambda: us.ffn_res_fwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 0.0, 0), 7),                          # tau must be in (0, 1]
        (lambda: us.ffn_res_bwd(16, 16, 16, 16, 16, 16, 16, 16, None, 16, 16, 16, 16, 16, 16, 1.5, 0), 7),
        (lambda: us.linear_bias_fwd(16, 16, 16, 16, 16, 16, 16, F16, F16, F32), 4),                          # bias needs an FP16 result
        (lambda: us.linear_bias_fwd(16, 16, 8, 16, 16, 16, 16, F16, F16), 3),
        (lambda: us.bias_grad(16, F32, 16, 32, 32, 0.0, 16, 1 << 20), 4),
        (lambda: us.bias_grad(16, F16, 16, 32, 24, 0.0, 16, 1 << 20), 2),
        (lambda: us.bias_grad(16, F16, None, 32, 32, 0.0, 16, 1 << 20), 1),
        (lambda: us.bias_grad(16, F16, 16, 32, 32, 0.0, 16, 100), 5),
        (lambda: us.ffn_bias_bwd(16, 16, 16, 16, 16, 16, 16, None, 16, 16, 16, 16, 16, 16, 16, 16, 16, 0, 16, 1 << 20), 1),  # FP16 step without dZ16
        (lambda: us.ffn_bias_bwd(16, 16, 16, 16, 16, 16, None, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 0, 16, 1 << 20), 1),          # db2 without G16
        (lambda: us.ffn_bias_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 64, 16, 16, 0, 16, 1000), 5),
        (lambda: us.softmax_fwd(16, 16, 4, 12), 2),                                                        # s not a multiple of 8
        (lambda: us.softmax_fwd(16, 16, 4, 8192), 2),                                                      # row too long
        (lambda: us.softmax_fwd(16, None, 4, 64), 1),
        (lambda: us.softmax_fwd(16, 16, 4, 64, -1.0), 7),
        (lambda: us.softmax_bwd(16, 16, 24, 4, 64), 3),
        (lambda: us.softmax_xent(16, 16, None, None, 4, 64), 1),                                           # neither output
        (lambda: us.softmax_xent(16, 18, 16, 16, 4, 64), 3),                                               # targets not 4-byte aligned
        (lambda: us.softmax_xent(16, 16, 16, 16, 4, 65544), 2),
        (lambda: us.matmul_batched(16, 16, 16, 2, 16, 16, 16, 1, 1, F16, F16, F16, 1.0), 2),               # both transposed
        (lambda: us.matmul_batched(16, 16, 16, 2, 16, 16, 16, 0, 1, E4, E4, F16, 1.0), 4),                 # not one of the FP8 pairs
        (lambda: us.matmul_batched(16, 16, 16, 70000, 16, 16, 16, 0, 0, F16, F16, F16, 1.0), 2),
        (lambda: us.matmul_batched(16, 16, 16, 2, 16, 16, 16, 0, 0, F16, F16, F16, 0.0), 7),
        (lambda: us.matmul_batched(16, None, 16, 2, 16, 16, 16, 0, 0, F16, F16, F16, 1.0), 1),
        (lambda: us.attention_fwd(16, 16, 16, 16, 16, 16, 2, 8192, 64), 2),                                # rows longer than the softmax takes
        (lambda: us.attention_fwd(16, 16, 16, 16, None, 16, 2, 64, 64), 1),
        (lambda: us.attention_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 16, None, 2, 64, 64), 1),
        (lambda: us.sum_fwd(16, 16, 4, 12), 2),
        (lambda: us.sum_fwd(16, None, 4, 16), 1),
        (lambda: us.sum_bwd(16, 24, 4, 16), 3),
        (lambda: us.gelu_tables(None, 1 << 20), 1),
        (lambda: us.gelu_tables(16, 1000), 5),                       # smaller than the table area
        (lambda: us.gelu_tables(24, 1 << 20), 3),
        (lambda: us.linear_fwd(16, 16, 16, 16, 16, 16, F16, F16, F16, 0.0, us.EPI_GELU | us.EPI_TABLES_READY), 1),   # flag is masked off
    ]
    for fn, status in cases:
        with pytest.raises(us.UsError) as e:
            fn()
        assert e.value.status == status, (status, e.value)

    with pytest.raises(us.UsError) as e:
        us.cast_fp8_batch([16] * 9, [32] * 9, [4] * 9, [E4] * 9)         # more than US_CAST_BATCH_MAX tensors
    assert e.value.status == 2
    with pytest.raises(us.UsError) as e:
        us.cast_fp8_batch([16, 24], [32, 32], [4, 4], [E4, E5])          # second source misaligned
    assert e.value.status == 3
    with pytest.raises(us.UsError) as e:
        us.cast_fp8_batch([16], [32], [4], [F16])
    assert e.value.status == 4
    us.cast_fp8_batch([], [], [], [])
    # empty problems are accepted without touching any pointer
    us.cast_fp8(None, F16, None, E4, 0)
    us.gelu_fwd(None, None, 0)
    us.linear_fwd(None, None, None, 0, 16, 16, F16, F16)
    us.linear_bwd(None, None, None, None, None, 0, 0, 0, F16, F16, F16)
    us.bias_grad(None, F16, None, 0, 0)
    us.softmax_fwd(None, None, 0, 64)
    us.softmax_xent(None, None, None, None, 0, 64)


def test_composite_calls_check_every_product_before_the_first_launch():
    """A bad argument of a LATER product of a composite call is reported with its own status.  Had the first product
    been enqueued before that check, this GPU-less container would answer "launch failed" (6) instead -- and on a GPU
    the failing call would already have written into its outputs."""
    ws, wsb = 256, 1 << 30
    cases = [
        (lambda: us.ffn_fwd(16, 16, 16, 16, 16, 24, 16, 16, 16, 0, ws, wsb), 3),                         # Y misaligned
        (lambda: us.ffn_fwd(16, 16, 16, 16, 16, None, 16, 16, 16, us.FFN_FP8, ws, wsb), 1),
        (lambda: us.ffn_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 24, 16, 16, 16, 16, 0, ws, wsb), 3),     # dW1 misaligned
        (lambda: us.ffn_bwd(16, 16, 16, 16, 16, 16, 16, 16, 24, 16, 16, 16, 16, 16, us.FFN_FP8, ws, wsb), 3),   # dX misaligned
        (lambda: us.ffn_res_fwd(16, 16, 16, 16, 16, 16, 24, 16, 16, 16, 0.5, 0, ws, wsb), 3),            # Out misaligned
        (lambda: us.ffn_res_fwd(None, 16, 16, 16, 16, 16, 16, 16, 16, 16, 0.5, 0, ws, wsb), 1),          # no skip input
        (lambda: us.ffn_res_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 24, 16, 16, 16, 16, 0.5, 0, ws, wsb), 3),   # dW1
        (lambda: us.ffn_res_bwd(16, 16, 16, 16, 16, None, 16, 16, 16, 16, 16, 16, 16, 16, 16, 0.5, 0, ws, wsb), 1), # no Gskip
        (lambda: us.ffn_bias_fwd(16, 16, 16, 16, 24, 16, 16, 16, 16, 16, 16, 0, ws, wsb), 3),            # b2 misaligned
        (lambda: us.ffn_bias_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 24, 16, 16, 16, 16, 0, ws, wsb), 3),   # db1
        (lambda: us.ffn_bias_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 16, 24, 16, 16, 16, 16, 16, 16, 0, ws, wsb), 3),   # dW1
        (lambda: us.attention_fwd(16, 16, 16, 16, 16, 24, 2, 64, 64), 3),                                # O misaligned
        (lambda: us.attention_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 24, 16, 2, 64, 64), 3),            # dK misaligned
        (lambda: us.attention_fwd(16, 16, 16, 16, 16, 16, 70000, 64, 64), 2),
        # the entry point without a workspace: a shape whose slices exceed its static scratch, and ordinary argument errors
        (lambda: us.linear_bwd_noalloc(16, 16, 16, 16, 16, 4096, 512, 2048, us.F16, us.F16, us.F16), 5),
        (lambda: us.linear_bwd_noalloc(16, 16, 16, 16, 24, 1040, 2048, 1008, us.F16, us.F16, us.F16), 3),
        (lambda: us.linear_bwd_noalloc(16, 16, None, 16, 16, 1040, 2048, 1008, us.F16, us.F16, us.F16), 1),
    ]
    for fn, status in cases:
        with pytest.raises(us.UsError) as e:
            fn()
        assert e.value.status == status, (status, e.value)
