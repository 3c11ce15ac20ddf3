"""MI355X-native integer-only ASR encoder inference (arXiv 2103.16827, Sec. 2.1-2.2).

The product is `libqasr.so` (hand-written HIP kernels for gfx950 behind a C ABI, declared in
include/qasr.h).  This package is the thin Python binding: argument marshalling only.  Every
step of the path runs in the library's kernels; there is no CPU or PyTorch fallback, and
importing the binding fails loudly if the library has not been built.
"""
from .binding import (  # noqa: F401
    QasrError, lib, conv1d_out_len, conv1d_int8, requant, pack_weights, packed_weight_bytes,
    conv1d_kernel_name, Encoder, EncoderGraph, ConvDesc, FLAG_RELU, FLAG_W_PACKED, status_string,
    quantize, dequantize, IExp, Act, ACT_SIGMOID, ACT_SWISH, ACT_GLU, iexp_init, make_act, act_int8,
    softmax_int32, conv1d_int8_multi, MAX_RESIDUALS, observe_minmax, dyadic_from_scale, fold_bn_quantize,
    tuning_reload, static_workspace_bytes, probe_copy, probe_mfma_i8, probe_mfma_outputs, plan_slot_buffers,
)
