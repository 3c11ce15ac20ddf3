"""The C-ABI library loads without a GPU, exports every symbol the header declares, and
rejects bad arguments before touching HIP (CPU only: no compute calls here)."""
import ctypes
import os
import re

import pytest

import paper_2103_16827_amd as Q
from paper_2103_16827_amd.binding import make_desc, _Op, LIB_PATH

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qasr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qasr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(LIB_PATH)
    names = declared_symbols()
    assert {"qasr_conv1d_int8", "qasr_requant", "qasr_encoder_forward", "qasr_encoder_create",
            "qasr_pack_weights", "qasr_conv1d_out_len"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_out_len_formula():
    assert Q.conv1d_out_len(make_desc(1, 64, 256, 1600, k=33, stride=2, pad_left=16, pad_right=16)) == 800
    assert Q.conv1d_out_len(make_desc(1, 512, 512, 800, k=87, dilation=2, pad_left=86, pad_right=86, groups=512)) == 800
    assert Q.conv1d_out_len(make_desc(1, 512, 512, 400, k=32, pad_left=15, pad_right=16, groups=512)) == 400
    assert Q.conv1d_out_len(make_desc(1, 4, 4, 10, k=3)) == 8
    assert Q.conv1d_out_len(make_desc(1, 4, 4, 10, k=3, stride=3)) == 3
    assert Q.conv1d_out_len(make_desc(1, 4, 4, 2, k=5)) == -2          # no output frame: SHAPE


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), -2), (dict(Cin=0), -2), (dict(k=0), -2), (dict(stride=0), -2), (dict(dilation=0), -2),
    (dict(pad_left=-1), -2), (dict(flags=4), -3), (dict(groups=2), -4), (dict(groups=4, Cout=8), -4),
    (dict(x_batch_stride=5), -2), (dict(y_batch_stride=3), -2),
])
def test_descriptor_validation(kw, status):
    base = dict(B=1, Cin=4, Cout=4, Tin=10, k=3)
    base.update(kw)
    d = make_desc(**base)
    assert Q.conv1d_out_len(d) == status
    fake = ctypes.c_void_p(4096)
    L = Q.lib()
    assert L.qasr_conv1d_int8(ctypes.byref(d), fake, fake, None, fake, fake, None, ctypes.c_void_p(1 << 20), None) == status


def test_null_and_alias_rejected_before_any_launch():
    L = Q.lib()
    d = make_desc(1, 4, 4, 10, k=3)
    f = lambda a: ctypes.c_void_p(a)
    assert L.qasr_conv1d_int8(None, f(4096), f(8192), None, f(1), f(1), None, f(1 << 20), None) == -1
    assert L.qasr_conv1d_int8(ctypes.byref(d), None, f(8192), None, f(1), f(1), None, f(1 << 20), None) == -1
    assert L.qasr_conv1d_int8(ctypes.byref(d), f(4096), f(8192), None, f(1), None, None, f(1 << 20), None) == -1
    # y inside x
    assert L.qasr_conv1d_int8(ctypes.byref(d), f(4096), f(8192), None, f(1), f(1), None, f(4096 + 8), None) == -5
    # y overlapping the residual
    assert L.qasr_conv1d_int8(ctypes.byref(d), f(4096), f(8192), None, f(1), f(1), f(1 << 20), f((1 << 20) + 31), None) == -5
    assert L.qasr_requant(None, 1, 1, 1, None, f(1), f(1), None, 0, f(64), None) == -1
    assert L.qasr_requant(f(4096), 1, 0, 1, None, f(1), f(1), None, 0, f(64), None) == -2
    assert L.qasr_requant(f(4096), 1, 1, 1, None, f(1), f(1), None, 2, f(64), None) == -3
    assert L.qasr_requant(f(4096), 1, 1, 4, None, f(1), f(1), None, 0, f(4100), None) == -5
    assert L.qasr_pack_weights(ctypes.byref(d), None, f(64), None) == -1
    assert Q.packed_weight_bytes(d) == 4 * 4 * 3
    assert Q.packed_weight_bytes(make_desc(1, 4, 4, 10, k=3, groups=4)) == 4 * 3
    # matrix-core operand order: Cout rounded up to 16 rows
    assert Q.packed_weight_bytes(make_desc(1, 64, 29, 10, k=3)) == 3 * 32 * 64
    assert Q.packed_weight_bytes(make_desc(1, 128, 32, 10)) == 32 * 128


def test_quantiser_arguments_rejected_before_any_launch():
    L = Q.lib()
    f = ctypes.c_void_p
    assert L.qasr_quantize(f(4096), 16, 0.0, f(1 << 20), None) == -3          # alpha must be > 0
    assert L.qasr_quantize(f(4096), 16, -1.0, f(1 << 20), None) == -3
    assert L.qasr_quantize(f(4096), 16, float("inf"), f(1 << 20), None) == -3
    assert L.qasr_quantize(f(4096), 16, float("nan"), f(1 << 20), None) == -3
    assert L.qasr_quantize(f(4096), 16, 1e-44, f(1 << 20), None) == -3        # alpha / 127 underflows to 0
    assert L.qasr_quantize(None, 16, 1.0, f(1 << 20), None) == -1
    assert L.qasr_quantize(f(4096), 16, 1.0, None, None) == -1
    assert L.qasr_quantize(None, 0, 1.0, None, None) == 0                     # nothing to do
    assert L.qasr_quantize(f(4096), 16, 1.0, f(4096 + 60), None) == -5        # q inside x
    assert L.qasr_dequantize(f(4096), 16, float("nan"), f(1 << 20), None) == -3
    assert L.qasr_dequantize(None, 16, 1.0, f(1 << 20), None) == -1
    assert L.qasr_dequantize(None, 0, 1.0, None, None) == 0
    assert L.qasr_dequantize(f(4096 + 8), 16, 1.0, f(4096), None) == -5       # x over q


def _ops(specs):
    arr = (_Op * len(specs))()
    for i, (d, i_s, r_s, o_s) in enumerate(specs):
        arr[i] = _Op(d, 4096, None, 4096, 4096, i_s, r_s, o_s)
    return arr


@pytest.mark.parametrize("specs,n_slots,status", [
    # out == in
    ([(make_desc(1, 4, 4, 10), 0, -1, 0)], 2, -3),
    # first op must read slot 0
    ([(make_desc(1, 4, 4, 10), 1, -1, 2)], 3, -3),
    # reading a slot nobody wrote
    ([(make_desc(1, 4, 4, 10), 0, -1, 1), (make_desc(1, 4, 4, 10), 2, -1, 1)], 3, -3),
    # channel mismatch through the slot
    ([(make_desc(1, 4, 8, 10), 0, -1, 1), (make_desc(1, 4, 4, 10), 1, -1, 2)], 3, -3),
    # frame-count mismatch through the slot
    ([(make_desc(1, 4, 4, 10, k=3), 0, -1, 1), (make_desc(1, 4, 4, 10), 1, -1, 2)], 3, -3),
    # residual shape mismatch
    ([(make_desc(1, 4, 8, 10), 0, -1, 1), (make_desc(1, 4, 4, 10), 0, 1, 2)], 3, -3),
    # slot index out of range
    ([(make_desc(1, 4, 4, 10), 0, -1, 5)], 2, -3),
    # packed flag not allowed in an op list
    ([(make_desc(1, 4, 4, 10, flags=2), 0, -1, 1)], 2, -3),
    # batch must be the same everywhere
    ([(make_desc(1, 4, 4, 10), 0, -1, 1), (make_desc(2, 4, 4, 10), 1, -1, 2)], 3, -2),
])
def test_encoder_create_validates_wiring_on_the_host(specs, n_slots, status):
    h = ctypes.c_void_p()
    assert Q.lib().qasr_encoder_create(_ops(specs), len(specs), n_slots, ctypes.byref(h)) == status
    assert not h.value


def test_status_strings():
    assert Q.status_string(0) == "ok"
    assert "workspace" in Q.status_string(-6)
    assert all(Q.status_string(s) for s in range(-7, 1))


def test_kernel_dispatch_names():
    # config-2 shapes go to the matrix-core kernels; odd geometry falls back to the generic one
    assert Q.conv1d_kernel_name(make_desc(32, 512, 512, 800, k=63, pad_left=31, pad_right=31, groups=512)) == "dw_pipe"
    assert Q.conv1d_kernel_name(make_desc(1, 512, 512, 800, k=63, pad_left=31, pad_right=31, groups=512)) == "dw_mfma"
    assert Q.conv1d_kernel_name(make_desc(32, 512, 512, 800, flags=Q.FLAG_W_PACKED)) == "pw_pipe"
    assert Q.conv1d_kernel_name(make_desc(32, 256, 128, 800, flags=Q.FLAG_W_PACKED)) == "pw_stream"
    assert Q.conv1d_kernel_name(make_desc(32, 1024, 29, 800, flags=Q.FLAG_W_PACKED)) == "pw_tile"
    assert Q.conv1d_kernel_name(make_desc(1, 5, 5, 9, k=3, stride=2, groups=5)) == "conv_generic"
    assert Q.conv1d_kernel_name(make_desc(1, 5, 7, 9, k=3)) == "conv_generic"
