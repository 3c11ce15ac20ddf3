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


def test_multi_residual_arguments_rejected_before_any_launch():
    L = Q.lib()
    f = ctypes.c_void_p
    d = make_desc(1, 4, 4, 16)
    call = lambda rs, n, y=f(1 << 20): L.qasr_conv1d_int8_multi(ctypes.byref(d), f(4096), f(8192), None, f(8192), f(8192),
                                                                 rs, n, y, None)
    two = (ctypes.c_void_p * 2)(1 << 21, 1 << 22)
    assert call(two, -1) == -3
    assert call(two, Q.MAX_RESIDUALS + 1) == -3
    assert call(None, 2) == -1
    assert call((ctypes.c_void_p * 2)(1 << 21, None), 2) == -1
    assert call((ctypes.c_void_p * 2)(1 << 21, (1 << 20) + 8), 2) == -5          # second operand overlaps y
    # an op list: further operands need the first one, valid slots, and the output's shape
    def create(specs, n_slots):
        arr = (_Op * len(specs))()
        for i, (dd, i_s, r_s, o_s, more) in enumerate(specs):
            arr[i] = _Op(dd, 4096, None, 4096, 4096, i_s, r_s, o_s, None, len(more),
                         (ctypes.c_int32 * (Q.MAX_RESIDUALS - 1))(*more))
        h = ctypes.c_void_p()
        st = L.qasr_encoder_create(arr, len(specs), n_slots, ctypes.byref(h))
        assert not h.value or st == 0
        return st
    a = make_desc(1, 4, 4, 10)
    assert create([(a, 0, -1, 1, []), (a, 1, -1, 2, [1])], 3) == -3              # no first operand
    assert create([(a, 0, -1, 1, []), (a, 0, 1, 2, [7])], 3) == -3               # slot out of range
    assert create([(a, 0, -1, 1, []), (a, 0, 1, 2, [2])], 3) == -3               # operand is the output
    assert create([(a, 0, -1, 1, []), (make_desc(1, 4, 8, 10), 0, -1, 2, []), (a, 0, 1, 3, [2])], 4) == -3   # wrong shape


def test_dyadic_from_scale_on_the_host(golden):
    for row in golden("calibration_vectors.txt"):
        if row[0] == "dyadic":
            assert Q.dyadic_from_scale(float(row[1])) == (int(row[2]), int(row[3])), row
    assert Q.dyadic_from_scale(0.5 - 1e-13) == (1 << 30, 31)                 # the mantissa carries
    from fractions import Fraction
    for e in range(-30, 20):
        M = 1.2345678901 * 2.0 ** e
        m, s = Q.dyadic_from_scale(M)
        assert (1 << 30) <= m < (1 << 31) and abs(Fraction(m, 2 ** s) - Fraction(M)) <= Fraction(1, 2 ** (s + 1))
    L = Q.lib()
    m, s = ctypes.c_int32(), ctypes.c_int32()
    for bad in (0.0, -1.0, float("nan"), float("inf"), 2.0 ** 31, 2.0 ** -40):
        assert L.qasr_dyadic_from_scale(bad, ctypes.byref(m), ctypes.byref(s)) == -3
    assert L.qasr_dyadic_from_scale(1.0, None, ctypes.byref(s)) == -1


def test_calibration_arguments_rejected_before_any_launch():
    L = Q.lib()
    f = ctypes.c_void_p
    assert L.qasr_observe_minmax(None, 16, f(1 << 20), None) == -1
    assert L.qasr_observe_minmax(f(4096), 16, None, None) == -1
    assert L.qasr_observe_minmax(None, 0, None, None) == 0
    assert L.qasr_observe_minmax(f(4096), 16, f(4096 + 32), None) == -5
    ptrs = [f(1 << 20), f(2 << 20), f(3 << 20), f(4 << 20), f(5 << 20), f(6 << 20)]
    outs = [f(7 << 20), f(8 << 20), f(9 << 20), f(10 << 20), None, None]
    call = lambda w=ptrs[0], g=ptrs[2], eps=1e-5, Cout=4, per=12, Sx=0.1, Sy=0.1, qw=outs[0]: L.qasr_fold_bn_quantize(
        w, ptrs[1], g, ptrs[3], ptrs[4], ptrs[5], eps, Cout, per, Sx, Sy, qw, outs[1], outs[2], outs[3], None, None, None)
    assert call(w=None) == -1 and call(g=None) == -1 and call(qw=None) == -1
    assert call(Cout=0) == -2 and call(per=0) == -2
    assert call(Sx=0.0) == -3 and call(Sy=float("nan")) == -3 and call(eps=-1.0) == -3 and call(Sx=float("inf")) == -3
    assert call(qw=f((1 << 20) + 64)) == -5


def test_iexp_constants_on_the_host():
    c = Q.iexp_init(0.1, 0)                      # floor(6.93), floor(13.53), floor(0.344 / 0.003585)
    assert (c.u, c.q_ln2, c.q_b, c.q_c) == (0, 6, 13, 95)
    c = Q.iexp_init(0.1, 3)                      # the same at a step of 0.0125
    assert (c.u, c.q_ln2, c.q_b, c.q_c) == (3, 55, 108, 6141)
    L = Q.lib()
    out = Q.IExp()
    for S, u in [(0.0, 0), (-1.0, 0), (float("nan"), 0), (float("inf"), 0), (1.0, 0), (0.1, -1), (0.1, 17), (1e-9, 8)]:
        assert L.qasr_iexp_init(S, u, ctypes.byref(out)) == -3, (S, u)
    assert L.qasr_iexp_init(0.1, 0, None) == -1


def test_activation_arguments_rejected_before_any_launch():
    L = Q.lib()
    f = ctypes.c_void_p
    e = Q.iexp_init(6.0 / 127, 8)
    ok = Q.make_act(Q.ACT_SWISH, e, 1 << 30, 45)
    call = lambda a, x, B, C, T, xbs, ybs, y: L.qasr_act_int8(ctypes.byref(a) if a is not None else None, x, B, C, T, xbs, ybs, y, None)
    assert call(None, f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -1
    assert call(ok, None, 1, 4, 16, 0, 0, f(1 << 20)) == -1
    assert call(ok, f(4096), 1, 4, 16, 0, 0, None) == -1
    assert call(Q.make_act(0, e, 1 << 30, 45), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3      # kind
    assert call(Q.make_act(4, e, 1 << 30, 45), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3
    assert call(Q.make_act(2, e, -1, 45), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3           # m
    assert call(Q.make_act(2, e, 1 << 30, 0), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3       # s
    assert call(Q.make_act(2, e, 1 << 30, 63), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3
    bad = Q.IExp(8, 0, 0, 100, 100)                                                            # q_ln2 < 1
    assert call(Q.make_act(2, bad, 1 << 30, 45), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3
    bad = Q.IExp(8, 0, 10, 1 << 24, 100)                                                       # q_b too large
    assert call(Q.make_act(2, bad, 1 << 30, 45), f(4096), 1, 4, 16, 0, 0, f(1 << 20)) == -3
    assert call(ok, f(4096), 0, 4, 16, 0, 0, f(1 << 20)) == -2
    assert call(ok, f(4096), 1, 4, 0, 0, 0, f(1 << 20)) == -2
    assert call(ok, f(4096), 2, 4, 16, 63, 0, f(1 << 20)) == -2                                # stride < item
    assert call(Q.make_act(3, e, 1 << 30, 45), f(4096), 2, 4, 16, 64, 0, f(1 << 20)) == -2     # GLU item is 2 C T
    assert call(ok, f(4096), 2, 4, 16, 0, 0, f(4096 + 32)) == -5                               # partial overlap
    assert call(ok, f(4096), 2, 4, 16, 128, 64, f(4096)) == -5                                 # same base, other stride
    sm = lambda c, x, rows, Lr, y: L.qasr_softmax_int32(ctypes.byref(c) if c is not None else None, x, rows, Lr, y, None)
    assert sm(None, f(4096), 4, 16, f(1 << 20)) == -1
    assert sm(e, None, 4, 16, f(1 << 20)) == -1
    assert sm(e, f(4096), 0, 16, f(1 << 20)) == -2
    assert sm(e, f(4096), 4, 0, f(1 << 20)) == -2
    assert sm(e, f(4096), 4, 16385, f(1 << 20)) == -2
    assert sm(Q.IExp(17, 0, 10, 10, 10), f(4096), 4, 16, f(1 << 20)) == -3
    assert sm(e, f(4096), 4, 16, f(4096 + 100)) == -5
    assert sm(Q.IExp(0, 0, 1 << 22, (1 << 24) - 1, 1 << 47), f(4096), 4, 16384, f(1 << 20)) == -3   # row sum could overflow


def test_encoder_create_validates_activations_on_the_host():
    e = Q.iexp_init(6.0 / 127, 8)
    def create(act, Cout=4):
        arr = (_Op * 1)()
        arr[0] = _Op(make_desc(1, 4, Cout, 10), 4096, None, 4096, 4096, 0, -1, 1,
                     ctypes.pointer(act) if act is not None else None, 0)
        h = ctypes.c_void_p()
        st = Q.lib().qasr_encoder_create(arr, 1, 2, ctypes.byref(h))
        assert not h.value or st == 0
        return st
    assert create(Q.make_act(7, e, 1 << 30, 45)) == -3
    assert create(Q.make_act(Q.ACT_SWISH, e, 1 << 30, 99)) == -3
    assert create(Q.make_act(Q.ACT_GLU, e, 1 << 30, 45), Cout=5) == -2          # GLU needs an even channel count


def _ops(specs):
    arr = (_Op * len(specs))()
    for i, (d, i_s, r_s, o_s) in enumerate(specs):
        arr[i] = _Op(d, 4096, None, 4096, 4096, i_s, r_s, o_s, None, 0)
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
    assert Q.conv1d_kernel_name(make_desc(32, 256, 128, 800, flags=Q.FLAG_W_PACKED)) == "pw_tile"
    assert Q.conv1d_kernel_name(make_desc(32, 1024, 29, 800, flags=Q.FLAG_W_PACKED)) == "pw_tile"
    assert Q.conv1d_kernel_name(make_desc(1, 5, 5, 9, k=3, stride=2, groups=5)) == "conv_generic"
    assert Q.conv1d_kernel_name(make_desc(1, 5, 7, 9, k=3)) == "conv_generic"


def test_no_kernel_uses_scratch_memory():
    """The kernels count their own outstanding vector-memory requests; a register spill would add
    scratch loads and stores to that count behind their back.  The build records what the compiler
    reported per kernel: none may use scratch or spill, and the big pipelined kernels must keep two
    waves per SIMD."""
    import os
    path = os.path.join(os.path.dirname(Q.__file__), "resource_usage.txt")
    if not os.path.exists(path):
        pytest.skip("library was not built in this tree")
    rows = [l.split() for l in open(path) if l.strip()]
    assert len(rows) >= 80
    assert any("team_kernel" in r[0] for r in rows)
    for r in rows:
        f = dict(kv.split(":", 1) for kv in r[1:])
        assert f["ScratchSize[bytes/lane]"] == "0" and f["VGPRsSpill"] == "0", r[0]
        # scalar registers parked in lanes of a vector register touch no memory; only the persistent
        # team kernel (several layer bodies in one function) has them, at the bodies' boundaries
        assert f["SGPRsSpill"] == "0" or "team_kernel" in r[0], r[0]
        assert f["DynamicStack"] == "False", r[0]
        if "pw_pipe_kernel" in r[0] or "conv_pipe_kernel" in r[0] or "team_kernel" in r[0]:
            assert int(f["VGPRs"]) <= 256 and int(f["Occupancy[waves/SIMD]"]) >= 2, r[0]


def test_build_refuses_kernels_that_spill():
    """The pipelined kernels count their own memory requests, so a build in which the compiler
    spilled registers to scratch memory must not produce a library."""
    from paper_2103_16827_amd.build import kernels_using_scratch
    ok = ["k_ok", "TotalSGPRs:73", "VGPRs:249", "ScratchSize[bytes/lane]:0", "Occupancy[waves/SIMD]:2"]
    bad = ["k_spills", "TotalSGPRs:88", "VGPRs:256", "ScratchSize[bytes/lane]:520", "Occupancy[waves/SIMD]:2"]
    silent = ["k_without_figure", "VGPRs:12"]
    assert kernels_using_scratch([ok]) == []
    assert kernels_using_scratch([ok, bad, silent]) == ["k_spills", "k_without_figure"]


def test_build_checks_reads_after_partial_register_writes():
    """A vector instruction that reads a register in the slot right after a byte-selected write to it
    gets stale bytes on this chip; the compiler guards its own code, the build guards the hand-written
    asm by reading the device assembly."""
    from paper_2103_16827_amd.build import partial_write_hazards
    sdwa = "v_ashrrev_i32_sdwa v160, v226, v163 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
    ok = "\n".join(["\t" + sdwa, "\tds_write_b32 v162, v160 offset:2048", "\tv_add_u32_e32 v5, v160, v1"])
    spaced = "\n".join(["\t" + sdwa, "\t; a comment", "\tv_mfma_i32_16x16x64_i8 v[0:3], v[4:7], v[8:11], v[0:3]", "\t" + sdwa.replace("BYTE_1", "BYTE_2")])
    bad = "\n".join(["\t" + sdwa, ".Ltmp1:", "\t" + sdwa.replace("BYTE_1", "BYTE_2")])
    other_reg = "\n".join(["\t" + sdwa, "\tv_add_u32_e32 v5, v16, v1600"])
    full = "\n".join(["\tv_add_u32_sdwa v7, v1, v2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD", "\tv_add_u32_e32 v5, v7, v1"])
    assert partial_write_hazards(ok) == []
    assert partial_write_hazards(spaced) == []
    assert len(partial_write_hazards(bad)) == 1
    assert partial_write_hazards(other_reg) == []
    assert partial_write_hazards(full) == []


def test_the_partial_write_check_follows_includes_and_no_kernel_uses_such_writes_now(tmp_path):
    """Byte-selected register writes in hand-written asm are checked by the build wherever they are,
    also in a header; the kernels themselves use none any more (the one epilogue that did went back to
    whole-register instructions)."""
    import glob
    from paper_2103_16827_amd.build import source_with_local_includes, CSRC
    hit = sorted(os.path.basename(s) for s in glob.glob(os.path.join(CSRC, "*.hip"))
                 if "_sdwa" in source_with_local_includes(s))
    assert hit == [], hit
    (tmp_path / "h.hpp").write_text('asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0");\n')
    (tmp_path / "k.hip").write_text('#include "h.hpp"\n__global__ void k() {}\n')
    assert "_sdwa" in source_with_local_includes(str(tmp_path / "k.hip"))


def _replay(wiring, in_buf, res_buf, out_buf):
    """Symbolic replay: every op must find, in the buffer the plan points it to, the value that the
    caller's slot wiring meant; no op may write a buffer it reads."""
    slot_val, buf_val = {0: 0}, {0: 0}
    for i, (si, sr, so) in enumerate(wiring):
        assert buf_val.get(in_buf[i]) == slot_val[si], f"op {i}: wrong input value"
        if sr >= 0:
            assert buf_val.get(res_buf[i]) == slot_val[sr], f"op {i}: wrong residual value"
        else:
            assert res_buf[i] == -1
        assert out_buf[i] not in (in_buf[i], res_buf[i]) and out_buf[i] >= 1
        slot_val[so] = buf_val[out_buf[i]] = i + 1


@pytest.mark.parametrize("depth", [0, 1, 2, 4, 7])
def test_slot_buffer_plan_keeps_the_dataflow_and_avoids_recently_touched_buffers(depth):
    """qasr_plan_slot_buffers on the wiring of every benchmark configuration: the dataflow of the
    slots is kept (symbolic replay), and for depth >= 1 no op writes a buffer that one of the `depth`
    ops before it read or wrote."""
    import qasr_workloads as W
    for cfg in range(7):
        net = W.build_config(cfg)
        wiring = [(o.in_slot, o.res_slot, o.out_slot) for o in net.ops if not o.more_res]
        if len(wiring) != len(net.ops):
            continue                       # (dense residuals: more operands than this entry point takes)
        ib, rb, ob, nb = Q.plan_slot_buffers([w[0] for w in wiring], [w[1] for w in wiring], [w[2] for w in wiring],
                                             net.n_slots, depth)
        _replay(wiring, ib, rb, ob)
        if depth == 0:
            assert (ib, rb, ob) == ([w[0] for w in wiring], [w[1] for w in wiring], [w[2] for w in wiring])
            continue
        assert nb <= net.n_slots + depth + 1
        for i in range(len(wiring)):
            for j in range(max(0, i - depth), i):
                assert ob[i] not in (ib[j], rb[j], ob[j]), (cfg, i, j)


def test_slot_buffer_plan_rejects_bad_wiring():
    with pytest.raises(Q.QasrError):
        Q.plan_slot_buffers([0, 2], [-1, -1], [1, 3], 4, 4)       # slot 2 read before anything wrote it
    with pytest.raises(Q.QasrError):
        Q.plan_slot_buffers([0], [-1], [1], 2, 17)
    with pytest.raises(Q.QasrError):
        Q.plan_slot_buffers([0, 1], [-1, -1], [1, 1], 2, 1)       # writes the slot it reads
