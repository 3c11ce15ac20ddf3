"""Bit-exact parity of the HIP path (through the C ABI) against the CPU oracle.

Every case prints its name before touching the GPU, so that a fault can be traced to a
case from the tail of the log.  Integer results: the bar is equality of every byte.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2103_16827_amd as Q
import qasr_workloads as W
from qasr_workloads.rng import randint_array
from qasr_workloads.nets import OpSpec, FLAG_RELU
from gpu_util import dev, desc_of, gpu_layer, GpuNet

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def draw(seed, shape, lo, hi, dtype):
    return randint_array(seed, shape, lo, hi, dtype)


# ----------------------------------------------------------------------------- qasr_requant
@pytest.mark.parametrize("B,C,T", [(1, 1, 1), (2, 3, 17), (1, 5, 16), (2, 7, 200), (3, 64, 800), (1, 256, 1000), (2, 2, 4099)])
@pytest.mark.parametrize("mode", ["config", "generic"])
def test_requant(B, C, T, mode):
    say(f"requant B={B} C={C} T={T} mode={mode}")
    sd = 100 * B + 10 * C + T
    acc = draw(sd, (B, C, T), -(1 << 28), 1 << 28, np.int32)
    acc.reshape(-1)[:5] = [-(1 << 31), (1 << 31) - 1, 0, -1, 1][: min(5, acc.size)]
    if mode == "config":
        m = draw(sd + 1, (C,), 1 << 30, (1 << 31) - 1, np.int32)
        s = draw(sd + 2, (C,), 36, 58, np.int32)
    else:
        m = draw(sd + 1, (C,), 0, (1 << 31) - 1, np.int32)
        s = draw(sd + 2, (C,), 1, 62, np.int32)
        m[0], s[0] = 1 << 30, 30            # the identity pair
        if C > 2:
            s[1], s[2] = 32, 33             # both sides of the fast-path boundary
    bias = draw(sd + 3, (C,), -(1 << 16), 1 << 16, np.int32)
    res = draw(sd + 4, (B, C, T), -128, 127, np.int8)
    for use_bias, use_res, relu in ((True, True, False), (False, False, True), (True, False, False), (False, True, True)):
        b_ = bias if use_bias else None
        r_ = res if use_res else None
        if use_bias:
            a = np.clip(acc.astype(np.int64), -(1 << 31) + (1 << 16), (1 << 31) - 1 - (1 << 16)).astype(np.int32)
        else:
            a = acc
        ref = oracle.requant(a, b_, m, s, r_, relu)
        y = torch.full((B, C, T), 55, dtype=torch.int8, device="cuda")
        Q.requant(dev(a), dev(b_), dev(m), dev(s), dev(r_), Q.FLAG_RELU if relu else 0, y)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), ref), (use_bias, use_res, relu)


# ----------------------------------------------------------------------------- single layers
def layer_case(name, B, Cin, Cout, T, k=1, stride=1, dil=1, pad=None, dw=False, relu=True, bias=True,
               res=False, seed=1, wmin=-127, s_lo=36, s_hi=44, packed=False, prefix_of=None):
    if pad is None:
        tot = dil * (k - 1)
        pad = (tot // 2, tot - tot // 2)
    xbs = prefix_of * T if prefix_of else 0
    op = OpSpec(name, Cin, Cout, T, k, stride, dil, pad[0], pad[1], Cin if dw else 1, xbs,
                FLAG_RELU if relu else 0, bias)
    Cx = prefix_of or Cin
    sd = seed * 7919 + Cin * 31 + Cout * 17 + T + k
    x = draw(sd, (B, Cx, T), -128, 127, np.int8)
    p = {"w": draw(sd + 1, (Cout, 1 if dw else Cin, k), wmin, 127, np.int8),
         "bias": draw(sd + 2, (Cout,), -(1 << 16), 1 << 16, np.int32) if bias else None,
         "m": draw(sd + 3, (Cout,), 1 << 30, (1 << 31) - 1, np.int32),
         "s": draw(sd + 4, (Cout,), s_lo, s_hi, np.int32)}
    r = draw(sd + 5, (B, Cout, op.Tout), -128, 127, np.int8) if res else None
    return op, p, x, r, packed


def run_layer_case(case, ybs_extra=None):
    """ybs_extra: None = dense output; n = output (and residual) batch stride Cout*Tout + n."""
    op, p, x, r, packed = case
    B = x.shape[0]
    ybs = 0 if ybs_extra is None else op.Cout * op.Tout + ybs_extra
    d = desc_of(op, B, Q.FLAG_W_PACKED if packed else 0)
    d.y_batch_stride = ybs
    kern = Q.conv1d_kernel_name(d)
    say(f"layer {op.name} B={B} Cin={op.Cin} Cout={op.Cout} T={op.Tin} k={op.k} s={op.stride} d={op.dilation} "
        f"pad=({op.pad_left},{op.pad_right}) dw={op.depthwise} packed={packed} ybs={ybs} -> {kern}")
    ref = oracle.run_op(op, p, x, r)
    got = gpu_layer(op, B, p, x, r, packed=packed, ybs=ybs)
    bad = np.argwhere(got != ref)
    assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]} want {ref[tuple(bad[0])]}"
    return kern


SMALL = [
    dict(name="tiny_pw", B=1, Cin=1, Cout=1, T=1),
    dict(name="odd_pw", B=2, Cin=5, Cout=7, T=9, res=True),
    dict(name="odd_dense", B=2, Cin=3, Cout=5, T=17, k=3, stride=2, dil=2, pad=(2, 1), res=True, relu=False),
    dict(name="odd_dw", B=2, Cin=5, Cout=5, T=23, k=5, dw=True, pad=(1, 3), bias=False, relu=False),
    dict(name="dw_stride2", B=1, Cin=8, Cout=8, T=40, k=3, stride=2, dw=True),
    dict(name="dw_longer_than_T", B=2, Cin=4, Cout=4, T=7, k=33, dw=True, bias=False),
    dict(name="dense_minus128", B=1, Cin=16, Cout=8, T=33, k=5, wmin=-128),
    dict(name="k_even", B=1, Cin=8, Cout=8, T=30, k=4, dw=True, pad=(1, 2)),
    dict(name="generic_s", B=1, Cin=6, Cout=6, T=12, k=3, s_lo=1, s_hi=35),
    dict(name="dense_packed_odd", B=1, Cin=6, Cout=10, T=21, k=3, packed=True, res=True),
]


@pytest.mark.parametrize("kw", SMALL, ids=[c["name"] for c in SMALL])
def test_small_and_odd_layers(kw):
    run_layer_case(layer_case(**kw))


# Shapes of the benchmark networks (one or two batch items keep the oracle in seconds) plus
# ragged variants that span several tiles and a tail.
REAL = [
    dict(name="cfg0_dw", B=1, Cin=256, Cout=256, T=200, k=33, dw=True, bias=False, relu=False),
    dict(name="cfg0_pw", B=1, Cin=256, Cout=256, T=200),
    dict(name="dw_k33", B=2, Cin=256, Cout=256, T=800, k=33, dw=True, bias=False, relu=False),
    dict(name="dw_k39", B=2, Cin=256, Cout=256, T=800, k=39, dw=True, bias=False, relu=False),
    dict(name="dw_k51", B=1, Cin=512, Cout=512, T=800, k=51, dw=True, bias=False, relu=False),
    dict(name="dw_k63", B=1, Cin=512, Cout=512, T=800, k=63, dw=True, bias=False, relu=False),
    dict(name="dw_k75", B=1, Cin=512, Cout=512, T=800, k=75, dw=True, bias=False, relu=False),
    dict(name="dw_k87_d2", B=1, Cin=512, Cout=512, T=800, k=87, dil=2, dw=True, bias=False, relu=False),
    dict(name="dw_k32_prefix", B=2, Cin=512, Cout=512, T=400, k=32, dw=True, bias=False, relu=False, prefix_of=1024),
    dict(name="dw_ragged_T", B=3, Cin=70, Cout=70, T=1037, k=39, dw=True, bias=True, relu=True, res=True),
    dict(name="dw_T_not4", B=2, Cin=33, Cout=33, T=203, k=33, dw=True, bias=True, res=True),
    dict(name="dw_long_T", B=1, Cin=16, Cout=16, T=5000, k=75, dw=True, bias=False),
    dict(name="dw_minus128", B=1, Cin=64, Cout=64, T=320, k=33, dw=True, wmin=-128, bias=False),
    dict(name="dw_generic_s", B=1, Cin=64, Cout=64, T=320, k=33, dw=True, s_lo=20, s_hi=40),
    dict(name="pw_256_256", B=2, Cin=256, Cout=256, T=800),
    dict(name="pw_256_512_res", B=1, Cin=256, Cout=512, T=800, relu=False),
    dict(name="pw_512_512_res", B=2, Cin=512, Cout=512, T=800, res=True),
    dict(name="pw_512_1024", B=1, Cin=512, Cout=1024, T=800),
    dict(name="pw_1024_29", B=2, Cin=1024, Cout=29, T=800, relu=False),
    dict(name="pw_2048_512", B=1, Cin=2048, Cout=512, T=400, relu=False),
    dict(name="pw_ragged", B=3, Cin=192, Cout=200, T=333, res=True),
    dict(name="pw_T_not4", B=2, Cin=128, Cout=64, T=203, res=True),
    dict(name="pw_minus128", B=1, Cin=128, Cout=64, T=160, wmin=-128),
    dict(name="pw_generic_s", B=1, Cin=128, Cout=64, T=160, s_lo=20, s_hi=40),
    dict(name="pw_512_512_packed", B=2, Cin=512, Cout=512, T=800, res=True, packed=True),
    dict(name="pw_256_256_packed", B=1, Cin=256, Cout=256, T=800, packed=True),
    dict(name="pw_1024_29_packed", B=2, Cin=1024, Cout=29, T=800, relu=False, packed=True),
    dict(name="pw_2048_512_packed", B=1, Cin=2048, Cout=512, T=400, relu=False, packed=True),
    dict(name="pw_192_200_packed_T333", B=3, Cin=192, Cout=200, T=333, res=True, packed=True),
    dict(name="pw_320_72_packed_T332", B=2, Cin=320, Cout=72, T=332, res=True, packed=True),
    dict(name="pw_64_64_packed_generic_s", B=1, Cin=64, Cout=64, T=160, s_lo=20, s_hi=40, packed=True),
    dict(name="c1_dense_s2", B=2, Cin=64, Cout=256, T=1600, k=33, stride=2, pad=(16, 16), packed=True),
    dict(name="c1_dense_s2_raw", B=1, Cin=64, Cout=256, T=400, k=33, stride=2, pad=(16, 16)),
    dict(name="jasper_k11", B=1, Cin=256, Cout=256, T=800, k=11, packed=True, res=True),
    dict(name="jasper_k13_384", B=1, Cin=384, Cout=384, T=400, k=13, packed=True),
    dict(name="jasper_k25_768", B=1, Cin=768, Cout=768, T=200, k=25, packed=True),
    dict(name="jasper_pro", B=1, Cin=64, Cout=256, T=1600, k=11, stride=2, pad=(5, 5), packed=True),
    dict(name="jasper_epi_d2", B=1, Cin=768, Cout=896, T=200, k=29, dil=2, packed=True),
    dict(name="dense_ragged", B=2, Cin=128, Cout=72, T=211, k=7, packed=True, res=True),
]


@pytest.mark.parametrize("kw", REAL, ids=[c["name"] for c in REAL])
def test_real_shape_layers(kw):
    run_layer_case(layer_case(**kw))


# Output (and residual) batch strides larger than Cout*Tout, for every kernel family: a multiple of
# 16 bytes beyond the dense stride (the pipelined kernels keep serving the layer) and an odd
# multiple of 4 (their alignment conditions send the layer to another kernel).  gpu_layer checks that
# the gap bytes between the batch items' blocks and the canary bands around the buffer stay untouched.
STRIDED = [
    dict(name="ybs_dw_pipe", B=13, Cin=24, Cout=24, T=800, k=33, dw=True, bias=False),
    dict(name="ybs_dw_mfma_res", B=3, Cin=70, Cout=70, T=1037, k=39, dw=True, res=True),
    dict(name="ybs_dw_mfma", B=2, Cin=256, Cout=256, T=800, k=51, dw=True, bias=False, relu=False),
    dict(name="ybs_pw_pipe_res", B=3, Cin=512, Cout=512, T=336, res=True, packed=True),
    dict(name="ybs_pw_pipe", B=2, Cin=256, Cout=768, T=800, packed=True),
    dict(name="ybs_pw_pipe_streamed_res", B=2, Cin=2048, Cout=512, T=400, res=True, packed=True),
    dict(name="ybs_pw_tile_res", B=2, Cin=1024, Cout=29, T=800, relu=False, res=True, packed=True),
    dict(name="ybs_pw_tile_narrow", B=2, Cin=256, Cout=128, T=320, res=True, packed=True),
    dict(name="ybs_gemm_mfma_wide_res", B=2, Cin=1280, Cout=72, T=320, res=True, packed=True),
    dict(name="ybs_conv_pipe_res", B=2, Cin=128, Cout=328, T=428, k=11, packed=True, res=True),
    dict(name="ybs_conv_pipe_s2", B=2, Cin=64, Cout=256, T=1600, k=33, stride=2, pad=(16, 16), packed=True),
    dict(name="ybs_gemm_mfma_res", B=3, Cin=192, Cout=200, T=333, res=True, packed=True),
    dict(name="ybs_generic_res", B=2, Cin=3, Cout=5, T=17, k=3, stride=2, dil=2, pad=(2, 1), res=True, relu=False),
]


@pytest.mark.parametrize("extra", [16, 4, 4096])
@pytest.mark.parametrize("kw", STRIDED, ids=[c["name"] for c in STRIDED])
def test_output_batch_stride(kw, extra):
    run_layer_case(layer_case(**kw), ybs_extra=extra)


def test_output_batch_stride_cases_cover_every_kernel_family():
    seen = set()
    for kw in STRIDED:
        op, p, x, r, packed = layer_case(**kw)
        for extra in (16, 4):
            d = desc_of(op, x.shape[0], Q.FLAG_W_PACKED if packed else 0)
            d.y_batch_stride = op.Cout * op.Tout + extra
            seen.add(Q.conv1d_kernel_name(d))
    say(f"kernels reached with a padded output stride: {sorted(seen)}")
    assert {"dw_pipe", "dw_mfma", "pw_pipe", "pw_tile", "conv_pipe", "gemm_mfma", "conv_generic"} <= seen, seen


# The pipelined depthwise kernel (batches of 12 and more): one and two 64-chunk slices per row,
# short rows that share a 256-frame tile, long rows, every rescale form, odd batch sizes.
DWPIPE = [
    dict(name="dwp_k33", B=16, Cin=24, Cout=24, T=800, k=33, dw=True, bias=False),
    dict(name="dwp_k87_d2_two_slices", B=12, Cin=16, Cout=16, T=800, k=87, dil=2, dw=True, bias=False),
    dict(name="dwp_k75_bias", B=32, Cin=8, Cout=8, T=800, k=75, dw=True, relu=False),
    dict(name="dwp_long_rows", B=13, Cin=8, Cout=8, T=1600, k=39, dw=True),
    dict(name="dwp_short_rows", B=29, Cin=40, Cout=40, T=208, k=33, dw=True, relu=False),
    dict(name="dwp_generic_s", B=12, Cin=16, Cout=16, T=320, k=33, dw=True, s_lo=20, s_hi=40),
    dict(name="dwp_minus128_k32", B=14, Cin=16, Cout=16, T=400, k=32, dw=True, wmin=-128, bias=False),
]


@pytest.mark.parametrize("kw", DWPIPE, ids=[c["name"] for c in DWPIPE])
def test_pipelined_depthwise_layers(kw):
    assert run_layer_case(layer_case(**kw)) == "dw_pipe"


@pytest.mark.parametrize("rs", ["2,1", "1,1", "1,2", "2,2"])
def test_pipelined_depthwise_row_and_split_choices(rs, tuning_env):
    """Rows per iteration and batch splits other than the ones the heuristic picks."""
    tuning_env("QASR_DWP", rs)
    assert run_layer_case(layer_case(name="dwp_rs", B=48, Cin=8, Cout=8, T=400, k=51, dw=True)) == "dw_pipe"


# Every tile of the pipelined dense kernel (16 MT frames x 64 NT channels per wave), on shapes with
# ragged frame and channel tiles, a residual, a stride and a dilation.
CP_TILES = ["%d,%d" % (mt, nt) for nt in (4, 2) for mt in (8, 7, 6, 5, 4)]
CP_SHAPES = [
    dict(name="cp_k11_res", B=2, Cin=128, Cout=328, T=428, k=11, packed=True, res=True),
    dict(name="cp_k5_s2_d3", B=1, Cin=64, Cout=200, T=600, k=5, stride=2, dil=3, pad=(6, 6), packed=True, relu=False),
]


@pytest.mark.parametrize("tile", CP_TILES)
@pytest.mark.parametrize("kw", CP_SHAPES, ids=[c["name"] for c in CP_SHAPES])
def test_pipelined_dense_tile_choices(kw, tile, tuning_env):
    if kw.get("stride", 1) > 1 and tile.startswith("8"):
        pytest.skip("128 output frames at stride 2 exceed the kernel's 256 LDS rows")
    tuning_env("QASR_CP_TILE", tile)
    assert run_layer_case(layer_case(**kw)) == "conv_pipe"


# Dense convolutions through the older implicit-GEMM kernel too (the fallback of conv_pipe).
DENSE = [c for c in REAL if c.get("k", 1) > 1 and not c.get("dw") and c.get("packed")]


@pytest.mark.parametrize("kw", DENSE, ids=[c["name"] for c in DENSE])
def test_dense_layers_through_the_unpipelined_kernel(kw, tuning_env):
    tuning_env("QASR_NO_CONV_PIPE", "1")
    assert run_layer_case(layer_case(**kw)) in ("gemm_mfma", "conv_generic")


# The pipelined pointwise kernel: 2..8 passes of 256 output channels, a last pass that only some
# waves take part in, rows that leave a ragged last tile, every epilogue variant.
PIPE = [
    dict(name="pipe_512_1024_res", B=1, Cin=512, Cout=1024, T=800, res=True, packed=True),
    dict(name="pipe_512_2048_norelu", B=1, Cin=512, Cout=2048, T=400, relu=False, packed=True),
    dict(name="pipe_256_600_ragged", B=3, Cin=256, Cout=600, T=336, res=True, packed=True),
    dict(name="pipe_512_264_nobias", B=2, Cin=512, Cout=264, T=176, bias=False, packed=True),
    dict(name="pipe_512_512_generic_s", B=1, Cin=512, Cout=512, T=320, res=True, s_lo=20, s_hi=40, packed=True),
    dict(name="pipe_256_256_s33", B=2, Cin=256, Cout=256, T=160, s_lo=33, s_hi=34, res=True, packed=True),
    dict(name="pipe_256_768_minus128", B=1, Cin=256, Cout=768, T=480, wmin=-128, packed=True),
    dict(name="pipe_512_768_s_50_to_60", B=1, Cin=512, Cout=768, T=208, s_lo=50, s_hi=60, packed=True),   # both sides of s = 55
    dict(name="pipe_256_1024_s33", B=2, Cin=256, Cout=1024, T=160, s_lo=33, s_hi=33, packed=True),         # smallest short-form shift
    # 1024 / 2048 input channels: the activation chunks stream through a ring of 8 in LDS
    dict(name="pipe_2048_512_res", B=2, Cin=2048, Cout=512, T=400, res=True, packed=True),
    dict(name="pipe_2048_256_norelu_ragged_rows", B=3, Cin=2048, Cout=256, T=176, relu=False, packed=True),
    dict(name="pipe_1024_1024_generic_s", B=1, Cin=1024, Cout=1024, T=320, res=True, s_lo=20, s_hi=40, packed=True),
    dict(name="pipe_1024_2048_nobias", B=1, Cin=1024, Cout=2048, T=96, bias=False, packed=True),
]


@pytest.mark.parametrize("kw", PIPE, ids=[c["name"] for c in PIPE])
def test_pipelined_pointwise_layers(kw):
    assert run_layer_case(layer_case(**kw)) == "pw_pipe"


@pytest.mark.parametrize("split", [1, 2, 4, 8])
@pytest.mark.parametrize("case", ["2048_res_mixed", "1024_norelu_ragged_rows"])
def test_pipelined_pointwise_output_channel_splits(case, split, tuning_env):
    """Several workgroups per frame tile, each with its own run of 256-channel passes (what the
    heuristic chooses when the tiles alone do not fill the chip), forced here."""
    if case == "2048_res_mixed":
        op, p, x, r, packed = layer_case(name="pipe_split", B=2, Cin=512, Cout=2048, T=400, res=True, packed=True)
        p["s"][256 * 3:256 * 4] = draw(7, (256,), 20, 32, np.int32)          # one unpipelined pass in a run
    else:
        if split == 8:
            pytest.skip("4 passes")
        op, p, x, r, packed = layer_case(name="pipe_split", B=3, Cin=256, Cout=1024, T=336, relu=False, packed=True)
    tuning_env("QASR_PWP_SPLIT", str(split))
    assert run_layer_case((op, p, x, r, packed)) == "pw_pipe"


# The lean form of the pointwise kernel (one 256-channel pass per workgroup, two workgroups per
# compute unit): chosen by launch size in the encoders, forced here on small layers so that every
# epilogue variant, a ragged last tile and padded output strides go through it.
LEAN = [
    dict(name="lean_512_512_ragged_tiles", B=3, Cin=512, Cout=512, T=336, packed=True),
    dict(name="lean_256_1024_norelu", B=2, Cin=256, Cout=1024, T=160, relu=False, packed=True),
    dict(name="lean_512_768_nobias_generic_s", B=1, Cin=512, Cout=768, T=208, bias=False, s_lo=20, s_hi=40, packed=True),
    dict(name="lean_256_256_s33", B=2, Cin=256, Cout=256, T=160, s_lo=33, s_hi=33, packed=True),
    dict(name="lean_512_2048_minus128", B=1, Cin=512, Cout=2048, T=400, wmin=-128, packed=True),
    dict(name="lean_256_512_s_50_to_60", B=2, Cin=256, Cout=512, T=112, s_lo=50, s_hi=60, packed=True),
    # with a residual operand: its rows land in an LDS area of their own (256 input channels) or in the
    # LDS of activation chunks the products are done with (512)
    dict(name="lean_512_512_res_ragged_tiles", B=3, Cin=512, Cout=512, T=336, res=True, packed=True),
    dict(name="lean_512_1024_res_generic_s", B=2, Cin=512, Cout=1024, T=208, res=True, s_lo=20, s_hi=40, packed=True),
    dict(name="lean_256_256_res_norelu", B=2, Cin=256, Cout=256, T=160, res=True, relu=False, packed=True),
    dict(name="lean_256_768_res_s33", B=1, Cin=256, Cout=768, T=480, res=True, s_lo=33, s_hi=33, packed=True),
]


@pytest.mark.parametrize("extra", [0, 16])
@pytest.mark.parametrize("kw", LEAN, ids=[c["name"] for c in LEAN])
def test_lean_pointwise_layers(kw, extra, tuning_env):
    tuning_env("QASR_PW_LEAN", "1")
    assert run_layer_case(layer_case(**kw), extra) == "pw_pipe"


def test_lean_pointwise_is_what_large_launches_take_and_can_be_switched_off(tuning_env):
    """A layer with enough workgroups to share the units (the size at which the encoders use the
    lean form), then the same layer with the form switched off: same bytes."""
    case = layer_case(name="lean_by_size", B=8, Cin=256, Cout=1024, T=800, packed=True)
    assert run_layer_case(case) == "pw_pipe"
    tuning_env("QASR_NO_PW_LEAN", "1")
    assert run_layer_case(case) == "pw_pipe"


@pytest.mark.parametrize("slow_passes", [(1,), (0,), (1, 2), (0, 3)])
def test_pipelined_pointwise_mixed_rescale_forms(slow_passes):
    """Passes whose s values are all >= 33 are pipelined, the others take the 64-bit form right
    after their own loop: every order of the two kinds, with a residual."""
    op, p, x, r, packed = layer_case(name="pipe_mixed", B=1, Cin=256, Cout=1024, T=320, res=True, packed=True)
    for ps in slow_passes:
        p["s"][256 * ps:256 * (ps + 1)] = draw(99 + ps, (256,), 20, 32, np.int32)
    assert run_layer_case((op, p, x, r, packed)) == "pw_pipe"


def test_benchmark_shapes_use_the_matrix_core_kernels():
    """The fast kernels, not the generic fallback, serve every op of the benchmark networks."""
    for cfg in range(5):
        net = W.build_config(cfg)
        for o in net.ops:
            flags = 0 if o.depthwise else Q.FLAG_W_PACKED
            name = Q.conv1d_kernel_name(desc_of(o, net.B, flags))
            if o.depthwise:
                # the pipelined kernel needs at least 3 rows per wave (4 waves per channel)
                want = "dw_pipe" if net.B >= 12 else "dw_mfma"
            elif o.k == 1 and o.Tin % 16 == 0:
                # pipelined / weights-in-registers kernels for the instantiated widths, else the tile kernels
                if (o.Cin in (256, 512) and 256 <= o.Cout <= 2048) or \
                        (o.Cin in (1024, 2048) and o.Cout in (256, 512, 1024, 2048)):
                    want = "pw_pipe"          # pipelined-epilogue kernel for the instantiated widths
                elif o.Cin % 128 == 0 and o.Cin <= 1024:
                    want = "pw_tile"
                else:
                    want = "gemm_mfma"
            else:
                # dense k > 1: the pipelined implicit GEMM; pointwise on rows that are not a
                # multiple of 16 frames: the older one
                want = "conv_pipe" if o.k > 1 else "gemm_mfma"
            assert name == want, (cfg, o.name, name)


# ----------------------------------------------------------------------------- encoders
def oracle_items(net, params, x, y, items, what):
    """Oracle on the given batch items (each item of the batch is an independent utterance, so its
    output equals the oracle run on that item alone), compared with rows of the GPU output y."""
    sub = W.NetSpec(net.name, net.config_id, 1, net.Cin, net.Tin, net.ops, net.n_slots)
    for b in items:
        say(f"  oracle on {what} item {b}")
        ref, outs = oracle.encoder_forward(sub, params, np.ascontiguousarray(x[b:b + 1]), keep=True)
        if not np.array_equal(y[b:b + 1], ref):
            # localise: replay op by op on the GPU from the oracle's intermediates
            slots = {0: x[b:b + 1]}
            for i, (op, p) in enumerate(zip(net.ops, params)):
                r = slots[op.res_slot] if op.res_slot >= 0 else None
                if getattr(op, "more_res", None):
                    r = [r] + [slots[q] for q in op.more_res]
                got = gpu_layer(op, 1, p, slots[op.in_slot], r, packed=(not op.depthwise and op.k > 1))
                assert np.array_equal(got, outs[i]), f"item {b}: first failing op {i} {op.name}"
                slots[op.out_slot] = outs[i]
            raise AssertionError(f"item {b}: encoder output differs although every op matches in isolation")
        flat = ref.reshape(-1)
        assert len(set(flat.tolist())) > 16, "degenerate reference output"


_gpu_runs = {}


def gpu_forward_cached(key, make_net, seed, **draw_kw):
    """(net, params, x, y) of one GPU forward of the whole batch, computed once per key and shared by
    the tests that compare groups of its batch items with the oracle."""
    if key not in _gpu_runs:
        _gpu_runs.clear()                           # one full-size network at a time
        net = make_net()
        params = W.draw_net_params(net, seed, **draw_kw)
        x = W.draw_input(net, seed)
        g = GpuNet(net, params)
        y = g.forward(dev(x)).cpu().numpy()
        g.check_guards()
        g.enc.close()
        _gpu_runs[key] = (net, params, x, y)
    return _gpu_runs[key]


def check_encoder(net, seed, items=None, **draw_kw):
    """GPU forward of the whole batch vs the oracle on the chosen batch items (default: all)."""
    net_, params, x, y = gpu_forward_cached((net.name, net.config_id, net.B, net.Tin, len(net.ops), seed), lambda: net,
                                            seed, **draw_kw)
    oracle_items(net_, params, x, y, list(range(net.B)) if items is None else items, f"{net.name} seed={seed}")
    return y


def truncated(net, n_ops):
    """The first n_ops ops of a network as a network of its own (its output: that op's output)."""
    return W.NetSpec(f"{net.name}[:{n_ops}]", net.config_id, net.B, net.Cin, net.Tin, net.ops[:n_ops], net.n_slots)


@pytest.mark.parametrize("seed", range(1, 21))
def test_config0_separable_module(seed):
    say(f"config0 seed={seed}")
    check_encoder(W.build_config(0), seed)


@pytest.mark.parametrize("cfg", range(5))
def test_tiny_encoders(cfg):
    say(f"tiny encoder {cfg}")
    net = W.tiny_config(cfg)
    params = W.draw_net_params(net, 3, s_lo=37, s_hi=38, bias_mag=300)
    x = W.draw_input(net, 3)
    g = GpuNet(net, params)
    y = g.forward(dev(x)).cpu().numpy()
    g.check_guards()
    assert np.array_equal(y, oracle.encoder_forward(net, params, x))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_config1_quartznet_5x5(seed):
    say(f"config1 seed={seed}")
    check_encoder(W.build_config(1), seed)


# Configurations 2 to 4 at full size, in the launch configuration the benchmark times: the oracle
# checks EVERY batch item (the kernels' tiles straddle the items at a different offset for each).
# The items are spread over several tests so that none of them is silent for long.
@pytest.mark.parametrize("half", [0, 1])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_config2_quartznet_15x5_batch32(seed, half):
    say(f"config2 seed={seed} items {16 * half}..{16 * half + 15}")
    check_encoder(W.build_config(2), seed, items=range(16 * half, 16 * half + 16))


@pytest.mark.parametrize("n_ops,items", [(12, range(32)), (23, [0, 9, 18, 31]), (167, [0, 13, 31])],
                         ids=["block1_end", "block2_end", "C2_depthwise"])
def test_config2_intermediate_tensors(n_ops, items):
    """Outputs inside the network (the end of the first and second block, the output of the dilated
    depthwise layer before the last pointwise layers), so that the saturating layers downstream
    cannot hide a wrong byte: the first n_ops ops run as an encoder of their own."""
    net = truncated(W.build_config(2), n_ops)
    say(f"config2 truncated after op {n_ops - 1} ({net.ops[-1].name})")
    check_encoder(net, 1, items=items)


@pytest.mark.parametrize("group", [0, 1, 2, 3])
def test_config3_jasper_10x5_batch16_seed1_every_item(group):
    say(f"config3 seed=1 items {4 * group}..{4 * group + 3}")
    check_encoder(W.build_config(3), 1, items=range(4 * group, 4 * group + 4))


@pytest.mark.parametrize("seed", [2, 3])
def test_config3_jasper_10x5_batch16(seed):
    """Further seeds: two full-size items each, and the whole of a B=2, T=400 instance."""
    say(f"config3 seed={seed}")
    check_encoder(W.build_config(3), seed, items=[seed, 15 - seed])
    check_encoder(W.jasper(2, 400, config_id=3), seed)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_config4_conformer_shaped_batch16(seed):
    say(f"config4 seed={seed}")
    check_encoder(W.build_config(4), seed)


def test_forward_is_deterministic_and_leaves_guard_bytes():
    """Integer results: any run-to-run difference would be a race.  Also checks that nothing
    is written past the output tensor."""
    net = W.build_config(1)
    params = W.draw_net_params(net, 5)
    x = dev(W.draw_input(net, 5))
    g = GpuNet(net, params)
    n = g.y.numel()
    buf = torch.full((n + 4096,), 91, dtype=torch.int8, device="cuda")
    outs = []
    for _ in range(3):
        g.ws.fill_(-7)
        g.enc.forward(x, buf, g.ws)
        torch.cuda.synchronize()
        outs.append(buf[:n].clone())
        assert bool((buf[n:] == 91).all())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("depth", ["0", "1", "7"])
def test_buffer_plan_depths_give_the_same_bytes(depth, tuning_env):
    """The library decides which workspace buffer a slot's value lives in (no op writes a buffer
    that recent ops touched); whatever the depth of that plan, the caller's slots themselves
    included, the outputs are the same bytes, and the workspace grows with the depth."""
    net = W.quartznet(4, 640, 1, config_id=1)
    params = W.draw_net_params(net, 4)
    x = dev(W.draw_input(net, 4))
    g0 = GpuNet(net, params)                       # the default plan
    want = g0.forward(x).clone()
    g0.check_guards()
    tuning_env("QASR_SLOT_DEPTH", depth)
    g = GpuNet(net, params)
    got = g.forward(x)
    g.check_guards()
    assert torch.equal(got, want)
    if depth == "0":
        assert g.enc.workspace_bytes < g0.enc.workspace_bytes
    if depth == "7":
        assert g.enc.workspace_bytes > g0.enc.workspace_bytes
    ref = oracle.encoder_forward(W.NetSpec(net.name, net.config_id, 1, net.Cin, net.Tin, net.ops, net.n_slots), params,
                                 np.ascontiguousarray(W.draw_input(net, 4)[1:2]))
    assert np.array_equal(got[1:2].cpu().numpy(), ref)


def test_workspace_errors():
    net = W.tiny_config(1)
    params = W.draw_net_params(net, 1)
    g = GpuNet(net, params)
    x = dev(W.draw_input(net, 1))
    small = torch.empty(16, dtype=torch.int8, device="cuda")
    with pytest.raises(Q.QasrError) as e:
        g.enc.forward(x, g.y, small)
    assert e.value.status == -6


GRAPH_NETS = {
    "quartznet_5x5": lambda: W.build_config(1),
    "quartznet_15x5_batch32": lambda: W.build_config(2),          # the benchmark's launch configuration
    "jasper_dense_residual": lambda: W.jasper(2, 400, config_id=8, dense_residual=True),
    "conformer_nonlinear": lambda: W.conformer_shaped(4, 400, config_id=5, layers=3, nonlinear=True),
}


@pytest.mark.parametrize("which", list(GRAPH_NETS))
def test_encoder_graph_replays_match_eager_forwards(which):
    """The forward captured as a HIP graph: several
    replays, each on new input written into the same buffer, with eager work and synchronisation
    in between, each checked against the eager forward of the same input (and the first against
    the oracle)."""
    net = GRAPH_NETS[which]()
    params = W.draw_net_params(net, 5)
    g = GpuNet(net, params)
    x = dev(W.draw_input(net, 5))
    gr = g.enc.graph(x, g.y, g.ws)
    y_eager = torch.empty_like(g.y)
    for rep in range(6):
        say(f"graph replay {which} {rep}")
        xr = W.draw_input(net, 5 + rep)
        x.copy_(dev(xr))
        g.enc.forward(x, y_eager, g.ws)                 # eager work between the replays
        torch.cuda.synchronize()
        g.y.zero_()
        torch.cuda.synchronize()
        gr.launch()
        torch.cuda.synchronize()
        assert torch.equal(g.y, y_eager), f"replay {rep} differs from the eager forward"
        if rep == 0:
            sub = W.NetSpec(net.name, net.config_id, 1, net.Cin, net.Tin, net.ops, net.n_slots)
            ref = oracle.encoder_forward(sub, params, np.ascontiguousarray(xr[:1]))
            assert np.array_equal(g.y[:1].cpu().numpy(), ref)
    gr.close()
    g.enc.close()


# ----------------------------------------------------------------------------- quantiser / dequantiser
def _features(n, seed, alpha):
    """Seeded float32 features: mostly inside the clipping range, with exact ties, values at and
    beyond +-alpha, zeros of both signs, infinities and NaNs mixed in."""
    raw = randint_array(seed, (n,), -(1 << 20), 1 << 20, np.int32).astype(np.float32)
    x = raw * np.float32(alpha * 1.3 / (1 << 20))
    S = np.float32(alpha) / np.float32(127.0)
    k = randint_array(seed + 1, (n,), -130, 130, np.int32).astype(np.float32)
    tie = (k + np.float32(0.5)) * S
    sel = randint_array(seed + 2, (n,), 0, 15, np.int32)
    x = np.where(sel == 0, tie, x)
    x = np.where(sel == 1, k * S, x)
    special = np.array([alpha, -alpha, 0.0, -0.0, np.inf, -np.inf, np.nan, 3 * alpha, -3 * alpha], dtype=np.float32)
    m = min(n, len(special))
    x[:m] = special[:m]
    return x.astype(np.float32)


@pytest.mark.parametrize("n,alpha,offset", [
    (0, 1.0, 0), (1, 1.0, 0), (3, 4.75, 0), (1000003, 4.75, 0), (32 * 64 * 1600, 11.3, 0),
    (4099, 0.037, 1), (4099, 127.0, 3),      # pointers off the 16- / 4-byte grid: the element-wise path
])
def test_quantiser_matches_oracle(n, alpha, offset):
    say(f"quantise n={n} alpha={alpha} offset={offset}")
    x = _features(n + offset, 17 + n % 13, alpha)[offset:]
    ref = oracle.quantize(x, alpha)
    xd = torch.from_numpy(_features(n + offset, 17 + n % 13, alpha)).cuda()[offset:]
    qd = torch.full((n + offset + 8,), 99, dtype=torch.int8, device="cuda")
    Q.quantize(xd, alpha, qd[offset:offset + n])
    torch.cuda.synchronize()
    got = qd.cpu().numpy()
    assert np.array_equal(got[offset:offset + n], ref)
    assert np.all(got[:offset] == 99) and np.all(got[offset + n:] == 99)      # nothing written outside
    if n > 1000:
        assert len(set(ref.tolist())) == 255


@pytest.mark.parametrize("n,S,offset", [(0, 1.0, 0), (5, 0.25, 0), (1000003, 0.0371, 0), (32 * 29 * 800, 0.118, 0), (4099, 3.0, 3)])
def test_dequantiser_matches_oracle(n, S, offset):
    say(f"dequantise n={n} S={S} offset={offset}")
    q = randint_array(23 + n % 7, (n + offset,), -128, 127, np.int8)
    ref = oracle.dequantize(q[offset:], S)
    qd = torch.from_numpy(q).cuda()
    xd = torch.full((n + offset + 8,), -7.0, dtype=torch.float32, device="cuda")
    Q.dequantize(qd[offset:], S, xd[offset:offset + n])
    torch.cuda.synchronize()
    got = xd.cpu().numpy()
    assert np.array_equal(got[offset:offset + n].view(np.uint32), ref.view(np.uint32))   # bit for bit
    assert np.all(got[:offset] == -7.0) and np.all(got[offset + n:] == -7.0)


# ----------------------------------------------------------------------------- integer activations
ACT_CASES = [
    # kind, B, C, T, S, u, m, s, layout
    (Q.ACT_SWISH, 2, 64, 400, 6.0 / 127, 8, 1 << 30, 45, "dense"),
    (Q.ACT_SWISH, 16, 2048, 400, 5.1 / 127, 8, 1518500250, 45, "inplace"),       # ffn1 of configuration 4
    (Q.ACT_SWISH, 3, 7, 37, 8.0 / 127, 6, 1300000000, 44, "dense"),               # ragged: element-wise tail
    (Q.ACT_SWISH, 2, 5, 33, 4.0 / 127, 8, 1 << 30, 45, "unaligned"),
    (Q.ACT_SWISH, 3, 16, 64, 4.4 / 127, 8, 2000000000, 46, "strided"),
    (Q.ACT_SIGMOID, 2, 32, 100, 6.0 / 127, 8, 1 << 30, 38, "dense"),              # sigma at scale 2^-7
    (Q.ACT_SIGMOID, 1, 1, 256, 16.0 / 127, 10, 1 << 30, 38, "all_codes"),
    (Q.ACT_SWISH, 1, 1, 256, 0.1, 6, 1 << 30, 45, "all_codes"),
    (Q.ACT_SWISH, 1, 1, 256, 6.0 / 127, 8, 123456789, 20, "all_codes"),           # small s: saturating outputs
    (Q.ACT_GLU, 2, 64, 400, 6.0 / 127, 8, 1 << 30, 45, "dense"),
    (Q.ACT_GLU, 16, 512, 400, 6.6 / 127, 8, 1700000000, 45, "inplace"),           # pw1 of configuration 4
    (Q.ACT_GLU, 3, 7, 37, 8.0 / 127, 6, 1300000000, 44, "dense"),                 # halves off the 16-byte grid
    (Q.ACT_GLU, 2, 5, 33, 4.0 / 127, 8, 1 << 30, 45, "unaligned"),
    (Q.ACT_GLU, 3, 16, 64, 4.4 / 127, 8, 2000000000, 46, "strided"),
    (Q.ACT_GLU, 1, 256, 256, 5.0 / 127, 8, 1 << 30, 45, "all_pairs"),
]


@pytest.mark.parametrize("kind,B,C,T,S,u,m,s,layout", ACT_CASES)
def test_activations_match_oracle(kind, B, C, T, S, u, m, s, layout):
    say(f"act kind={kind} B={B} C={C} T={T} S={S:.5f} u={u} m={m} s={s} {layout}")
    Cx = 2 * C if kind == Q.ACT_GLU else C
    x = randint_array(31 + C + T, (B, Cx, T), -128, 127, np.int8)
    if layout == "all_codes":
        x[0, 0, :] = np.arange(-128, 128)
    if layout == "all_pairs":                      # value c - 128 against every gate code
        x[0, :C] = (np.arange(C) - 128).reshape(C, 1)
        x[0, C:] = (np.arange(T) - 128).reshape(1, T)
    ref = oracle.act(kind, x, oracle.iexp_constants(S, u), m, s)
    a = Q.make_act(kind, Q.iexp_init(S, u), m, s)
    off = 1 if layout == "unaligned" else 0
    xbs = Cx * T + (48 if layout == "strided" else 0)
    ybs = xbs if layout == "inplace" else C * T + (80 if layout == "strided" else 0)
    xd = torch.full((off + B * xbs + 8,), 55, dtype=torch.int8, device="cuda")
    xd[off:off + B * xbs].view(B, xbs)[:, :Cx * T] = torch.from_numpy(x.reshape(B, -1)).cuda()
    yd = xd if layout == "inplace" else torch.full((off + B * ybs + 8,), 99, dtype=torch.int8, device="cuda")
    before = xd.clone()
    Q.act_int8(a, xd[off:], B, C, T, yd[off:], xbs, ybs)
    torch.cuda.synchronize()
    got = yd.cpu().numpy()
    body = got[off:off + B * ybs].reshape(B, ybs)
    assert np.array_equal(body[:, :C * T].reshape(B, C, T), ref)
    # nothing else written: the gaps between items, the bytes before and after, the gate half
    fill = before.cpu().numpy() if layout == "inplace" else np.full_like(got, 99)
    assert np.array_equal(body[:, C * T:], fill[off:off + B * ybs].reshape(B, ybs)[:, C * T:])
    assert np.array_equal(got[:off], fill[:off]) and np.array_equal(got[off + B * ybs:], fill[off + B * ybs:])
    if layout != "inplace":
        assert torch.equal(xd, before)
    if C * T >= 256 and s >= 38:
        assert len(set(ref.reshape(-1).tolist())) > 16


@pytest.mark.parametrize("rows,L,S,u", [(1, 1, 0.01, 2), (7, 37, 0.002, 0), (64, 400, 0.01, 2), (3, 1000, 1.0 / 64, 4),
                                         (2, 16384, 0.004, 1), (1024, 400, 0.0073, 3),
                                         (33, 300, 1e-5, 0),        # exponentials beyond 32 bits
                                         (5, 512, 0.01, 2), (9, 513, 0.01, 2)])
def test_softmax_matches_oracle(rows, L, S, u):
    say(f"softmax rows={rows} L={L} S={S} u={u}")
    x = randint_array(41 + L, (rows, L), -int(6 / S), int(6 / S), np.int32)
    x[0, :: max(1, L // 5)] = np.int32(2_000_000_000)          # int32 extremes must not wrap
    if rows > 1:
        x[1, :] = np.int32(-2_000_000_000)
        x[1, L // 2] = np.int32(2_000_000_000)
    ref = oracle.softmax(x, oracle.iexp_constants(S, u))
    xd = torch.from_numpy(x).cuda()
    yd = torch.full((rows * L + 16,), 99, dtype=torch.int8, device="cuda")
    Q.softmax_int32(Q.iexp_init(S, u), xd, yd[: rows * L].view(rows, L))
    torch.cuda.synchronize()
    got = yd.cpu().numpy()
    assert np.array_equal(got[: rows * L].reshape(rows, L), ref)
    assert np.all(got[rows * L:] == 99)


def test_tiny_conformer_with_integer_activations():
    net = W.tiny_config(5)
    params = W.draw_net_params(net, 3, s_lo=37, s_hi=38, bias_mag=300)
    x = W.draw_input(net, 3)
    g = GpuNet(net, params)
    y = g.forward(dev(x)).cpu().numpy()
    assert np.array_equal(y, oracle.encoder_forward(net, params, x))
    g.enc.close()


def test_conformer_shaped_batch16_with_integer_activations():
    """Configuration 4 with Swish after ffn1 and the depthwise convolution and GLU after pw1."""
    check_encoder(W.build_config(5), 1, items=[0, 15])


def test_which_activations_run_inside_the_layer_kernel():
    """Swish after the 512 -> 2048 layers and after the depthwise convolutions goes through the
    producing kernel's epilogue table; the GLU keeps the separate in-place pass (the parity test
    above covers both routes: it runs this very encoder)."""
    net = W.build_config(5)
    g = GpuNet(net, W.draw_net_params(net, 1))
    kinds = {}
    for i, (op, p) in enumerate(zip(net.ops, g.params)):
        a = p.get("act")
        if a:
            kinds.setdefault((a["kind"], g.kernels()[i], g.enc.op_act_fused(i)), 0)
            kinds[(a["kind"], g.kernels()[i], g.enc.op_act_fused(i))] += 1
        else:
            assert not g.enc.op_act_fused(i)
    assert kinds[(Q.ACT_SWISH, "pw_pipe", True)] == 17
    assert kinds[(Q.ACT_SWISH, "dw_pipe", True)] == 17
    assert kinds[(Q.ACT_GLU, "pw_pipe", False)] == 17
    g.enc.close()


@pytest.mark.gpu
@pytest.mark.parametrize("seed", [1, 2])
def test_fused_activation_with_relu_residual_and_several_passes(seed):
    """Table lookups in the pointwise kernel's epilogue next to everything else that epilogue does:
    ReLU before the activation, a residual operand, two passes of output channels, both unary kinds."""
    from qasr_workloads.nets import _Builder
    b = _Builder("fused_act_probe", 99, 3, 256, 160)
    b.op("p1", 256, relu=True)
    t2 = b.op("p2", 512, relu=True, act=Q.ACT_SIGMOID)
    b.op("p3", 512, relu=False, act=Q.ACT_SWISH)
    b.op("p4", 512, relu=True, res=t2, act=Q.ACT_SIGMOID)
    b.op("p5", 256, relu=False)
    net = b.done()
    params = W.draw_net_params(net, seed)
    for p in params:                       # a sigmoid code has 15 fraction bits: bring it to int8 range
        if p.get("act") and p["act"]["kind"] == Q.ACT_SIGMOID:
            p["act"]["s"] = 39
    x = W.draw_input(net, seed)
    ref, outs = oracle.encoder_forward(net, params, x, keep=True)
    for o, a in zip(net.ops, outs):
        assert len(set(a.reshape(-1).tolist())) > 16, f"degenerate reference output of {o.name}"
    g = GpuNet(net, params)
    assert g.kernels() == ["pw_pipe"] * 5
    assert [g.enc.op_act_fused(i) for i in range(5)] == [False, True, True, True, False]
    y = g.forward(dev(x)).cpu().numpy()
    g.enc.close()
    assert np.array_equal(y, ref)


# ----------------------------------------------------------------------------- variants of the same families
def test_quartznet_10x5():
    """The medium model of the latency comparison (Sec. 3.2): each block type twice."""
    check_encoder(W.quartznet(4, 1600, 2, config_id=6), 1, items=[0, 3])


def test_quartznet_15x5_with_separable_first_layer():
    net = W.quartznet(2, 1600, 3, config_id=7, separable_c1=True)
    check_encoder(net, 1, items=[1])


@pytest.mark.parametrize("cfg", [1, 3])
def test_w6a8_six_bit_weight_codes_in_int8_storage(cfg):
    """W6A8 (Sec. 3.1): weights in [-31, 31]; the rescale shifts are two smaller so that the
    activations keep their range."""
    net = W.build_config(1) if cfg == 1 else W.jasper(2, 400, config_id=3)
    check_encoder(net, 2, w_bits=6, s_lo=34, s_hi=42)


@pytest.mark.parametrize("n_res,shape", [
    (2, dict(B=2, Cin=128, Cout=328, T=428, k=11, packed=True)),       # pipelined dense kernel, ragged tiles
    (12, dict(B=1, Cin=64, Cout=64, T=96, k=3, packed=True)),          # the maximum number of operands
    (3, dict(B=2, Cin=20, Cout=7, T=53, k=5, packed=False)),           # general kernel
    (4, dict(B=2, Cin=16, Cout=16, T=64, k=9, dw=True, packed=False)), # depthwise: general kernel too
    (5, dict(B=1, Cin=256, Cout=256, T=800, k=1, packed=True)),        # pointwise with several operands
])
def test_layers_with_several_residual_operands(n_res, shape):
    kw = dict(shape)
    packed, dw = kw.pop("packed"), kw.pop("dw", False)
    B, Cin, Cout, T, k = kw["B"], kw["Cin"], kw["Cout"], kw["T"], kw["k"]
    say(f"multi-residual n_res={n_res} {shape}")
    op = W.OpSpec("mr", Cin, Cout, T, k, 1, 1, (k - 1) // 2, k - 1 - (k - 1) // 2, Cin if dw else 1)
    x = randint_array(3, (B, Cin, T), -128, 127, np.int8)
    p = {"w": randint_array(4, (Cout, 1 if dw else Cin, k), -127, 127, np.int8),
         "bias": randint_array(5, (Cout,), -65536, 65536, np.int32),
         "m": randint_array(6, (Cout,), 1 << 30, (1 << 31) - 1, np.int32),
         "s": randint_array(7, (Cout,), 38 if dw else 40, 46, np.int32)}
    rs = [randint_array(20 + r, (B, Cout, T), -128, 127, np.int8) for r in range(n_res)]
    ref = oracle.conv1d_int8(x, p["w"], p["bias"], p["m"], p["s"], rs, pad_left=op.pad_left, pad_right=op.pad_right,
                             groups=op.groups)
    got = gpu_layer(op, B, p, x, rs, packed=packed)
    assert np.array_equal(got, ref)
    assert not np.array_equal(ref, oracle.conv1d_int8(x, p["w"], p["bias"], p["m"], p["s"], rs[0], pad_left=op.pad_left,
                                                      pad_right=op.pad_right, groups=op.groups))


def test_tiny_jasper_with_dense_residuals():
    net = W.tiny_config(7)
    params = W.draw_net_params(net, 3, s_lo=37, s_hi=38, bias_mag=300)
    x = W.draw_input(net, 3)
    g = GpuNet(net, params)
    y = g.forward(dev(x)).cpu().numpy()
    assert np.array_equal(y, oracle.encoder_forward(net, params, x))
    g.enc.close()


def test_jasper_dense_residual_batch2():
    """The dense-residual variant at a quarter of the frames (same ops: up to 9 further operands)."""
    net = W.jasper(2, 400, config_id=8, dense_residual=True)
    y = check_encoder(net, 1)
    g = GpuNet(net, W.draw_net_params(net, 1))
    ks = g.kernels()
    assert all(ks[i] == "conv_pipe" for i, o in enumerate(net.ops) if o.more_res)
    g.enc.close()


# ----------------------------------------------------------------------------- offline calibration helpers
@pytest.mark.parametrize("n,offset", [(1, 0), (5, 0), (1000003, 0), (16 * 64 * 1600, 0), (4099, 1), (32 * 512 * 800, 0)])
def test_observer_matches_oracle(n, offset):
    say(f"observer n={n} offset={offset}")
    x = (randint_array(50 + n % 11, (n + offset,), -(1 << 22), 1 << 22, np.int32).astype(np.float32) * np.float32(3e-4))
    if n > 100:
        x[[7, n // 2, n - 1]] = np.nan
        x[n // 3] = np.float32(-2000.5)
        x[n // 5] = np.float32(1999.25)
    ref = oracle.minmax(x[offset:])
    xd = torch.from_numpy(x).cuda()
    mm = torch.tensor([float("inf"), float("-inf"), 123.0], dtype=torch.float32, device="cuda")
    Q.observe_minmax(xd[offset:], mm)
    torch.cuda.synchronize()
    got = mm.cpu().numpy()
    assert got[0] == ref[0] and got[1] == ref[1] and got[2] == 123.0
    # running: a second tensor only widens the range
    y = torch.tensor([float("nan"), 5000.0, -1.0], dtype=torch.float32, device="cuda")
    Q.observe_minmax(y, mm)
    torch.cuda.synchronize()
    got2 = mm.cpu().numpy()
    assert got2[0] == min(ref[0], np.float32(-1.0)) and got2[1] == np.float32(5000.0)


@pytest.mark.parametrize("Cout,Cin_g,k,with_bias", [(256, 256, 11, True), (512, 1, 51, False), (29, 1024, 1, True), (5, 3, 2, True)])
def test_fold_and_quantize_matches_oracle(Cout, Cin_g, k, with_bias):
    say(f"fold Cout={Cout} Cin/g={Cin_g} k={k} bias={with_bias}")
    f = lambda sd, shape, lo, hi: (randint_array(sd, shape, 0, 1 << 24, np.int32).astype(np.float32) / np.float32(1 << 24)
                                   * np.float32(hi - lo) + np.float32(lo))
    w = f(1, (Cout, Cin_g, k), -0.3, 0.3)
    if Cout > 4:
        w[3] = 0.0                                              # an all-zero channel
    b = f(2, (Cout,), -0.5, 0.5) if with_bias else None
    gamma = f(3, (Cout,), 0.4, 1.6); gamma[0] = -gamma[0]
    beta, mean, var = f(4, (Cout,), -0.5, 0.5), f(5, (Cout,), -1.0, 1.0), f(6, (Cout,), 0.1, 3.0)
    eps, S_x, S_y = 1e-3, 4.0 / 127, 6.5 / 127
    if Cout > 4:
        beta[2] = np.float32(3e9)                               # a bias that leaves int32: counted, set to 0
    qw_r, bq_r, m_r, s_r, Sw_r, bad_r = oracle.fold_quantize(w, b, gamma, beta, mean, var, eps, S_x, S_y)
    d = lambda a: None if a is None else torch.from_numpy(a).cuda()
    qw = torch.full((Cout * Cin_g * k + 16,), 99, dtype=torch.int8, device="cuda")
    bq, m, s = (torch.full((Cout,), -1, dtype=torch.int32, device="cuda") for _ in range(3))
    Sw = torch.zeros(Cout, dtype=torch.float32, device="cuda")
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    Q.fold_bn_quantize(d(w), d(b), d(gamma), d(beta), d(mean), d(var), eps, S_x, S_y, qw, bq, m, s, Sw, bad)
    torch.cuda.synchronize()
    got = qw.cpu().numpy()
    assert np.array_equal(got[:-16].reshape(w.shape), qw_r) and np.all(got[-16:] == 99)
    assert np.array_equal(bq.cpu().numpy(), bq_r) and np.array_equal(m.cpu().numpy(), m_r) and np.array_equal(s.cpu().numpy(), s_r)
    assert np.array_equal(Sw.cpu().numpy().view(np.uint32), Sw_r.view(np.uint32))
    assert int(bad.item()) == bad_r == (1 if Cout > 4 else 0)
    assert np.all(np.abs(qw_r.reshape(Cout, -1)).max(axis=1)[[c for c in range(Cout) if not (Cout > 4 and c == 3)]] == 127)


# ----------------------------------------------------------------------------- seeded random shapes
def _random_cases(n, seed):
    """Seeded layer shapes biased towards the boundaries of the kernels' applicability conditions
    (multiples of 16 / 64 / 256 and their neighbours), so that every dispatch decision is taken
    from both sides."""
    r = randint_array(seed, (n, 12), 0, (1 << 31) - 1, np.int64)
    near = lambda v, base: int(base + (v % 5) - 2)                       # base-2 .. base+2
    cases = []
    for i in range(n):
        v = [int(t) for t in r[i]]
        kind = v[0] % 3                                                   # 0 pointwise, 1 depthwise, 2 dense
        B = [1, 2, 3, 13][v[1] % 4]
        T = [16, 48, 96, 112, 208, 336][v[2] % 6] + (0 if v[3] % 4 else (v[3] % 7) - 3)
        cbase = [16, 64, 128, 256, 512][v[4] % 5]
        Cin = cbase if v[5] % 3 else max(1, near(v[5] // 3, cbase))
        obase = [16, 64, 256, 512, 1024][v[6] % 5]
        Cout = obase if v[7] % 3 else max(1, near(v[7] // 3, obase))
        k = 1 if kind == 0 else [2, 3, 5, 11, 33][v[8] % 5]
        stride = 1 if v[9] % 4 else 2
        dil = 1 if v[9] % 5 else 2
        if kind == 0:
            stride = dil = 1
        if kind == 1:
            Cout = Cin = min(Cin, 96)
        else:
            Cin, Cout = min(Cin, 520), min(Cout, 1030)
            if kind == 2:
                Cin, Cout = min(Cin, 260), min(Cout, 300)
        T = max(T, 4)
        cases.append(dict(name=f"rand{seed}_{i}", B=B, Cin=Cin, Cout=Cout, T=T, k=k, stride=stride, dil=dil, dw=kind == 1,
                          relu=bool(v[10] & 1), bias=bool(v[10] & 2), res=bool(v[10] & 4),
                          s_lo=[36, 20, 33][v[11] % 3], s_hi=[44, 40, 34][v[11] % 3],
                          packed=(kind != 1 and Cin % 64 == 0 and (v[10] >> 3) % 4 != 0)))
    return cases


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_seeded_random_layer_shapes(seed):
    kernels = {}
    for kw in _random_cases(100, seed):
        k = run_layer_case(layer_case(**kw))
        kernels[k] = kernels.get(k, 0) + 1
    say(f"kernels hit: {kernels}")
    assert len(kernels) >= 6


def test_forward_from_float_features_to_float_outputs():
    """Quantiser, integer encoder and dequantiser in one call against the three oracle steps."""
    net = W.build_config(1)
    params = W.draw_net_params(net, 4)
    alpha, S_out = 3.7, 0.0625
    xf = _features(net.B * net.Cin * net.Tin, 9, alpha).reshape(net.B, net.Cin, net.Tin)
    ref = oracle.dequantize(oracle.encoder_forward(net, params, oracle.quantize(xf, alpha)), S_out)
    g = GpuNet(net, params)
    ws = torch.empty(g.enc.workspace_bytes_f32, dtype=torch.int8, device="cuda")
    y = torch.empty((net.B, net.Cout, net.Tout), dtype=torch.float32, device="cuda")
    g.enc.forward_f32(torch.from_numpy(xf).cuda(), alpha, S_out, y, ws)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    small = torch.empty(g.enc.workspace_bytes_f32 - 256, dtype=torch.int8, device="cuda")
    with pytest.raises(Q.QasrError) as e:
        g.enc.forward_f32(torch.from_numpy(xf).cuda(), alpha, S_out, y, small)
    assert e.value.status == -6
    g.enc.close()
