"""Pins for the CPU oracle against things other than itself (CPU only).

The paper prints no worked numeric example of the integer pipeline, so the oracle is pinned
by: arbitrary-precision brute force on tiny shapes (a definition written differently: explicit
zero-padded signals and exact rational rounding), a float64 library convolution at real
shapes (exact below 2^53), closed forms, the (2^30, 30) identity, hand-worked rounding and
saturation vectors (tests/golden/requant_vectors.txt) and the float product within 1 LSB
(linearity of Sec. 2.2).
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import qasr_workloads as W
from qasr_workloads.rng import randint_array


# ----------------------------------------------------------------------------- big-int model
def py_round_half_up(fr: Fraction) -> int:
    return math.floor(fr + Fraction(1, 2))


def py_layer(x, w, bias, m, s, residual, stride, dil, pl, pr, depthwise, relu, Cin=None):
    """Nested Python lists, exact ints / rationals.  The conv is written over an explicitly
    zero-padded signal so that it does not share the oracle's index arithmetic."""
    B = len(x)
    Cin = len(x[0]) if Cin is None else Cin
    Tin = len(x[0][0])
    Cout, k = len(w), len(w[0][0])
    y = []
    for b in range(B):
        padded = [[0] * pl + [int(v) for v in x[b][c]] + [0] * pr for c in range(Cin)]
        L = Tin + pl + pr
        yb = []
        for co in range(Cout):
            row = []
            to = 0
            while to * stride + dil * (k - 1) < L:
                start = to * stride
                chans = [co] if depthwise else range(Cin)
                A = int(bias[co]) if bias is not None else 0
                for idx, ci in enumerate(chans):
                    taps = w[co][0] if depthwise else w[co][ci]
                    A += sum(int(taps[j]) * padded[ci][start + j * dil] for j in range(k))
                v = py_round_half_up(Fraction(A * int(m[co]), 2 ** int(s[co])))
                if residual is not None:
                    # one operand [B][C][T], or a list of such operands: all added, one clamp
                    ops_r = residual if isinstance(residual, tuple) else (residual,)
                    v += sum(int(r[b][co][to]) for r in ops_r)
                row.append(min(127, max(0 if relu else -128, v)))
                to += 1
            yb.append(row)
        y.append(yb)
    return y


def _draw(seed, shape, lo, hi, dtype):
    return randint_array(seed, shape, lo, hi, dtype)


# ----------------------------------------------------------------------------- a2-a8 brute force
GEOMS = [(k, stride, dil, pl, pr) for k in (1, 2, 3, 5) for stride in (1, 2) for dil in (1, 2)
         for (pl, pr) in ((0, 0), (2, 1), (dil * (k - 1) // 2, dil * (k - 1) - dil * (k - 1) // 2))]


@pytest.mark.parametrize("depthwise", [False, True])
def test_brute_force_tiny_layers(depthwise):
    n = 0
    for gi, (k, stride, dil, pl, pr) in enumerate(GEOMS):
        for (B, Cin, Cout, T) in ((1, 1, 1, 9), (2, 3, 5, 17), (1, 8, 8, 12)):
            if depthwise:
                Cout = Cin
            if T + pl + pr < dil * (k - 1) + 1:
                continue
            sd = 1000 * gi + 10 * Cin + T + (5 if depthwise else 0)
            x = _draw(sd, (B, Cin, T), -128, 127, np.int8)
            w = _draw(sd + 1, (Cout, 1 if depthwise else Cin, k), -128, 127, np.int8)
            bias = _draw(sd + 2, (Cout,), -300, 300, np.int32) if gi % 3 else None
            # small scales so that outputs are neither all saturated nor all zero
            m = _draw(sd + 3, (Cout,), 1 << 30, (1 << 31) - 1, np.int32)
            s = _draw(sd + 4, (Cout,), 36, 42, np.int32)
            Tout = oracle.out_len(T, k, stride, dil, pl, pr)
            res = _draw(sd + 5, (B, Cout, Tout), -128, 127, np.int8) if gi % 2 else None
            relu = bool(gi % 4 < 2)
            got = oracle.conv1d_int8(x, w, bias, m, s, res, stride=stride, dilation=dil, pad_left=pl,
                                     pad_right=pr, groups=Cin if depthwise else 1, relu=relu)
            ref = py_layer(x.tolist(), w.tolist(), None if bias is None else bias.tolist(), m.tolist(),
                           s.tolist(), None if res is None else res.tolist(), stride, dil, pl, pr,
                           depthwise, relu)
            assert got.shape == (B, Cout, Tout)
            assert got.tolist() == ref, (k, stride, dil, pl, pr, B, Cin, Cout, T)
            n += 1
    assert n > 100


def test_brute_force_is_not_vacuous():
    """The scales above give a spread of outputs (not all 0 / saturated)."""
    x = _draw(7, (2, 8, 40), -128, 127, np.int8)
    w = _draw(8, (8, 8, 5), -127, 127, np.int8)
    m = _draw(9, (8,), 1 << 30, (1 << 31) - 1, np.int32)
    s = np.full(8, 38, np.int32)
    y = oracle.conv1d_int8(x, w, None, m, s, pad_left=2, pad_right=2)
    vals = set(y.reshape(-1).tolist())
    assert len(vals) > 50


# ----------------------------------------------------------------------------- library routine at real shapes
@pytest.mark.parametrize("Cin,Cout,T,k,stride,dil,groups", [
    (64, 256, 400, 33, 2, 1, 1),      # C1-like dense, stride 2
    (256, 256, 200, 33, 1, 1, 256),   # config-0 depthwise
    (256, 256, 200, 1, 1, 1, 1),      # config-0 pointwise
    (512, 512, 300, 87, 1, 2, 512),   # C2-like depthwise, dilation 2
    (96, 80, 150, 29, 1, 2, 1),       # Jasper-epilogue-like dense, dilation 2
    (512, 512, 100, 32, 1, 1, 512),   # even kernel, asymmetric pad
])
def test_accumulators_equal_float64_library_conv(Cin, Cout, T, k, stride, dil, groups):
    tot = dil * (k - 1)
    pl, pr = tot // 2, tot - tot // 2
    x = _draw(11, (2, Cin, T), -128, 127, np.int8)
    w = _draw(12, (Cout, 1 if groups != 1 else Cin, k), -128, 127, np.int8)
    bias = _draw(13, (Cout,), -(1 << 16), 1 << 16, np.int32)
    acc = oracle.conv1d_acc(x, w, bias, stride=stride, dilation=dil, pad_left=pl, pad_right=pr, groups=groups)
    xt = torch.nn.functional.pad(torch.from_numpy(x).double(), (pl, pr))
    ref = torch.nn.functional.conv1d(xt, torch.from_numpy(w).double(), torch.from_numpy(bias).double(),
                                     stride=stride, dilation=dil, groups=groups)
    assert ref.abs().max() < 2 ** 52
    assert np.array_equal(acc, ref.numpy().astype(np.int64))


# ----------------------------------------------------------------------------- closed forms
def _identity_scale(C):
    return np.full(C, 1 << 30, np.int32), np.full(C, 30, np.int32)


def test_one_hot_tap_shifts_the_input():
    C, T, k = 3, 20, 7
    x = _draw(21, (1, C, T), -128, 127, np.int8)
    m, s = _identity_scale(C)
    for j in range(k):
        w = np.zeros((C, 1, k), np.int8)
        w[:, 0, j] = 1
        y = oracle.conv1d_int8(x, w, None, m, s, pad_left=3, pad_right=3, groups=C)
        shift = j - 3                       # y[t] = x[t + shift], zeros outside
        ref = np.zeros_like(x)
        for t in range(T):
            if 0 <= t + shift < T:
                ref[0, :, t] = x[0, :, t + shift]
        assert np.array_equal(y, ref)


def test_identity_pointwise_and_channel_sum():
    C, T = 6, 15
    x = _draw(22, (2, C, T), -128, 127, np.int8)
    m, s = _identity_scale(C)
    eye = np.eye(C, dtype=np.int8).reshape(C, C, 1)
    assert np.array_equal(oracle.conv1d_int8(x, eye, None, m, s), x)
    ones = np.ones((1, C, 1), np.int8)
    acc = oracle.conv1d_acc(x, ones)
    assert np.array_equal(acc[:, 0, :], x.astype(np.int64).sum(axis=1))


def test_weight_order_is_cout_cin_k_and_no_flip():
    """A transposed weight operand or a flipped kernel must fail: single non-zero weight."""
    Cin, Cout, T, k = 3, 4, 10, 3
    x = _draw(23, (1, Cin, T), -128, 127, np.int8)
    w = np.zeros((Cout, Cin, k), np.int8)
    w[2, 1, 0] = 1                           # out-channel 2 reads in-channel 1 at tap 0
    acc = oracle.conv1d_acc(x, w, pad_left=0, pad_right=0)
    assert acc.shape == (1, Cout, T - 2)
    assert np.array_equal(acc[0, 2], x[0, 1, :T - 2].astype(np.int64))
    assert not acc[0, [0, 1, 3]].any()


def test_linearity_in_the_weights():
    x = _draw(24, (1, 5, 30), -128, 127, np.int8)
    w1 = _draw(25, (4, 5, 3), -60, 60, np.int8)
    w2 = _draw(26, (4, 5, 3), -60, 60, np.int8)
    a = oracle.conv1d_acc(x, w1, pad_left=1, pad_right=1)
    b = oracle.conv1d_acc(x, w2, pad_left=1, pad_right=1)
    c = oracle.conv1d_acc(x, (w1 + w2).astype(np.int8), pad_left=1, pad_right=1)
    assert np.array_equal(a + b, c)


def test_channel_prefix_view_reads_first_cin_channels():
    x = _draw(27, (2, 8, 9), -128, 127, np.int8)
    w = _draw(28, (4, 1, 4), -127, 127, np.int8)
    m, s = _identity_scale(4)
    s[:] = 36
    full = oracle.conv1d_int8(x, w, None, m, s, pad_left=1, pad_right=2, groups=4, Cin=4, x_batch_stride=8 * 9)
    sliced = oracle.conv1d_int8(np.ascontiguousarray(x[:, :4]), w, None, m, s, pad_left=1, pad_right=2, groups=4)
    assert np.array_equal(full, sliced)


# ----------------------------------------------------------------------------- a6 requant
def test_identity_requant_on_int32_edges_and_samples():
    edges = [-(1 << 31), -(1 << 31) + 1, -129, -128, -1, 0, 1, 127, 128, (1 << 31) - 2, (1 << 31) - 1]
    rnd = [int(v) for v in _draw(31, (2000,), -(1 << 31), (1 << 31) - 1, np.int64)]
    for A in edges + rnd:
        assert oracle.requant_scalar(A, 1 << 30, 30) == A


def test_hand_worked_vectors(golden):
    rows = golden("requant_vectors.txt")
    assert len(rows) >= 24
    for A, m, s, v, y, yr in (map(int, r) for r in rows):
        assert oracle.requant_scalar(A, m, s) == v, (A, m, s)
        acc = np.array([[[A]]], np.int32)
        mm, ss = np.array([m], np.int32), np.array([s], np.int32)
        assert oracle.requant(acc, None, mm, ss).item() == y
        assert oracle.requant(acc, None, mm, ss, relu=True).item() == yr


def test_requant_equals_exact_rational_rounding_everywhere():
    rnd = np.random.RandomState(5)
    cases = [(A, m, s) for A in (-(1 << 31), -1, 0, 1, (1 << 31) - 1)
             for m in (0, 1, 1 << 30, (1 << 31) - 1) for s in (1, 2, 30, 31, 32, 33, 44, 62)]
    for _ in range(3000):
        cases.append((int(rnd.randint(-(1 << 31), 1 << 31)), int(rnd.randint(0, 1 << 31)), int(rnd.randint(1, 63))))
    for A, m, s in cases:
        assert oracle.requant_scalar(A, m, s) == py_round_half_up(Fraction(A * m, 1 << s)), (A, m, s)


def test_float_dequantised_product_within_one_lsb():
    """Sec. 2.2: S_W S_x Conv(q_W, q_x); the dyadic pair (m, s) stands for the real scale
    m / 2^s, so the float product must agree with the integer rescale to within 1 LSB, and
    exactly when the product is not within 1e-6 of a tie."""
    rnd = np.random.RandomState(6)
    A = rnd.randint(-(1 << 28), 1 << 28, size=20000).astype(np.int64)
    m = rnd.randint(1 << 30, 1 << 31, size=20000).astype(np.int64)
    s = rnd.randint(36, 45, size=20000).astype(np.int64)
    f = A.astype(np.float64) * (m.astype(np.float64) / np.exp2(s.astype(np.float64)))
    fr = np.floor(f + 0.5)
    got = np.array([oracle.requant_scalar(int(a), int(mm), int(ss)) for a, mm, ss in zip(A, m, s)], np.float64)
    assert np.abs(got - fr).max() <= 1
    far = np.abs((f + 0.5) - np.round(f + 0.5)) > 1e-6
    assert far.mean() > 0.99 and np.array_equal(got[far], fr[far])


# ----------------------------------------------------------------------------- a7, a8 residual + clamp
def test_residual_is_added_before_the_single_clamp():
    """rq = 200 (beyond int8), r = -100  =>  100, not clamp(127 - 100) = 27."""
    acc = np.array([[[200, 200, -300, 50]]], np.int32)
    r = np.array([[[-100, 100, 127, -128]]], np.int8)
    m, s = _identity_scale(1)
    assert oracle.requant(acc, None, m, s, r).reshape(-1).tolist() == [100, 127, -128, -78]
    assert oracle.requant(acc, None, m, s, r, relu=True).reshape(-1).tolist() == [100, 127, 0, 0]


def test_bias_is_added_before_the_rescale():
    acc = np.array([[[3], [3]]], np.int32)
    bias = np.array([1, -1], np.int32)
    m, s = np.full(2, 1 << 30, np.int32), np.full(2, 31, np.int32)     # halve, ties up
    assert oracle.requant(acc, bias, m, s).reshape(-1).tolist() == [2, 1]


def test_per_channel_scales_are_indexed_by_output_channel():
    x = np.full((1, 2, 4), 64, np.int8)
    w = np.zeros((3, 2, 1), np.int8)
    w[:, 0, 0] = 1
    m = np.full(3, 1 << 30, np.int32)
    s = np.array([30, 31, 32], np.int32)
    y = oracle.conv1d_int8(x, w, None, m, s)
    assert y[0, :, 0].tolist() == [64, 32, 16]


def test_overflow_is_detected():
    Cin, k = 2200, 64                      # fan-in 140800 * 128 * 128 > 2^31
    x = np.full((1, Cin, k), -128, np.int8)
    w = np.full((1, Cin, k), -128, np.int8)
    m, s = _identity_scale(1)
    with pytest.raises(OverflowError):
        oracle.conv1d_int8(x, w, None, m, s)


def test_several_residual_operands_are_summed_before_the_one_clamp():
    """Dense-residual layers: v = requant(A) + sum of the operands, then one clamp.  Hand-worked:
    the main branch gives 100 (x = 100 through the identity scale); operands (100, -100) leave
    100, where saturating after the first addition would give 127 - 100 = 27; operands
    (-128, -128, 127) on a main value of 120 give 120 - 129 = -9."""
    x = np.array([[[100, 120]]], dtype=np.int8)
    w = np.ones((1, 1, 1), dtype=np.int8)
    m, s = _identity_scale(1)
    r = lambda a, b: np.array([[[a, b]]], dtype=np.int8)
    y = oracle.conv1d_int8(x, w, None, m, s, [r(100, -128), r(-100, -128), r(0, 127)])
    assert y.reshape(-1).tolist() == [100, -9]
    # one operand in a list is the ordinary residual layer; with ReLU the clamp is [0, 127]
    assert np.array_equal(oracle.conv1d_int8(x, w, None, m, s, [r(5, -7)]), oracle.conv1d_int8(x, w, None, m, s, r(5, -7)))
    assert oracle.conv1d_int8(x, w, None, m, s, [r(-100, 10), r(-100, 10)], relu=True).reshape(-1).tolist() == [0, 127]
    # brute force against the big-integer definition on a small dense layer with three operands
    xs = _draw(5, (2, 3, 9), -128, 127, np.int8)
    ws = _draw(6, (4, 3, 3), -127, 127, np.int8)
    bias = _draw(7, (4,), -300, 300, np.int32)
    mm = _draw(8, (4,), 1 << 30, (1 << 31) - 1, np.int32)
    ss = np.full(4, 38, np.int32)
    rs = [_draw(9 + i, (2, 4, 9), -128, 127, np.int8) for i in range(3)]
    got = oracle.conv1d_int8(xs, ws, bias, mm, ss, rs, pad_left=1, pad_right=1)
    ref = py_layer(xs.tolist(), ws.tolist(), bias.tolist(), mm.tolist(), ss.tolist(), tuple(r_.tolist() for r_ in rs),
                   1, 1, 1, 1, False, False)
    assert got.tolist() == ref


def test_output_batch_stride_places_blocks_and_reads_the_residual_there():
    """y_batch_stride: item b's [Cout, Tout] block starts at b * stride, in the output and in the
    residual operand alike; nothing else is read or written.  Checked against the big-integer
    layer, whose operands are gathered from / scattered to the strided layout here."""
    B, Cin, Cout, T, k = 3, 3, 5, 17, 3
    x = _draw(41, (B, Cin, T), -128, 127, np.int8)
    w = _draw(42, (Cout, Cin, k), -128, 127, np.int8)
    bias = _draw(43, (Cout,), -300, 300, np.int32)
    m = _draw(44, (Cout,), 1 << 30, (1 << 31) - 1, np.int32)
    s = _draw(45, (Cout,), 36, 40, np.int32)
    Tout = oracle.out_len(T, k, 1, 1, 1, 1)
    for ybs in (Cout * Tout, Cout * Tout + 4, Cout * Tout + 23):
        res = _draw(46 + ybs, (B, ybs), -128, 127, np.int8)
        res_blocks = [[[int(res[b, co * Tout + t]) for t in range(Tout)] for co in range(Cout)] for b in range(B)]
        for r_flat, r_blocks in ((None, None), (res, res_blocks)):
            got = oracle.conv1d_int8(x, w, bias, m, s, r_flat, pad_left=1, pad_right=1, y_batch_stride=ybs,
                                     y_fill=55)
            ref = py_layer(x.tolist(), w.tolist(), bias.tolist(), m.tolist(), s.tolist(), r_blocks, 1, 1, 1, 1,
                           False, False)
            assert got.shape == (B, ybs)
            assert got[:, : Cout * Tout].reshape(B, Cout, Tout).tolist() == ref
            assert (got[:, Cout * Tout:] == 55).all()
    # two residual operands at the stride
    ybs = Cout * Tout + 9
    rs = [_draw(60 + i, (B, ybs), -128, 127, np.int8) for i in range(2)]
    blocks = tuple([[[int(r[b, co * Tout + t]) for t in range(Tout)] for co in range(Cout)] for b in range(B)]
                   for r in rs)
    got = oracle.conv1d_int8(x, w, bias, m, s, rs, pad_left=1, pad_right=1, y_batch_stride=ybs, y_fill=-9)
    ref = py_layer(x.tolist(), w.tolist(), bias.tolist(), m.tolist(), s.tolist(), blocks, 1, 1, 1, 1, False, False)
    assert got[:, : Cout * Tout].reshape(B, Cout, Tout).tolist() == ref
    assert (got[:, Cout * Tout:] == -9).all()


# ----------------------------------------------------------------------------- a9 wiring on tiny encoders
LN2_40 = Fraction(6931471805599453094172321214581765680755, 10 ** 40)    # ln 2 to 40 decimals


def py_act_constants(S: float, u: int):
    """The exponential's three integer constants from their defining inequalities, in exact rationals
    (S is the double the workload drew; the refined step is S / 2^u): the largest integers with
    q_ln2 S' <= ln 2,  q_b S' <= 1.353,  q_c 0.3585 S'^2 <= 0.344."""
    Sr = Fraction(S) / 2 ** u
    q_ln2 = math.floor(LN2_40 / Sr)
    q_b = math.floor(Fraction(1353, 1000) / Sr)
    q_c = math.floor(Fraction(344, 1000) / (Fraction(3585, 10000) * Sr * Sr))
    return q_ln2, q_b, q_c


def py_iexp(r: int, q_ln2: int, q_b: int, q_c: int) -> int:
    """Integer exponential of r <= 0 in unbounded integers: the power of two is split off by a
    floor division, the second-order polynomial is evaluated on the remainder."""
    assert r <= 0
    z = (-r) // q_ln2
    p = r + z * q_ln2
    assert -q_ln2 < p <= 0
    return ((p + q_b) ** 2 + q_c) // 2 ** z


def py_sigmoid_code(q: int, u: int, q_ln2: int, q_b: int, q_c: int) -> int:
    """Sigmoid as the two-way softmax of (x, 0), 15 fractional bits."""
    E = py_iexp(-abs(q) * 2 ** u, q_ln2, q_b, q_c)
    E0 = q_b * q_b + q_c
    return ((E0 if q >= 0 else E) * 2 ** 15) // (E0 + E)


def py_act_in_place(a, y):
    """An op's activation applied to its output [B][C][T] (nested lists) as the encoder does it:
    sigmoid / swish replace every value; GLU (value = first half of the channels, gate = second
    half) writes its C/2 channels over the value half and leaves the gate half as it was.  Each
    result goes back to int8 by the activation's own dyadic rescale (round half up) and clamp."""
    kind, u, m, s = a["kind"], a["u"], a["m"], a["s"]
    cst = py_act_constants(a["S"], u)
    sig = lambda q: py_sigmoid_code(q, u, *cst)
    out = [[list(row) for row in item] for item in y]
    for b, item in enumerate(y):
        C = len(item)
        n_val = C // 2 if kind == 3 else C
        for ch in range(n_val):
            for t, q in enumerate(item[ch]):
                if kind == 1:
                    v = sig(q)
                elif kind == 2:
                    v = q * sig(q)
                else:
                    v = q * sig(item[n_val + ch][t])
                out[b][ch][t] = min(127, max(-128, py_round_half_up(Fraction(v * m, 2 ** s))))
    return out


def py_encoder(net, params, x):
    slots = {0: x.tolist()}
    for op, p in zip(net.ops, params):
        res = slots[op.res_slot] if op.res_slot >= 0 else None
        if getattr(op, "more_res", None):
            res = (res,) + tuple(slots[r] for r in op.more_res)
        y = py_layer(
            slots[op.in_slot], p["w"].tolist(), None if p["bias"] is None else p["bias"].tolist(),
            p["m"].tolist(), p["s"].tolist(), res, op.stride, op.dilation, op.pad_left, op.pad_right,
            op.depthwise, bool(op.flags & 1), Cin=op.Cin)
        if op.act:
            y = py_act_in_place(p["act"], y)
        slots[op.out_slot] = y
    return slots[net.ops[-1].out_slot]


@pytest.mark.parametrize("cfg,w_bits", [(0, 8), (1, 8), (2, 8), (3, 8), (4, 8), (5, 8), (6, 8), (7, 8), (1, 6)])
def test_tiny_encoders_match_big_int_composition(cfg, w_bits):
    net = W.tiny_config(cfg)
    for seed in (1, 2):
        # scales chosen for the tiny fan-in so that layers neither saturate nor vanish
        params = W.draw_net_params(net, seed, s_lo=37 - (8 - w_bits), s_hi=38 - (8 - w_bits), bias_mag=300,
                                   w_bits=w_bits)
        if cfg == 5:
            # activation outputs at the tiny network's range: swish of codes up to 127 with a
            # sigmoid code of 15 bits is below 2^22; a ratio near 2^-15 brings it back to int8
            for p in params:
                if p.get("act"):
                    p["act"]["s"] = 45 if p["act"]["kind"] != 1 else 38
        x = W.draw_input(net, seed)
        y, outs = oracle.encoder_forward(net, params, x, keep=True)
        assert y.tolist() == py_encoder(net, params, x)
        assert y.shape == (net.B, net.Cout, net.Tout)
        live = [len(set(o.reshape(-1).tolist())) for o in outs]
        assert min(live) >= 5, live        # no layer collapsed to a constant


def test_activation_hook_layouts_against_the_big_int_form():
    """apply_act on its own: every kind, against the unbounded-integer form, on a tensor that holds
    every int8 code in both halves; GLU's output sits in the first half, the gate half is unchanged;
    the exponential's constants equal the ones fixed by their defining inequalities."""
    B, C, T = 2, 6, 256
    codes = np.arange(-128, 128, dtype=np.int8)
    y = np.empty((B, C, T), dtype=np.int8)
    for b in range(B):
        for ch in range(C):
            y[b, ch] = np.roll(codes, 37 * ch + 11 * b)
    for kind, s in ((1, 38), (2, 45), (3, 45)):
        for S, u in ((0.05, 8), (6.0 / 127.0, 8), (0.02, 4)):
            a = {"kind": kind, "S": S, "u": u, "m": (1 << 30) + 123456789, "s": s}
            c = oracle.iexp_constants(S, u)
            assert (c["q_ln2"], c["q_b"], c["q_c"]) == py_act_constants(S, u)
            got = oracle.apply_act(a, y)
            assert got.shape == y.shape and got.dtype == np.int8
            assert got.tolist() == py_act_in_place(a, y.tolist()), (kind, S, u)
            if kind == 3:
                assert np.array_equal(got[:, C // 2:], y[:, C // 2:])
                assert not np.array_equal(got[:, : C // 2], y[:, : C // 2])
            assert len(set(got[:, : (C // 2 if kind == 3 else C)].reshape(-1).tolist())) > 20


def test_config0_oracle_is_not_degenerate():
    net = W.build_config(0)
    params = W.draw_net_params(net, 1)
    x = W.draw_input(net, 1)
    y, outs = oracle.encoder_forward(net, params, x, keep=True)
    for o in outs:
        flat = o.reshape(-1)
        sat = np.mean((flat == 127) | (flat == -128))
        assert 0.02 < sat < 0.98 and len(set(flat.tolist())) > 100


# ----------------------------------------------------------------------------- quantiser / dequantiser
def test_quantiser_hand_worked_codes(golden):
    """Eq. 1, b = 8: clip, divide by S = alpha / 127, round to nearest with ties to even."""
    rows = [(float(a), float(x), int(q)) for a, x, q in golden("quantizer_vectors.txt")]
    assert len(rows) >= 25
    for alpha, x, q in rows:
        got = int(oracle.quantize(np.array([x], dtype=np.float32), alpha)[0])
        assert got == q, (alpha, x, got, q)


def test_quantiser_nan_maps_to_zero_and_codes_stay_in_range():
    x = np.array([np.nan, 3.0, -np.nan], dtype=np.float32)
    assert oracle.quantize(x, 10.0).tolist() == [0, 38, 0]          # 3 / (10/127) = 38.1
    big = randint_array(7, (4096,), -10**6, 10**6, np.int32).astype(np.float32) / 1000.0
    q = oracle.quantize(big, 3.25)
    assert q.min() == -127 and q.max() == 127                        # Eq. 1's range, never -128


@pytest.mark.parametrize("alpha", [127.0, 1.0, 0.037, 6.5, 1000.0, 2.0 ** -20])
def test_quantiser_matches_float64_recomputation_away_from_ties(alpha):
    """The same formula evaluated in float64: identical codes wherever x / S is not within
    1e-3 of a tie (single-precision division cannot move the quotient that far), and never more
    than one code apart."""
    rng = np.random.default_rng(int(alpha * 1000) + 3)
    x = (rng.standard_normal(200000) * alpha * 0.7).astype(np.float32)
    q = oracle.quantize(x, alpha).astype(np.int64)
    S = np.float64(np.float32(alpha) / np.float32(127.0))
    u = np.clip(x.astype(np.float64), -np.float64(np.float32(alpha)), np.float64(np.float32(alpha))) / S
    ref = np.rint(u).astype(np.int64)
    assert np.abs(q - ref).max() <= 1
    away = np.abs(u - np.floor(u) - 0.5) > 1e-3
    assert away.sum() > 150000 and np.array_equal(q[away], ref[away])


@pytest.mark.parametrize("alpha", [127.0, 1.0, 0.037, 6.5, 2.0 ** -20])
def test_dequantise_then_quantise_is_the_identity_on_all_codes(alpha):
    """Q(DQ(q, S), S) = q for every code of Eq. 1's range, DQ(q, S) = S q in single precision."""
    S = np.float32(alpha) / np.float32(127.0)
    q = np.arange(-127, 128, dtype=np.int8)
    xq = oracle.dequantize(q, float(S))
    assert np.array_equal(xq, (S * q.astype(np.float32)).astype(np.float32))
    assert xq.dtype == np.float32 and xq[127] == 0.0 and xq[254] > 0 > xq[0]
    assert np.array_equal(oracle.quantize(xq, alpha), q)


def test_quantiser_error_bound_symmetry_and_monotonicity():
    """|DQ(Q(x)) - clip(x)| <= S / 2 (plus rounding of the two float32 operations), Q(-x) = -Q(x),
    and Q is non-decreasing in x."""
    alpha = 4.75
    S = np.float32(alpha) / np.float32(127.0)
    x = np.sort((np.random.default_rng(11).standard_normal(100000) * 3.0).astype(np.float32))
    q = oracle.quantize(x, alpha)
    back = oracle.dequantize(q, float(S)).astype(np.float64)
    err = np.abs(back - np.clip(x.astype(np.float64), -alpha, alpha))
    assert err.max() <= float(S) * 0.5 * (1 + 1e-5)
    assert err.max() > float(S) * 0.49                               # the bound is attained: not vacuous
    assert np.array_equal(oracle.quantize(-x, alpha).astype(np.int32), -q.astype(np.int32))
    assert np.all(np.diff(q.astype(np.int32)) >= 0)


# ----------------------------------------------------------------------------- integer activations
# (Sec. 2.2, last sentence: Sigmoid, Softmax and Swish through second-order polynomials)
SCALES = [(8.0 / 127, 8), (4.0 / 127, 8), (0.1, 6), (16.0 / 127, 10), (1.0 / 127, 4)]


def test_exp_polynomial_error_on_its_interval():
    """The real-valued polynomial itself, before any integer step."""
    p = np.linspace(-math.log(2.0), 0.0, 20001)
    assert np.max(np.abs(0.3585 * (p + 1.353) ** 2 + 0.344 - np.exp(p))) < 2.2e-3


def test_iexp_hand_worked_values(golden):
    c = oracle.iexp_constants(0.1, 0)
    assert (c["q_ln2"], c["q_b"], c["q_c"]) == (6, 13, 95)
    for kind, arg, val in golden("iexp_vectors.txt"):
        got = oracle.iexp(int(arg), c) if kind == "iexp" else oracle.sigmoid_code(int(arg), c)
        assert got == int(val), (kind, arg)


@pytest.mark.parametrize("S,u", SCALES)
def test_iexp_against_float_exp_and_its_structure(S, u):
    c = oracle.iexp_constants(S, u)
    Sr = S / 2 ** u
    unit = 0.3585 * Sr * Sr
    assert c["q_ln2"] == math.floor(math.log(2.0) / Sr)
    assert oracle.iexp(0, c) == c["q_b"] ** 2 + c["q_c"]
    rs = sorted({-int(v) for v in np.linspace(0, 24.0 / Sr, 4001)}, reverse=True)
    prev = None
    for r in rs:
        E = oracle.iexp(r, c)
        # 2.2e-3 of the polynomial (on values >= 1/2, so 4.4e-3 relative), the floors of the three constants (relative 1/q each, and
        # z/q_ln2 accumulated over the z halvings), one unit of the final floor
        z = -r // c["q_ln2"]
        tol = (2.2e-3 / 0.5 + 3.0 / c["q_b"] + (z + 1) * 1.0 / c["q_ln2"]) * math.exp(r * Sr) + unit
        assert abs(E * unit - math.exp(r * Sr)) <= tol, (r, E)
        assert prev is None or E <= prev            # non-increasing as the argument falls
        prev = E
        assert oracle.iexp(r - c["q_ln2"], c) == E >> 1     # exactly halved per q_ln2
    assert oracle.iexp(-70 * c["q_ln2"], c) == 0


@pytest.mark.parametrize("S,u", SCALES)
def test_sigmoid_code_against_the_float_function(S, u):
    c = oracle.iexp_constants(S, u)
    codes = [oracle.sigmoid_code(q, c) for q in range(-128, 128)]
    ref = [1.0 / (1.0 + math.exp(-S * q)) for q in range(-128, 128)]
    assert max(abs(a / 32768.0 - b) for a, b in zip(codes, ref)) < 2.5e-3
    assert codes[128] == 16384                                    # sigmoid(0) = 1/2 exactly
    assert all(b >= a for a, b in zip(codes, codes[1:]))          # monotone
    for q in range(1, 128):                                       # sigma(q) + sigma(-q) = 1 up to one floor
        assert codes[128 + q] + codes[128 - q] in (32767, 32768)
    assert all(0 <= v <= 32768 for v in codes)


def dyadic_of(ratio: float):
    """(m, s) with m * 2^-s ~ ratio and 2^30 <= m < 2^31 (a test helper, not the method)."""
    e = math.floor(math.log2(ratio))
    s = 30 - e
    return int(round(ratio * 2.0 ** s)), s


@pytest.mark.parametrize("S,u", SCALES[:4])
def test_swish_and_sigmoid_outputs_within_one_code_of_the_float_function(S, u):
    c = oracle.iexp_constants(S, u)
    q = np.arange(-128, 128, dtype=np.int8).reshape(1, 1, 256)
    x = S * q.astype(np.float64)
    sig = 1.0 / (1.0 + np.exp(-x))
    # swish at the input's own scale, sigmoid at 2^-7
    m, s = dyadic_of(1.0 / 32768.0)
    y = oracle.act(oracle.ACT_SWISH, q, c, m, s).astype(np.int64)
    assert np.max(np.abs(y - np.clip(np.floor(x * sig / S + 0.5), -128, 127))) <= 1
    m, s = dyadic_of(128.0 / 32768.0)
    y = oracle.act(oracle.ACT_SIGMOID, q, c, m, s).astype(np.int64)
    assert np.max(np.abs(y - np.clip(np.floor(sig * 128.0 + 0.5), -128, 127))) <= 1
    # swish is negative only for negative inputs and never below its float minimum by more than a code
    sw = oracle.act(oracle.ACT_SWISH, q, c, *dyadic_of(1.0 / 32768.0)).reshape(-1).astype(np.int64)
    assert np.all(sw[128:] >= 0) and np.all(sw[:128] <= 0)
    assert sw.min() >= math.floor(-0.2785 / S) - 1


def test_glu_all_pairs_within_one_code_and_halves_are_value_then_gate():
    S, u = 6.0 / 127, 8
    c = oracle.iexp_constants(S, u)
    a, g = np.meshgrid(np.arange(-128, 128), np.arange(-128, 128), indexing="ij")
    x = np.stack([a.reshape(-1), g.reshape(-1)]).astype(np.int8).reshape(1, 2, -1)   # C = 1
    m, s = dyadic_of(1.0 / 32768.0)
    y = oracle.act(oracle.ACT_GLU, x, c, m, s).reshape(-1).astype(np.int64)
    ref = a.reshape(-1) * (1.0 / (1.0 + np.exp(-S * g.reshape(-1).astype(np.float64))))
    assert np.max(np.abs(y - np.clip(np.floor(ref + 0.5), -128, 127))) <= 1
    # a gate far to the right passes the value, far to the left blocks it
    x2 = np.zeros((2, 2, 3), dtype=np.int8)
    x2[:, 0] = [5, -7, 100]
    x2[0, 1] = 127                              # batch item 0: gates far right
    x2[1, 1] = -128                             # batch item 1: gates far left
    c2 = oracle.iexp_constants(0.2, 6)
    y2 = oracle.act(oracle.ACT_GLU, x2, c2, m, s)
    assert y2[0, 0].tolist() == [5, -7, 100] and y2[1, 0].tolist() == [0, 0, 0]
    # two channels: channel c is gated by channel C + c, not by its neighbour
    x3 = np.zeros((1, 4, 1), dtype=np.int8)
    x3[0, :, 0] = [100, 100, 127, -128]
    assert oracle.act(oracle.ACT_GLU, x3, c2, m, s)[0, :, 0].tolist() == [100, 0]


@pytest.mark.parametrize("S,u,L", [(0.002, 0, 37), (0.01, 2, 400), (1.0 / 64, 4, 9)])
def test_softmax_against_the_float_function_and_its_invariants(S, u, L):
    c = oracle.iexp_constants(S, u)
    x = randint_array(7, (16, L), -int(6 / S), int(6 / S), np.int32)
    y = oracle.softmax(x, c).astype(np.int64)
    z = S * x.astype(np.float64)
    ref = np.exp(z - z.max(axis=1, keepdims=True))
    ref = ref / ref.sum(axis=1, keepdims=True)
    # one code of the floor plus the polynomial's relative error on a probability <= 1
    assert np.max(np.abs(y - ref * 128.0)) <= 1.0 + 128 * 6.0e-3
    assert np.all(y >= 0) and np.all(y.sum(axis=1) <= 128) and np.all(y.sum(axis=1) >= 128 - L)
    assert np.array_equal(oracle.softmax(x + 12345, c), y)                    # shift invariance
    perm = np.argsort(randint_array(8, (L,), 0, 1 << 30, np.int64))
    assert np.array_equal(oracle.softmax(x[:, perm], c), y[:, perm])          # permutation
    # order is kept: a larger logit never gets a smaller code
    i = np.argsort(x[0])
    assert np.all(np.diff(y[0][i]) >= 0)


def test_softmax_closed_forms():
    c = oracle.iexp_constants(0.01, 2)
    for L in (1, 2, 3, 5, 128, 200):
        assert oracle.softmax(np.full((1, L), -77, dtype=np.int32), c)[0].tolist() == [min(127, 128 // L)] * L
    x = np.full((1, 50), -2_000_000_000, dtype=np.int32)
    x[0, 17] = 2_000_000_000                                                  # int32 extremes do not wrap
    y = oracle.softmax(x, c)[0]
    assert y[17] == 127 and int(np.abs(y).sum()) == 127
    # two logits ln 3 apart: probabilities 3/4 and 1/4 -> 96 and 32 within a code
    d = int(round(math.log(3.0) / 0.01))
    y = oracle.softmax(np.array([[d, 0]], dtype=np.int32), c)[0]
    assert abs(int(y[0]) - 96) <= 1 and abs(int(y[1]) - 32) <= 1


def test_iexp_constants_reject_unusable_scales():
    for S, u in [(0.0, 0), (-1.0, 0), (float("nan"), 0), (float("inf"), 0), (1.0, 0), (0.1, -1), (0.1, 17), (1e-9, 8)]:
        with pytest.raises(ValueError):
            oracle.iexp_constants(S, u)


# ----------------------------------------------------------------------------- offline calibration helpers
def test_observer_min_max():
    x = _draw(3, (100003,), -(1 << 20), 1 << 20, np.int32).astype(np.float32) * np.float32(1e-3)
    x[[5, 77, 4096]] = np.nan
    mm = oracle.minmax(x)
    assert mm[0] == np.nanmin(x) and mm[1] == np.nanmax(x)
    # running: a second tensor only widens the range; NaNs and an empty tensor change nothing
    y = np.array([np.nan, 1e9, np.nan], dtype=np.float32)
    mm2 = oracle.minmax(y, start=mm)
    assert mm2[0] == mm[0] and mm2[1] == np.float32(1e9)
    assert oracle.minmax(np.array([np.nan] * 7, dtype=np.float32), start=(3.0, -4.0)).tolist() == [3.0, -4.0]
    assert oracle.minmax(np.zeros(0, dtype=np.float32)).tolist() == [np.inf, -np.inf]
    assert oracle.minmax(np.array([-np.inf, 2.5, np.inf], dtype=np.float32)).tolist() == [-np.inf, np.inf]
    assert oracle.minmax(np.array([1.0, -2.0, 5.0], dtype=np.float32)).tolist() == [-2.0, 5.0]


def test_dyadic_form_of_a_multiplier(golden):
    for row in golden("calibration_vectors.txt"):
        if row[0] == "dyadic":
            assert oracle.dyadic(float(row[1])) == (int(row[2]), int(row[3])), row
    # nearest: |m 2^-s - M| <= 2^-s / 2, exactly, over twelve decades
    for i, e in enumerate(range(-24, 12)):
        M = float(_draw(40 + i, (1,), 1 << 20, 1 << 30, np.int64)[0]) * 2.0 ** (e - 25) * 1.0000001
        m, s = oracle.dyadic(M)
        assert (1 << 30) <= m < (1 << 31) and 1 <= s <= 62
        assert abs(Fraction(m, 2 ** s) - Fraction(M)) <= Fraction(1, 2 ** (s + 1))
    # just below a power of two the mantissa rounds up and carries
    assert oracle.dyadic(0.5 - 1e-13) == (1 << 30, 31)
    for bad in (0.0, -1.0, float("nan"), float("inf"), 2.0 ** 31, 2.0 ** -40):
        with pytest.raises(ValueError):
            oracle.dyadic(bad)


def test_fold_and_quantize_hand_worked(golden):
    row = [r for r in golden("calibration_vectors.txt") if r[0] == "fold"][0]
    qw, bq, m, s, Sw, bad = oracle.fold_quantize(np.array([[[1.0, -4.0]]]), [0.5], [2.0], [0.125], [0.25], [3.0], 1.0, 0.5, 0.25)
    assert bad == 0 and qw.reshape(-1).tolist() == [int(row[1]), int(row[2])]
    assert (int(bq[0]), int(m[0]), int(s[0])) == (int(row[3]), int(row[4]), int(row[5]))
    assert Sw[0] == np.float32(4.0) / np.float32(127.0)


def test_folded_integer_layer_reproduces_the_float_layer_with_batchnorm():
    """The point of the helper: conv + BatchNorm in floating point against the integer layer built
    from its outputs (quantised input, q_w, bias, (m, s)), within the quantisation error."""
    Cout, Cin, k, T = 6, 5, 3, 40
    g = lambda sd, shape, lo, hi: _draw(sd, shape, -1000, 1000, np.int32).astype(np.float64) / 1000.0 * (hi - lo) / 2 + (hi + lo) / 2
    w = g(1, (Cout, Cin, k), -0.5, 0.5); b = g(2, (Cout,), -0.3, 0.3)
    gamma = g(3, (Cout,), 0.5, 1.5); gamma[1] = -gamma[1]                      # a negative gain flips the channel
    beta = g(4, (Cout,), -0.4, 0.4); mu = g(5, (Cout,), -0.5, 0.5); var = g(6, (Cout,), 0.2, 2.0)
    eps = 1e-3
    x = g(7, (1, Cin, T), -2.0, 2.0)
    # float model (float64): valid convolution, then BatchNorm
    yf = np.zeros((1, Cout, T - k + 1))
    for c in range(Cout):
        for t in range(T - k + 1):
            yf[0, c, t] = np.sum(w[c] * x[0, :, t:t + k]) + b[c]
    yf = gamma[None, :, None] * (yf - mu[None, :, None]) / np.sqrt(var[None, :, None] + eps) + beta[None, :, None]
    S_x = 2.0 / 127
    S_y = float(np.abs(yf).max()) / 127
    qx = oracle.quantize(x.astype(np.float32), 2.0)
    qw, bq, m, s, Sw, bad = oracle.fold_quantize(w, b, gamma, beta, mu, var, eps, S_x, S_y)
    assert bad == 0
    yi = oracle.conv1d_int8(qx, qw, bq, m, s)
    # input rounding (S_x / 2 per tap through the folded weights), weight rounding (S_w / 2 per tap
    # on |x| <= 2), the output's own half step; all in units of S_y
    wf = np.abs(w * (gamma / np.sqrt(var + eps))[:, None, None]).sum(axis=(1, 2))
    bound = (wf * S_x / 2 + Cin * k * Sw / 2 * 2.0) / S_y + 0.5 + 0.5
    err = np.abs(yi[0].astype(np.float64) - yf[0] / S_y)
    assert np.all(err.max(axis=1) <= bound), (err.max(axis=1), bound)
    assert np.corrcoef(yi.reshape(-1), yf.reshape(-1))[0, 1] > 0.999
    # every channel uses its full code range, and the scales are the per-channel maxima
    assert np.all(np.abs(qw.reshape(Cout, -1)).max(axis=1) == 127)
    f32 = (gamma.astype(np.float32) / np.sqrt(var.astype(np.float32) + np.float32(eps)))
    assert np.allclose(Sw, np.abs(w.astype(np.float32) * f32[:, None, None]).reshape(Cout, -1).max(axis=1) / 127, rtol=1e-6)


def test_fold_with_identity_batchnorm_is_plain_per_channel_quantisation():
    w = _draw(11, (4, 3, 5), -1000, 1000, np.int32).astype(np.float32) / np.float32(777.0)
    w[2] = 0.0                                                                  # an all-zero channel
    one, zero = np.ones(4, np.float32), np.zeros(4, np.float32)
    qw, bq, m, s, Sw, bad = oracle.fold_quantize(w, None, one, zero, zero, one, 0.0, 0.25, 0.5)
    assert bad == 0 and np.all(bq == 0) and np.all(qw[2] == 0) and Sw[2] == 1.0
    for c in (0, 1, 3):
        Sc = np.abs(w[c]).max() / np.float32(127.0)
        assert Sw[c] == Sc and np.array_equal(qw[c], np.rint(w[c] / Sc).astype(np.int8))
        assert (int(m[c]), int(s[c])) == oracle.dyadic(float(Sc) * 0.25 / 0.5)
    # a multiplier out of range and a bias beyond int32 are counted, not silently wrapped
    assert oracle.fold_quantize(w[:1], [1e9], one[:1], zero[:1], zero[:1], one[:1], 0.0, 1e-6, 0.5)[5] == 1
    assert oracle.fold_quantize(w[:1], None, one[:1], zero[:1], zero[:1], one[:1], 0.0, 1e-30, 1.0)[5] == 1
