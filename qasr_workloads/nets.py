"""Layer geometry and activation-slot wiring of the five benchmark configurations.

Every network is a flat list of 1-D convolution ops over numbered activation slots
(slot 0 = network input, never written).  An op reads `in_slot`, optionally adds the int8
tensor in `res_slot` in its epilogue, and writes `out_slot`.  Only shapes and wiring live
here; what an op computes is defined elsewhere (once by the CPU oracle, once by the HIP
library).

Shapes follow the benchmark configuration texts: QuartzNet (time-channel-separable
modules, five block types 256/k33, 256/k39, 512/k51, 512/k63, 512/k75), Jasper (dense
convs, ten blocks) and a Conformer-L-shaped stack of integer linear layers.  These are the
model families the paper evaluates (Sec. 3, Table 1; Sec. 3.2 for QuartzNet 5x5/15x5).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from .rng import randint_array, tensor_seed

FLAG_RELU = 1


@dataclass
class OpSpec:
    name: str
    Cin: int
    Cout: int
    Tin: int
    k: int = 1
    stride: int = 1
    dilation: int = 1
    pad_left: int = 0
    pad_right: int = 0
    groups: int = 1
    x_batch_stride: int = 0      # elements; 0 => Cin*Tin
    flags: int = 0
    has_bias: bool = True
    in_slot: int = 0
    res_slot: int = -1
    out_slot: int = 1
    act: int = 0                 # 0 none, 1 sigmoid, 2 swish, 3 GLU (applied in place to the output)
    more_res: List[int] = field(default_factory=list)   # further residual operands (slots), summed with res_slot's

    @property
    def Tout(self) -> int:
        return out_len(self.Tin, self.k, self.stride, self.dilation, self.pad_left, self.pad_right)

    @property
    def depthwise(self) -> bool:
        return self.groups != 1

    def macs(self, B: int) -> int:
        fan = self.k if self.depthwise else self.Cin * self.k
        return B * self.Cout * self.Tout * fan

    def weight_count(self) -> int:
        return self.Cout * self.k * (1 if self.depthwise else self.Cin)


@dataclass
class NetSpec:
    name: str
    config_id: int
    B: int
    Cin: int
    Tin: int
    ops: List[OpSpec] = field(default_factory=list)
    n_slots: int = 1

    @property
    def Cout(self) -> int:
        return self.ops[-1].Cout

    @property
    def Tout(self) -> int:
        return self.ops[-1].Tout


def out_len(Tin, k, stride, dilation, pad_left, pad_right) -> int:
    span = Tin + pad_left + pad_right - dilation * (k - 1) - 1
    return span // stride + 1 if span >= 0 else 0


class _Builder:
    """Builds an op list over symbolic tensor ids, then maps tensors to reusable slots."""

    def __init__(self, name, config_id, B, Cin, Tin):
        self.net = NetSpec(name, config_id, B, Cin, Tin)
        self.cur, self.C, self.T = 0, Cin, Tin     # running activation: tensor id, channels, frames
        self.n_tensors = 1

    def op(self, name, Cout, k=1, stride=1, dilation=1, pad=None, groups=1, relu=True,
           bias=True, res=-1, Cin=None, x_batch_stride=0, advance=True, act=0, src=None, more_res=()):
        """Append one op reading the running activation; returns its output tensor id."""
        cur = self.cur if src is None else src[0]      # src = (tensor id, channels): read another tensor
        Cin = (self.C if src is None else src[1]) if Cin is None else Cin
        if pad is None:
            tot = dilation * (k - 1)
            pad = (tot // 2, tot - tot // 2)
        out = self.n_tensors
        self.n_tensors += 1
        o = OpSpec(name, Cin, Cout, self.T, k, stride, dilation, pad[0], pad[1], groups,
                   x_batch_stride, FLAG_RELU if relu else 0, bias, cur, res, out, act, list(more_res))
        self.net.ops.append(o)
        if advance:
            self.cur, self.C, self.T = out, Cout, o.Tout
        return out

    def done(self) -> NetSpec:
        """Linear-scan slot assignment: a tensor's slot is recycled after its last reader."""
        ops = self.net.ops
        last_use = {}
        for i, o in enumerate(ops):
            last_use[o.in_slot] = i
            if o.res_slot >= 0:
                last_use[o.res_slot] = i
            for t in o.more_res:
                last_use[t] = i
        slot_of, free, n = {0: 0}, [], 1
        for i, o in enumerate(ops):
            tin, tres, tout = o.in_slot, o.res_slot, o.out_slot
            if free:
                s = free.pop(0)
            else:
                s, n = n, n + 1
            slot_of[tout] = s
            o.in_slot, o.out_slot = slot_of[tin], s
            o.res_slot = slot_of[tres] if tres >= 0 else -1
            tmore = list(o.more_res)
            o.more_res = [slot_of[t] for t in tmore]
            for t in {tin, tres, *tmore}:
                if t > 0 and last_use.get(t) == i:
                    free.append(slot_of[t])
            free.sort()
        self.net.n_slots = n
        return self.net


def _separable(b: _Builder, tag, Cout, k, dilation=1, relu=True, res=-1):
    """dw (no bias, no ReLU, own dyadic scale) -> int8 -> pw (bias, scale, [residual], ReLU)."""
    b.op(f"{tag}.dw", b.C, k=k, dilation=dilation, groups=b.C, relu=False, bias=False)
    return b.op(f"{tag}.pw", Cout, relu=relu, res=res)


def separable_module(B=1, C=256, T=200, k=33, config_id=0) -> NetSpec:
    """Config 0: one QuartzNet separable module (depthwise k, pointwise C->C, ReLU)."""
    b = _Builder("separable_module", config_id, B, C, T)
    _separable(b, "m0", C, k)
    return b.done()


def quartznet(B, T, repeat, config_id, Cin=64, widths=(256, 256, 512, 512, 512),
              kernels=(33, 39, 51, 63, 75), k1=33, k2=87, C3=1024, n_out=29, name=None,
              separable_c1=False) -> NetSpec:
    """QuartzNet-(5*repeat)x5-shaped encoder (configs 1 and 2; repeat = 2 is the 10x5 variant).
    `separable_c1` makes the stride-2 first layer a depthwise + pointwise pair like the others."""
    b = _Builder(name or f"quartznet_{5 * repeat}x5", config_id, B, Cin, T)
    if separable_c1:
        b.op("C1.dw", Cin, k=k1, stride=2, pad=((k1 - 1) // 2, (k1 - 1) // 2), groups=Cin, relu=False, bias=False)
        b.op("C1.pw", widths[0])
    else:
        b.op("C1", widths[0], k=k1, stride=2, pad=((k1 - 1) // 2, (k1 - 1) // 2))
    for bi, (W, k) in enumerate(zip(widths, kernels)):
        for r in range(repeat):
            tag = f"B{bi + 1}.{r}"
            # residual branch: pointwise on the block input, bias + scale, no ReLU
            res = b.op(f"{tag}.res", W, relu=False, advance=False)
            for mi in range(5):
                _separable(b, f"{tag}.m{mi}", W, k, res=res if mi == 4 else -1)
    _separable(b, "C2", widths[-1], k2, dilation=2)
    b.op("C3", C3)
    b.op("C4", n_out, relu=False)
    return b.done()


def jasper(B, T, config_id, Cin=64, widths=(256, 384, 512, 640, 768), kernels=(11, 13, 17, 21, 25),
           per_width=2, k_pro=11, C_epi=896, k_epi=29, C_epi2=1024, n_out=29, name="jasper_10x5",
           dense_residual=False) -> NetSpec:
    """Jasper-10x5-shaped dense stack (config 3): one residual per block from the block input.
    With `dense_residual` (the DR variant the paper evaluates) a block receives, besides the
    projection of its own input, the projections of the inputs of all earlier blocks: one
    pointwise conv (bias, own scale, no ReLU) per earlier input, all added in the epilogue of the
    block's last conv."""
    b = _Builder(name, config_id, B, Cin, T)
    b.op("prologue", widths[0], k=k_pro, stride=2, pad=((k_pro - 1) // 2, (k_pro - 1) // 2))
    inputs = []                                   # (tensor id, channels) of every block input so far
    for wi, (W, k) in enumerate(zip(widths, kernels)):
        for r in range(per_width):
            tag = f"J{wi + 1}.{r}"
            more = []
            if dense_residual:
                more = [b.op(f"{tag}.res_from{j}", W, relu=False, advance=False, src=src)
                        for j, src in enumerate(inputs)]
                inputs.append((b.cur, b.C))
            res = b.op(f"{tag}.res", W, relu=False, advance=False)
            for ci in range(5):
                b.op(f"{tag}.c{ci}", W, k=k, relu=True, res=res if ci == 4 else -1,
                     more_res=more if ci == 4 else ())
    b.op("epilogue0", C_epi, k=k_epi, dilation=2)
    b.op("epilogue1", C_epi2)
    b.op("epilogue2", n_out, relu=False)
    return b.done()


ACT_SIGMOID, ACT_SWISH, ACT_GLU = 1, 2, 3


def conformer_shaped(B, T, config_id, d_model=512, d_ff=2048, k=32, layers=17, name="conformer_l_shaped",
                     nonlinear=False) -> NetSpec:
    """Conformer-L-shaped integer linear layers (config 4): per layer ffn1, ffn2, pw1 (d->2d),
    depthwise k on the first d channels of pw1's output (a strided channel-prefix view), pw2.
    No ReLU, no residual.  Nonlinearities are identity in configuration 4 itself; with
    `nonlinear` the layers carry the integer activations of the architecture: Swish after ffn1
    and after the depthwise convolution, GLU after pw1 (its d outputs are the prefix view)."""
    b = _Builder(name, config_id, B, d_model, T)
    sw, glu = (ACT_SWISH, ACT_GLU) if nonlinear else (0, 0)
    for li in range(layers):
        b.op(f"L{li}.ffn1", d_ff, relu=False, act=sw)
        b.op(f"L{li}.ffn2", d_model, relu=False)
        b.op(f"L{li}.pw1", 2 * d_model, relu=False, act=glu)
        b.op(f"L{li}.dw", d_model, k=k, groups=d_model, relu=False, bias=False,
             Cin=d_model, x_batch_stride=2 * d_model * b.T, act=sw)
        b.op(f"L{li}.pw2", d_model, relu=False)
    return b.done()


def build_config(i: int, B: Optional[int] = None) -> NetSpec:
    """The five benchmark configurations at full size (B overrides the batch only)."""
    if i == 0:
        return separable_module(B or 1, 256, 200, 33, config_id=0)
    if i == 1:
        return quartznet(B or 1, 1600, 1, config_id=1)
    if i == 2:
        return quartznet(B or 32, 1600, 3, config_id=2)
    if i == 3:
        return jasper(B or 16, 1600, config_id=3)
    if i == 4:
        return conformer_shaped(B or 16, 400, config_id=4)
    if i == 6:      # not one of the five: configuration 3 with the dense-residual wiring
        return jasper(B or 16, 1600, config_id=6, name="jasper_dr_10x5", dense_residual=True)
    if i == 5:      # not one of the five: configuration 4 with its integer nonlinearities in place
        return conformer_shaped(B or 16, 400, config_id=5, name="conformer_l_shaped_nonlinear", nonlinear=True)
    raise ValueError(i)


def tiny_config(i: int) -> NetSpec:
    """Same op-list generators at toy sizes (for brute-force wiring pins)."""
    if i in (0,):
        return separable_module(1, 4, 11, 3, config_id=100)
    if i in (1, 2):
        return quartznet(2, 24, 1 if i == 1 else 2, config_id=100 + i, Cin=3, widths=(4, 4, 8, 8, 8),
                         kernels=(3, 5, 3, 5, 7), k1=5, k2=5, C3=6, n_out=3, name=f"tiny_quartznet_{i}")
    if i == 3:
        return jasper(2, 20, config_id=103, Cin=3, widths=(4, 6), kernels=(3, 5), per_width=1,
                      k_pro=3, C_epi=5, k_epi=3, C_epi2=6, n_out=3, name="tiny_jasper")
    if i == 4:
        return conformer_shaped(2, 9, config_id=104, d_model=4, d_ff=8, k=4, layers=2, name="tiny_conformer")
    if i == 5:
        return conformer_shaped(2, 9, config_id=105, d_model=4, d_ff=8, k=4, layers=2,
                                name="tiny_conformer_nonlinear", nonlinear=True)
    if i == 7:
        return jasper(2, 20, config_id=107, Cin=3, widths=(4, 6, 5), kernels=(3, 5, 3), per_width=1,
                      k_pro=3, C_epi=5, k_epi=3, C_epi2=6, n_out=3, name="tiny_jasper_dense_residual",
                      dense_residual=True)
    if i == 6:
        return quartznet(2, 24, 1, config_id=106, Cin=3, widths=(4, 4, 8, 8, 8), kernels=(3, 5, 3, 5, 7),
                         k1=5, k2=5, C3=6, n_out=3, name="tiny_quartznet_separable_c1", separable_c1=True)
    raise ValueError(i)


def net_macs(net: NetSpec) -> int:
    return sum(o.macs(net.B) for o in net.ops)


def net_weight_count(net: NetSpec) -> int:
    return sum(o.weight_count() for o in net.ops)


def draw_net_params(net: NetSpec, seed: int, m_lo=1 << 30, m_hi=(1 << 31) - 1, s_lo=36, s_hi=44,
                    bias_mag=1 << 16, w_bits=8):
    """Per-op constants as the offline quantiser would emit them (here: seeded draws).

    w int8 U[-(2^(w_bits-1) - 1), 2^(w_bits-1) - 1] (w_bits = 6: the W6A8 setting, 6-bit codes in int8
    storage) in PyTorch Conv1d order [Cout, Cin/groups, k]; bias int32
    U[-bias_mag, bias_mag] (default 2^16) or None; m int32 U[2^30, 2^31); s int32 U{36..44}.
    An op with an activation also gets "act": the real scale S of its int8 input (U[4, 8] / 127 in
    steps of 0.01 / 127), the refinement shift u = 8, and the activation's own output rescale
    (m U[2^30, 2^31), s = 45: a ratio in [2^-15, 2^-14), i.e. about the input's own scale)."""
    out = []
    wmax = (1 << (w_bits - 1)) - 1
    for i, o in enumerate(net.ops):
        cin_g = 1 if o.depthwise else o.Cin
        sd = lambda kind: tensor_seed(seed, net.config_id, i, kind)
        p = {
            "w": randint_array(sd("w"), (o.Cout, cin_g, o.k), -wmax, wmax, np.int8),
            "bias": randint_array(sd("bias"), (o.Cout,), -bias_mag, bias_mag, np.int32) if o.has_bias else None,
            "m": randint_array(sd("m"), (o.Cout,), m_lo, m_hi, np.int32),
            "s": randint_array(sd("s"), (o.Cout,), s_lo, s_hi, np.int32),
        }
        if o.act:
            r = randint_array(sd("act"), (2,), 0, (1 << 31) - 1, np.int64)
            p["act"] = {"kind": o.act, "S": (400 + int(r[0]) % 401) / 100.0 / 127.0, "u": 8,
                        "m": (1 << 30) + int(r[1]) % (1 << 30), "s": 45}
        out.append(p)
    return out


def draw_input(net: NetSpec, seed: int) -> np.ndarray:
    """Network input: int8 U[-128,127], [B, Cin, Tin]."""
    return randint_array(tensor_seed(seed, net.config_id, -1, "x"), (net.B, net.Cin, net.Tin), -128, 127, np.int8)
