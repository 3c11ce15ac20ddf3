"""Helpers shared by the GPU parity tests: marshalling of workload specs to the C ABI."""
import numpy as np
import torch

import paper_2103_16827_amd as Q
from paper_2103_16827_amd.binding import make_desc


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def desc_of(op, B, flags_extra=0):
    return make_desc(B, op.Cin, op.Cout, op.Tin, op.k, op.stride, op.dilation, op.pad_left, op.pad_right,
                     op.groups, op.x_batch_stride, 0, op.flags | flags_extra)


def act_of(a):
    """Workload activation record -> qasr_act (constants through qasr_iexp_init), or None."""
    if not a:
        return None
    return Q.make_act(a["kind"], Q.iexp_init(a["S"], a["u"]), a["m"], a["s"])


GUARD = 4096          # bytes of canary before and after every output and workspace buffer
FILL = 77             # canary / gap value


class Guarded:
    """A device buffer of n int8 elements with GUARD canary bytes on either side."""

    def __init__(self, n, fill=FILL):
        self.n, self.fill = int(n), fill
        self.raw = torch.full((self.n + 2 * GUARD,), fill, dtype=torch.int8, device="cuda")
        self.view = self.raw[GUARD:GUARD + self.n]

    def check(self, what=""):
        lo, hi = self.raw[:GUARD], self.raw[GUARD + self.n:]
        assert bool((lo == self.fill).all()), f"bytes written before the buffer {what}"
        assert bool((hi == self.fill).all()), f"bytes written after the buffer {what}"


def gpu_layer(op, B, p, x, residual=None, packed=False, ybs=0):
    """One op through qasr_conv1d_int8; returns a numpy int8 array [B, Cout, Tout].
    The output sits between canary bands that must come back untouched.  With `ybs` (elements, >=
    Cout*Tout) output and residual operand(s) use that batch stride; the gap bytes between the
    batch items' blocks must come back untouched as well."""
    n_blk = op.Cout * op.Tout
    stride = ybs or n_blk
    assert stride >= n_blk
    d = make_desc(B, op.Cin, op.Cout, op.Tin, op.k, op.stride, op.dilation, op.pad_left, op.pad_right,
                  op.groups, op.x_batch_stride, ybs, op.flags)
    w = dev(p["w"])
    if packed:
        wp = torch.empty(Q.packed_weight_bytes(d), dtype=torch.int8, device="cuda")
        Q.pack_weights(d, w, wp)
        w = wp
        d.flags |= Q.FLAG_W_PACKED
    yg = Guarded(B * stride)
    y = yg.view

    def strided(r):                       # residual operand laid out like the output
        if r is None:
            return None
        full = np.full((B, stride), 19, dtype=np.int8)
        full[:, :n_blk] = np.ascontiguousarray(r).reshape(B, n_blk)
        return dev(full)

    if isinstance(residual, (list, tuple)):
        Q.conv1d_int8_multi(d, dev(x), w, dev(p["bias"]), dev(p["m"]), dev(p["s"]), [strided(r) for r in residual], y)
    else:
        Q.conv1d_int8(d, dev(x), w, dev(p["bias"]), dev(p["m"]), dev(p["s"]), strided(residual), y)
    if p.get("act"):
        a = p["act"]
        Q.act_int8(act_of(a), y, B, op.Cout // 2 if a["kind"] == Q.ACT_GLU else op.Cout, op.Tout, y,
                   stride, stride)
    torch.cuda.synchronize()
    yg.check(f"({op.name})")
    out = y.view(B, stride).cpu().numpy()
    assert (out[:, n_blk:] == FILL).all(), f"bytes written between the batch items' blocks ({op.name})"
    return np.ascontiguousarray(out[:, :n_blk]).reshape(B, op.Cout, op.Tout)


class GpuNet:
    """A workload NetSpec + drawn parameters resident on the GPU behind a qasr encoder.  Output and
    workspace sit between canary bands (`check_guards`)."""

    def __init__(self, net, params):
        self.net = net
        self.params = params
        self.dev_params = [{k: dev(v) for k, v in p.items() if k != "act"} for p in params]
        ops = [(desc_of(o, net.B), dp["w"], dp["bias"], dp["m"], dp["s"], o.in_slot, o.res_slot, o.out_slot,
                act_of(p.get("act")), list(getattr(o, "more_res", [])))
               for o, dp, p in zip(net.ops, self.dev_params, params)]
        self.enc = Q.Encoder(ops, net.n_slots)
        # (the workspace must be 256-byte aligned: the canary band before it is a multiple of that)
        self.wsg = Guarded(max(self.enc.workspace_bytes, 256))
        self.ws = self.wsg.view
        assert self.ws.data_ptr() % 256 == 0
        self.yg = Guarded(net.B * net.Cout * net.Tout)
        self.y = self.yg.view.view(net.B, net.Cout, net.Tout)

    def forward(self, x_dev):
        self.enc.forward(x_dev, self.y, self.ws)
        return self.y

    def check_guards(self):
        torch.cuda.synchronize()
        self.yg.check(f"(output of {self.net.name})")
        self.wsg.check(f"(workspace of {self.net.name})")

    def kernels(self):
        return [self.enc.op_kernel(i) for i in range(self.enc.n_ops)]
