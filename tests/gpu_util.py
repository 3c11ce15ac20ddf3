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


def gpu_layer(op, B, p, x, residual=None, packed=False):
    """One op through qasr_conv1d_int8; returns a numpy int8 array."""
    d = desc_of(op, B)
    w = dev(p["w"])
    if packed:
        wp = torch.empty(Q.packed_weight_bytes(d), dtype=torch.int8, device="cuda")
        Q.pack_weights(d, w, wp)
        w = wp
        d.flags |= Q.FLAG_W_PACKED
    y = torch.full((B, op.Cout, op.Tout), 77, dtype=torch.int8, device="cuda")
    if isinstance(residual, (list, tuple)):
        Q.conv1d_int8_multi(d, dev(x), w, dev(p["bias"]), dev(p["m"]), dev(p["s"]), [dev(r) for r in residual], y)
    else:
        Q.conv1d_int8(d, dev(x), w, dev(p["bias"]), dev(p["m"]), dev(p["s"]), dev(residual), y)
    if p.get("act"):
        a = p["act"]
        Q.act_int8(act_of(a), y, B, op.Cout // 2 if a["kind"] == Q.ACT_GLU else op.Cout, op.Tout, y,
                   op.Cout * op.Tout, op.Cout * op.Tout)
    torch.cuda.synchronize()
    return y.cpu().numpy()


class GpuNet:
    """A workload NetSpec + drawn parameters resident on the GPU behind a qasr encoder."""

    def __init__(self, net, params):
        self.net = net
        self.params = params
        self.dev_params = [{k: dev(v) for k, v in p.items() if k != "act"} for p in params]
        ops = [(desc_of(o, net.B), dp["w"], dp["bias"], dp["m"], dp["s"], o.in_slot, o.res_slot, o.out_slot,
                act_of(p.get("act")), list(getattr(o, "more_res", [])))
               for o, dp, p in zip(net.ops, self.dev_params, params)]
        self.enc = Q.Encoder(ops, net.n_slots)
        self.ws = torch.empty(max(self.enc.workspace_bytes, 256), dtype=torch.int8, device="cuda")
        self.y = torch.empty((net.B, net.Cout, net.Tout), dtype=torch.int8, device="cuda")

    def forward(self, x_dev):
        self.enc.forward(x_dev, self.y, self.ws)
        return self.y

    def kernels(self):
        return [self.enc.op_kernel(i) for i in range(self.enc.n_ops)]
