"""qasr_encoder_forward_static (activation slots in the library's static device array) against
qasr_encoder_forward with a caller's workspace: same bytes, on two calls in a row, the second with a
smaller network, and again after the array has been filled with other values."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2103_16827_amd as Q
import qasr_workloads as W
from gpu_util import dev, GpuNet

pytestmark = pytest.mark.gpu


def _both(net, seed):
    params = W.draw_net_params(net, seed)
    x = dev(W.draw_input(net, seed))
    g = GpuNet(net, params)
    assert g.enc.workspace_bytes <= Q.static_workspace_bytes()
    want = g.forward(x).clone()
    g.check_guards()
    got = torch.full_like(want, 33)
    g.enc.forward_static(x, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want), f"{net.name}: {(got != want).sum().item()} bytes differ"
    assert len(set(want.cpu().numpy().reshape(-1).tolist())) > 16
    return g, x, want


def test_static_workspace_forward_matches_on_two_calls_the_second_smaller():
    print("[case] static forward: quartznet 5x5 B=2, then the single separable module", flush=True)
    big = W.quartznet(2, 1600, 1, config_id=1)
    g1, x1, want1 = _both(big, 1)
    small = W.build_config(0)
    g2, x2, want2 = _both(small, 2)              # smaller input, the array still holds the first call's slots
    # and the first network again, after the smaller one
    got = torch.empty_like(want1)
    g1.enc.forward_static(x1, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want1)
    g1.enc.close()
    g2.enc.close()


def test_static_workspace_limit_is_an_error_before_any_launch():
    print("[case] static forward: encoder larger than the array", flush=True)
    net = W.build_config(2)                       # batch 32: needs more than the static array holds
    params = W.draw_net_params(net, 1)
    g = GpuNet(net, params)
    assert g.enc.workspace_bytes > Q.static_workspace_bytes()
    y = torch.full((net.B, net.Cout, net.Tout), 5, dtype=torch.int8, device="cuda")
    with pytest.raises(Q.QasrError) as e:
        g.enc.forward_static(dev(W.draw_input(net, 1)), y)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert bool((y == 5).all())
    g.enc.close()
