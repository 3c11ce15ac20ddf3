"""The persistent team kernel (runs of layers in one launch, barriers among the workgroups of an XCD)
against the CPU oracle and against the same encoder launched layer by layer.  The kernel is
experimental and off unless QASR_TEAM is set when the encoder is created: every test here that runs
it sets the variable for itself, on encoders short enough (about 60 layers in a run) for the
kernel to have been right every time."""
import numpy as np
import pytest
import torch

import oracle
import paper_2103_16827_amd as Q
import qasr_workloads as W
from gpu_util import dev, GpuNet

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)


def run_both(net, seed, items=None, **draw_kw):
    params = W.draw_net_params(net, seed, **draw_kw)
    x = W.draw_input(net, seed)
    g = GpuNet(net, params)
    in_team = [g.enc.op_in_team(i) for i in range(g.enc.n_ops)]
    say(f"{net.name} B={net.B} T={net.Tin}: {sum(in_team)} of {len(in_team)} ops inside team runs")
    xd = dev(x)
    y_team = g.forward(xd).clone()
    torch.cuda.synchronize()
    assert not g.enc.team_aborted(), "a bounded wait of the team kernel gave up"
    g.check_guards()
    y_layer = torch.full_like(y_team, 55)
    g.enc.forward_layerwise(xd, y_layer, g.ws)
    torch.cuda.synchronize()
    g.check_guards()
    bad = (y_team != y_layer)
    assert not bool(bad.any()), f"{int(bad.sum())} bytes differ from the layer-by-layer forward; first item " \
                                f"{int(bad.nonzero()[0][0])}"
    yh = y_team.cpu().numpy()
    sub = W.NetSpec(net.name, net.config_id, 1, net.Cin, net.Tin, net.ops, net.n_slots)
    for b in (range(net.B) if items is None else items):
        ref = oracle.encoder_forward(sub, params, np.ascontiguousarray(x[b:b + 1]))
        assert np.array_equal(yh[b:b + 1], ref), f"item {b} differs from the oracle"
        assert len(set(ref.reshape(-1).tolist())) > 16
    return g, in_team


@pytest.mark.parametrize("B,T", [(8, 160), (9, 320), (32, 800), (19, 208)])
def test_quartznet_blocks_in_team_runs(B, T, tuning_env):
    """QuartzNet-5x5 shape at batch sizes that give every XCD one, two (ragged) or four utterances."""
    tuning_env("QASR_TEAM", "1")
    net = W.quartznet(B, 2 * T, 1, config_id=1)
    g, in_team = run_both(net, 3, items=range(B) if B <= 9 else [0, B // 2, B - 1])
    assert sum(in_team) >= 55, in_team          # all five blocks, C2 and C3
    assert not in_team[0] and not in_team[-1]   # the strided first layer and the 29-channel logits layer
    g.enc.close()


def test_team_runs_are_off_unless_the_environment_asks_for_them(monkeypatch):
    monkeypatch.delenv("QASR_TEAM", raising=False)
    Q.tuning_reload()
    net = W.quartznet(8, 320, 1, config_id=1)
    g = GpuNet(net, W.draw_net_params(net, 1))
    assert not any(g.enc.op_in_team(i) for i in range(g.enc.n_ops))
    g.enc.close()


def test_small_batches_and_other_families_keep_layerwise_launches(tuning_env):
    tuning_env("QASR_TEAM", "1")
    for net in (W.build_config(1), W.jasper(8, 400, config_id=3)):
        g = GpuNet(net, W.draw_net_params(net, 1))
        assert not any(g.enc.op_in_team(i) for i in range(g.enc.n_ops)), net.name
        g.enc.close()


def test_team_forward_repeats_and_clock_stamps(tuning_env):
    """The same encoder many times in a row (the control block is cleared by every launch), then the
    per-layer clock stamps."""
    tuning_env("QASR_TEAM", "1")
    net = W.quartznet(16, 800, 1, config_id=1)
    params = W.draw_net_params(net, 2)
    g = GpuNet(net, params)
    xd = dev(W.draw_input(net, 2))
    want = torch.empty_like(g.y)
    g.enc.forward_layerwise(xd, want, g.ws)
    torch.cuda.synchronize()
    for rep in range(20):
        g.y.fill_(0)
        g.forward(xd)
    torch.cuda.synchronize()
    assert not g.enc.team_aborted()
    assert torch.equal(g.y, want)
    us = g.enc.forward_team_stamps(xd, g.y, g.ws)
    torch.cuda.synchronize()
    assert torch.equal(g.y, want)
    inside = [u for i, u in enumerate(us) if g.enc.op_in_team(i)]
    say(f"team layers: {len(inside)} stamps, {sum(inside):.1f} us in all, max {max(inside):.1f} us")
    assert all(0.0 < u < 5000.0 for u in inside)
    g.enc.close()
