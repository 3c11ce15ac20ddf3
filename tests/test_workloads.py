"""Pins for the seeded input generator and the network shape tables (CPU only)."""
import numpy as np
import pytest

import qasr_workloads as W
from qasr_workloads.rng import splitmix64_scalar, splitmix64_stream, randint_array, tensor_seed


def test_splitmix64_matches_public_test_vector(golden):
    ref = [int(r[0]) for r in golden("splitmix64_seed1234567.txt")]
    assert splitmix64_scalar(1234567, 5) == ref
    assert [int(v) for v in splitmix64_stream(1234567, 5)] == ref


def test_vectorised_stream_equals_scalar_stream():
    for seed in (0, 1, 2**63 + 12345, 2**64 - 1):
        a = [int(v) for v in splitmix64_stream(seed, 257)]
        assert a == splitmix64_scalar(seed, 257)
        b = [int(v) for v in splitmix64_stream(seed, 50, offset=207)]
        assert b == a[207:]


def test_randint_is_lo_plus_mod_span_and_chunking_is_invisible():
    seed = tensor_seed(1, 0, 0, "w")
    ref = [(-127 + (u % 255)) for u in splitmix64_scalar(seed, 1000)]
    got = randint_array(seed, (10, 100), -127, 127, np.int8)
    assert got.dtype == np.int8 and got.reshape(-1).tolist() == ref
    m = randint_array(seed, (64,), 1 << 30, (1 << 31) - 1, np.int32)
    assert m.min() >= 1 << 30 and m.max() < 1 << 31
    s = randint_array(seed, (4096,), 36, 44, np.int32)
    assert set(s.tolist()) == set(range(36, 45))


def test_tensor_seeds_are_distinct():
    seen = {tensor_seed(b, c, o, k) for b in (1, 2, 3) for c in range(5) for o in range(-1, 40)
            for k in ("x", "w", "bias", "m", "s")}
    assert len(seen) == 3 * 5 * 41 * 5


@pytest.mark.parametrize("cfg,n_ops,n_dw,macs_g,weights_m,out_shape", [
    (0, 2, 1, 0.0148, 0.074, (1, 256, 200)),
    (1, 60, 26, 5.77, 7.21, (1, 29, 800)),
    (2, 170, 76, 495.9, 19.37, (32, 29, 800)),
    (3, 64, 0, 4124.0, 322.2, (16, 29, 800)),
    (4, 85, 17, 315.5, 49.3, (16, 512, 400)),
])
def test_config_shapes(cfg, n_ops, n_dw, macs_g, weights_m, out_shape):
    net = W.build_config(cfg)
    assert len(net.ops) == n_ops
    assert sum(o.depthwise for o in net.ops) == n_dw
    assert W.net_macs(net) / 1e9 == pytest.approx(macs_g, rel=2e-3)
    assert W.net_weight_count(net) / 1e6 == pytest.approx(weights_m, rel=2e-3)
    assert (net.B, net.Cout, net.Tout) == out_shape
    # int32 accumulators cannot overflow at these shapes: fan_in * 128 * 127 + 2^16 < 2^31
    for o in net.ops:
        fan = o.k if o.depthwise else o.Cin * o.k
        assert fan * 128 * 127 + (1 << 16) < (1 << 31)


def test_networks_agree_with_paper_table1_size_and_bops(golden):
    tab = {r[0]: (float(r[1]), float(r[2])) for r in golden("table1_size_bops.txt")}
    # 10 s at 16 kHz with a 10 ms hop = 1000 feature frames, batch 1
    q = W.quartznet(1, 1000, 3, config_id=2)
    j = W.jasper(1, 1000, config_id=3)
    for net, key in ((q, "quartznet"), (j, "jasper")):
        size_mb, bops_t = tab[key]
        assert W.net_weight_count(net) / 1e6 == pytest.approx(size_mb, rel=0.10)
        assert W.net_macs(net) * 64 / 1e12 == pytest.approx(bops_t, rel=0.10)


def test_variants_of_the_same_families():
    """QuartzNet-10x5 (the medium model of Sec. 3.2), the separable first layer, 6-bit weights."""
    q10 = W.quartznet(1, 1600, 2, config_id=6)
    assert q10.name == "quartznet_10x5" and len(q10.ops) == 1 + 10 * 11 + 4
    assert sum(o.depthwise for o in q10.ops) == 51 and (q10.Cout, q10.Tout) == (29, 800)
    q5, q15 = W.build_config(1), W.quartznet(1, 1600, 3, config_id=2)
    # weights grow by one repeat of the five block types per step
    assert W.net_weight_count(q15) - W.net_weight_count(q10) == W.net_weight_count(q10) - W.net_weight_count(q5)
    # a separable first layer brings the 15x5 shape to within 2.5 % of the paper's model size
    qs = W.quartznet(1, 1000, 3, config_id=2, separable_c1=True)
    assert [o.name for o in qs.ops[:3]] == ["C1.dw", "C1.pw", "B1.0.res"]
    assert (qs.ops[0].groups, qs.ops[0].stride, qs.ops[0].Tout, qs.ops[1].Cin, qs.ops[1].Cout) == (64, 2, 500, 64, 256)
    assert W.net_weight_count(qs) / 1e6 == pytest.approx(18.45, rel=0.025)
    # W6A8: 6-bit codes [-31, 31] in int8 storage, everything else unchanged
    p8, p6 = W.draw_net_params(q5, 1), W.draw_net_params(q5, 1, w_bits=6)
    for a, b in zip(p8, p6):
        assert b["w"].dtype == np.int8 and b["w"].min() >= -31 and b["w"].max() <= 31
        assert np.array_equal(a["m"], b["m"]) and np.array_equal(a["s"], b["s"])
    big = p6[2]["w"]
    assert big.min() == -31 and big.max() == 31 and len(set(big.reshape(-1).tolist())) == 63


def test_dense_residual_jasper_wiring():
    net = W.jasper(1, 1000, config_id=3, dense_residual=True)
    assert len(net.ops) == 64 + 45                                   # one more projection per earlier block input
    last = [o for o in net.ops if o.name.endswith(".c4")]
    assert [len(o.more_res) for o in last] == list(range(10))        # block b adds b earlier inputs
    proj = [o for o in net.ops if ".res_from" in o.name]
    assert all(o.k == 1 and not (o.flags & 1) and o.has_bias for o in proj)
    j5 = [o for o in proj if o.name.startswith("J5.1.")]
    assert [o.Cin for o in j5] == [256, 256, 256, 384, 384, 512, 512, 640, 640] and all(o.Cout == 768 for o in j5)
    # BOPs of the dense-residual shape are within 1 % of the paper's Table 1 (10.7 T)
    assert W.net_macs(net) * 64 / 1e12 == pytest.approx(10.7, rel=0.01)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 7])
def test_slot_wiring_is_hazard_free(cfg):
    """No op writes a slot it reads, slot 0 is never written, and every read slot holds the
    tensor the builder meant (replay with symbolic tensor ids)."""
    nets = (W.jasper(2, 400, config_id=3, dense_residual=True), W.tiny_config(7)) if cfg == 7 else \
        (W.build_config(cfg), W.tiny_config(cfg))
    for net in nets:
        holds = {0: ("x", net.Cin, net.Tin)}
        for i, o in enumerate(net.ops):
            assert o.out_slot != 0 and o.out_slot != o.in_slot and o.out_slot != o.res_slot
            assert o.out_slot not in o.more_res and len(set(o.more_res + [o.res_slot])) == len(o.more_res) + 1
            for j, r in enumerate(o.more_res):
                assert holds[r][1:] == (o.Cout, o.Tout) and holds[r][0].endswith(f".res_from{j}")
            assert o.in_slot in holds
            _, c_in, t_in = holds[o.in_slot]
            assert t_in == o.Tin and c_in >= o.Cin
            if o.x_batch_stride:
                assert o.x_batch_stride == c_in * t_in
            else:
                assert c_in == o.Cin
            if o.res_slot >= 0:
                assert holds[o.res_slot][1:] == (o.Cout, o.Tout)
                assert holds[o.res_slot][0].endswith(".res")
            holds[o.out_slot] = (o.name, o.Cout, o.Tout)
            assert max(o.in_slot, o.res_slot, o.out_slot) < net.n_slots


def test_quartznet_block_structure():
    net = W.build_config(1)
    names = [o.name for o in net.ops]
    assert names[0] == "C1" and names[-3:] == ["C2.pw", "C3", "C4"]
    blk = net.ops[1:12]
    assert blk[0].name == "B1.0.res" and not blk[0].flags & 1
    assert [o.depthwise for o in blk[1:]] == [True, False] * 5
    assert all(o.res_slot < 0 for o in blk[:-1]) and blk[-1].res_slot == blk[0].out_slot
    assert all(not o.has_bias and not (o.flags & 1) for o in blk[1::2])     # depthwise: no bias, no ReLU
    assert all(o.has_bias and (o.flags & 1) for o in blk[2::2])            # pointwise: bias + ReLU
    b3 = [o for o in net.ops if o.name.startswith("B3.0")]
    assert (b3[0].Cin, b3[0].Cout) == (256, 512) and (b3[1].Cin, b3[1].k) == (256, 51)
    assert (b3[2].Cin, b3[2].Cout) == (256, 512)
    c2 = net.ops[-4]
    assert (c2.k, c2.dilation, c2.pad_left, c2.pad_right, c2.Tout) == (87, 2, 86, 86, 800)
    assert not net.ops[-1].flags & 1


def test_conformer_even_kernel_padding_and_view():
    net = W.build_config(4)
    dw = net.ops[3]
    assert (dw.k, dw.pad_left, dw.pad_right, dw.Tout) == (32, 15, 16, 400)
    assert dw.Cin == 512 and dw.x_batch_stride == 1024 * 400


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more ends with a message, before any GPU work."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
