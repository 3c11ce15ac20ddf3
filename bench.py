#!/usr/bin/env python3
"""Benchmark of the INT8 encoder hot path on one MI355X.

A "step" is one forward of the QuartzNet-15x5-shaped encoder at batch 32, T=1600 input frames
(benchmark config 2), on seeded synthetic int8 inputs and random int8 weights already resident
in HBM: one launch of the forward captured as a HIP graph (qasr_encoder_graph_launch), or with
--eager the 170 separate kernel launches of qasr_encoder_forward.  Prints ONE JSON line:

  value       input frames per second (B*T_in*steps / wall time of the timed steps)
  roofline    for the kernel family with the largest share of device time, measured live with
              HIP events around every op (a separate, untimed-for-`value` pass)
  stages      spec view: depthwise stages against HBM peak, pointwise stages against the
              int8 MFMA peak (algorithmic bytes / MACs over summed per-op device time)
  step_ms     mean / median / min / max of the timed steps, each bracketed by HIP events
  ceilings    what this chip sustained in this process: a streaming int8 copy and a register-resident
              int8 matrix-core loop; every fraction is given against the datasheet and against these
  stages_cold the per-stage figures again with nothing left in the caches by the previous pass
              (the passes rotate through buffer sets of more than 512 MB in all)
  cpu_baseline the CPU oracle timed on a bounded sample (batch items one at a time, about ten
              seconds of them) on the host cores; every item is also compared with the GPU output
  cpu_baseline_1thread  the same oracle held to one thread, on configs[0] and configs[1]
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0        # MI355X dense int8 MFMA, published (5.0 POP/s)


def op_algorithmic(op, B):
    """Algorithmic HBM bytes and MACs of one op: input + output (+ residual) int8 tensors,
    weights and per-channel constants once."""
    n_in = B * op.Cin * op.Tin
    n_out = B * op.Cout * op.Tout
    w = op.weight_count()
    consts = op.Cout * (8 + (4 if op.has_bias else 0))
    byts = n_in + n_out + (n_out if op.res_slot >= 0 else 0) + w + consts
    return byts, op.macs(B)


def measured_traffic(kernel, config):
    """HBM bytes per launch of `kernel` on this configuration as the hardware counters saw them
    (FETCH_SIZE + WRITE_SIZE, calibrated against a plain copy of known size): read from the committed
    counter summary profiles/<kernel>_config<N>_hbm_traffic.txt, whose header gives the commands
    that produced it; None when there is no such summary."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_config{config}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def oracle_child(config, max_seconds):
    """Run in a child process (see cpu_1thread): the oracle on one batch item of a configuration,
    repeated until max_seconds have gone; prints frames/s and the thread count as JSON."""
    import numpy as np
    import oracle
    import qasr_workloads as W
    net = W.build_config(config, 1)
    params = W.draw_net_params(net, 1)
    x = W.draw_input(net, 1)
    n, dt = 0, 0.0
    while n < 1 or (dt < max_seconds and n < 200):
        t0 = time.perf_counter()
        oracle.encoder_forward(net, params, x)
        dt += time.perf_counter() - t0
        n += 1
    print(json.dumps({"value": n * net.Tin / dt, "unit": "frames/s", "cores": oracle.num_threads(), "kind": "oracle",
                      "sample": f"configs[{config}] one batch item, {n} forwards ({n * W.net_macs(net) / 1e9:.2f} GMAC) "
                                f"in {dt:.2f} s"}))


def cpu_1thread(config, max_seconds):
    """The oracle as it stands, held to one thread by OMP_NUM_THREADS in a child process that never
    touches the GPU."""
    env = dict(os.environ, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, os.path.abspath(__file__), "--oracle-child", str(config),
                        "--oracle-child-seconds", str(max_seconds)], env=env, capture_output=True, text=True, timeout=300)
    if r.returncode != 0:
        return {"error": r.stderr.strip()[-300:]}
    return json.loads(r.stdout.strip().splitlines()[-1])


def measured_mfma_busy(kernel, config):
    """Fraction of the kernels' duration in which the matrix pipes were busy, by the hardware counters
    (profiles/<kernel>_config<N>_mfma_busy.txt, whose header gives the commands); None without one."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_config{config}_mfma_busy.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(f"mfma_busy_{kernel}:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 0..4 (default 2); 5 = configuration 4 with its integer activations, 6 = configuration 3 with dense residuals")
    ap.add_argument("--batch", type=int, default=0, help="override the configuration's batch size (e.g. 1: single-utterance latency)")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time separate kernel launches instead of the HIP graph")
    ap.add_argument("--profile-passes", type=int, default=5, help="per-op timed passes for the roofline")
    ap.add_argument("--softmax", default="", metavar="ROWS,LEN",
                    help="also run 12 qasr_softmax_int32 calls on seeded int32 logits of this shape (for profiler runs)")
    ap.add_argument("--observer-mib", type=int, default=0,
                    help="also run 12 qasr_observe_minmax calls on this many MiB of float32 values (for profiler runs)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the steps, run one plain elementwise int8 kernel that reads and writes this many MiB "
                         "(the known-size dispatch that calibrates the HBM byte counters of a --pmc run)")
    ap.add_argument("--cold-mib", type=int, default=600,
                    help="total size of the buffer sets the cold per-stage passes rotate through (0: skip them)")
    ap.add_argument("--oracle-child", type=int, default=-1, help=argparse.SUPPRESS)
    ap.add_argument("--oracle-child-seconds", type=float, default=4.0, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.oracle_child >= 0:
        oracle_child(args.oracle_child, args.oracle_child_seconds)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (batch sharding across GPUs needs no kernel work "
              "and is not part of it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    # the child processes of the one-thread oracle figures start before this process touches the GPU
    cpu_1t = None
    if not args.no_cpu_baseline:
        cpu_1t = {"configs[0]": cpu_1thread(0, 2.0), "configs[1]": cpu_1thread(1, 4.0)}

    import numpy as np
    import torch
    import paper_2103_16827_amd as Q
    from paper_2103_16827_amd.binding import make_desc
    import qasr_workloads as W

    torch.cuda.set_device(0)
    net = W.build_config(args.config, args.batch or None)
    workload_label = {5: "configs[4] with integer activations",
                      6: "configs[3] with dense residuals"}.get(args.config, f"configs[{args.config}]")
    params = W.draw_net_params(net, args.seed)
    x_host = W.draw_input(net, args.seed)

    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    dparams = [{k: dev(v) for k, v in p.items() if k != "act"} for p in params]
    ops = [(make_desc(net.B, o.Cin, o.Cout, o.Tin, o.k, o.stride, o.dilation, o.pad_left, o.pad_right,
                      o.groups, o.x_batch_stride, 0, o.flags), d["w"], d["bias"], d["m"], d["s"],
            o.in_slot, o.res_slot, o.out_slot,
            Q.make_act(p["act"]["kind"], Q.iexp_init(p["act"]["S"], p["act"]["u"]), p["act"]["m"], p["act"]["s"])
            if "act" in p else None, list(o.more_res)) for o, d, p in zip(net.ops, dparams, params)]
    enc = Q.Encoder(ops, net.n_slots)
    ws = torch.empty(max(enc.workspace_bytes, 256), dtype=torch.int8, device="cuda")
    y = torch.empty((net.B, net.Cout, net.Tout), dtype=torch.int8, device="cuda")
    x = dev(x_host)
    torch.cuda.synchronize()

    # The timed step: one launch of the forward captured as a HIP graph (qasr_encoder_graph_*),
    # unless --eager asks for qasr_encoder_forward's n_ops separate launches.
    graph = None if args.eager else enc.graph(x, y, ws)
    step = (lambda: enc.forward(x, y, ws)) if args.eager else graph.launch

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    ms_per_step, ms_per_step_events = timed(step, args.warmup, args.steps)

    # the same steps once more, each between two events of its own: spread of the step time
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)])
    step_ms = {"mean": float(per.mean()), "median": float(np.median(per)), "min": float(per.min()),
               "max": float(per.max()), "how": "one HIP event pair per step, a pass of its own after the timed one"}
    del evs

    # ---- ceilings measured here: streaming copy (read + write) and register-resident int8 MFMA loop
    def best_ms(fn, reps):
        out = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            out.append(a.elapsed_time(b))
        return float(np.median(out)), float(min(out))
    cp_bytes = 1 << 30
    cp_a = torch.zeros(cp_bytes, dtype=torch.int8, device="cuda")
    cp_b = torch.empty_like(cp_a)
    Q.probe_copy(cp_a, cp_b)
    copy_med, copy_min = best_ms(lambda: Q.probe_copy(cp_a, cp_b), 7)
    del cp_a, cp_b
    mf_out = torch.zeros(Q.probe_mfma_outputs(), dtype=torch.int32, device="cuda")
    mf_iters = 20000
    mf_ops = Q.probe_mfma_i8(mf_iters, mf_out)
    mf_med, mf_min = best_ms(lambda: Q.probe_mfma_i8(mf_iters, mf_out), 5)
    ceilings = {
        "hbm_copy_GBs": 2 * cp_bytes / (copy_med * 1e-3) / 1e9, "hbm_copy_GBs_best": 2 * cp_bytes / (copy_min * 1e-3) / 1e9,
        "hbm_copy_what": "qasr_probe_copy, 1 GiB read + 1 GiB written per launch, median (and best) of 7",
        "int8_mfma_TOPs": mf_ops / (mf_med * 1e-3) / 1e12, "int8_mfma_TOPs_best": mf_ops / (mf_min * 1e-3) / 1e12,
        "int8_mfma_what": "qasr_probe_mfma_i8, v_mfma_i32_16x16x64_i8 from registers, 8 waves per SIMD, median (and best) of 5",
        "datasheet": {"hbm_GBs": HBM_PEAK_GBS, "int8_mfma_TOPs": INT8_PEAK_TOPS}}
    del mf_out
    torch.cuda.empty_cache()
    # the other launch mode, for comparison (not the reported value)
    other_ms = None if args.eager else timed(lambda: enc.forward(x, y, ws), 3, max(5, args.steps // 5))[0]
    # The launch floor of this op list: a graph of as many dependent one-element kernels as the
    # forward has ops (nothing to compute or move), replayed the same way.  What the step costs
    # beyond it is what the layers' own work costs.
    floor_ms = None
    if not args.eager:
        one_q = torch.zeros(1, dtype=torch.int8, device="cuda")
        one_x = torch.zeros(1, dtype=torch.float32, device="cuda")
        n_launch = enc.n_ops + sum(1 for p in params if "act" in p)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            Q.dequantize(one_q, 1.0, one_x)
            side.synchronize()
            tiny = torch.cuda.CUDAGraph()
            with torch.cuda.graph(tiny, stream=side):
                for _ in range(n_launch):
                    Q.dequantize(one_q, 1.0, one_x)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        floor_ms = timed(tiny.replay, 3, args.steps)[0]
        del tiny
    frames = net.B * net.Tin
    value = frames / (ms_per_step * 1e-3)

    if args.softmax:
        # a side measurement for profiler runs: the integer softmax on attention-shaped logits
        rows_sm, len_sm = (int(v) for v in args.softmax.split(","))
        from qasr_workloads.rng import randint_array
        lg = torch.from_numpy(randint_array(args.seed, (rows_sm, len_sm), -600, 600, np.int32)).cuda()
        pr = torch.empty((rows_sm, len_sm), dtype=torch.int8, device="cuda")
        e_sm = Q.iexp_init(0.01, 2)
        for _ in range(12):
            Q.softmax_int32(e_sm, lg, pr)
        torch.cuda.synchronize()
        del lg, pr

    if args.observer_mib > 0:
        # a side measurement for profiler runs: the min/max observer on float32 activations
        act = torch.rand((args.observer_mib << 20) // 4, dtype=torch.float32, device="cuda")
        mm = torch.tensor([float("inf"), float("-inf")], dtype=torch.float32, device="cuda")
        for _ in range(12):
            Q.observe_minmax(act, mm)
        torch.cuda.synchronize()
        del act, mm

    if args.calib_copy_mib > 0:
        a = torch.zeros(args.calib_copy_mib << 20, dtype=torch.int8, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.bitwise_not(a, out=b)
        torch.cuda.synchronize()
        del a, b

    # ---- per-op device time (HIP events on the launch stream, inside the library)
    kernels = [enc.op_kernel(i) for i in range(enc.n_ops)]
    acc_ms = np.zeros(enc.n_ops)
    for _ in range(max(1, args.profile_passes)):
        acc_ms += np.array(enc.forward_timed(x, y, ws))
    op_ms = acc_ms / max(1, args.profile_passes)

    fam = {}
    for i, (o, k) in enumerate(zip(net.ops, kernels)):
        byts, macs = op_algorithmic(o, net.B)
        f = fam.setdefault(k, {"ms": 0.0, "bytes": 0, "macs": 0, "launches": 0})
        f["ms"] += op_ms[i]; f["bytes"] += byts; f["macs"] += macs; f["launches"] += 1
    dom = max(fam, key=lambda k: fam[k]["ms"])
    d = fam[dom]
    avg_ms = d["ms"] / d["launches"]
    if dom.startswith("dw_") or dom == "conv_generic":
        achieved = d["bytes"] / d["launches"] / (avg_ms * 1e-3) / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None}
    else:
        achieved = 2.0 * d["macs"] / d["launches"] / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                    "frac": achieved / INT8_PEAK_TOPS, "traffic": None}
    roofline["frac_of_measured_ceiling"] = achieved / (ceilings["hbm_copy_GBs"] if roofline["bound"] == "hbm"
                                                       else ceilings["int8_mfma_TOPs"])
    roofline["traffic"] = measured_traffic(dom, args.config)
    if roofline["bound"] == "mfma":
        roofline["mfma_busy_by_counters"] = measured_mfma_busy(dom, args.config)
    roofline["avg_launch_us"] = avg_ms * 1e3
    roofline["launches_per_step"] = d["launches"]
    roofline["share_of_device_time"] = d["ms"] / float(op_ms.sum())

    def stage(sel, t_ms):
        idx = [i for i, o in enumerate(net.ops) if sel(o)]
        if not idx:
            return None
        ms = float(t_ms[idx].sum())
        byts = sum(op_algorithmic(net.ops[i], net.B)[0] for i in idx)
        macs = sum(op_algorithmic(net.ops[i], net.B)[1] for i in idx)
        gbs, tops = byts / (ms * 1e-3) / 1e9, 2 * macs / (ms * 1e-3) / 1e12
        return {"ops": len(idx), "ms": ms, "GB/s": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
                "hbm_frac_of_measured_copy": gbs / ceilings["hbm_copy_GBs"],
                "TOP/s": tops, "mfma_frac": tops / INT8_PEAK_TOPS,
                "mfma_frac_of_measured_loop": tops / ceilings["int8_mfma_TOPs"]}

    def stage_table(t_ms):
        return {"depthwise": stage(lambda o: o.depthwise, t_ms),
                "pointwise": stage(lambda o: not o.depthwise and o.k == 1, t_ms),
                "dense": stage(lambda o: not o.depthwise and o.k > 1, t_ms),
                "device_ms_sum": float(t_ms.sum())}
    stages = stage_table(op_ms)
    stages["ms_per_step_events"] = ms_per_step_events

    # ---- the same per-op times with cold caches: the passes rotate through enough (x, workspace, y)
    # sets that a set, and the weights, were pushed out of L2 and the memory-side cache by more than
    # 512 MB of other traffic before they are touched again; within a pass a layer still finds the
    # previous layer's output where the pipeline leaves it
    stages_cold = None
    if args.cold_mib > 0:
        set_bytes = ws.numel() + x.numel() + y.numel()
        n_sets = max(2, -(-(args.cold_mib << 20) // set_bytes))
        sets = [(x.clone(), torch.empty_like(ws), torch.empty_like(y)) for _ in range(n_sets)]
        for xs_, ws_, ys_ in sets:                       # one untimed pass over every set
            enc.forward(xs_, ys_, ws_)
        torch.cuda.synchronize()
        acc_cold = np.zeros(enc.n_ops)
        for xs_, ws_, ys_ in sets:
            acc_cold += np.array(enc.forward_timed(xs_, ys_, ws_))
        same = all(bool(torch.equal(ys_, y)) for _, _, ys_ in sets)
        stages_cold = stage_table(acc_cold / n_sets)
        stages_cold["buffer_sets"] = n_sets
        stages_cold["bytes_rotated"] = n_sets * set_bytes
        stages_cold["outputs_equal_to_the_timed_steps"] = same
        del sets
        torch.cuda.empty_cache()

    # ---- the oracle on the host cores, on one batch item of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sub = W.NetSpec(net.name, net.config_id, 1, net.Cin, net.Tin, net.ops, net.n_slots)
        y_host = y.cpu().numpy()
        done, dt, ok = 0, 0.0, True
        while done < net.B and dt < 10.0:           # batch items one by one, about ten seconds of them
            xs = np.ascontiguousarray(x_host[done:done + 1])
            t0 = time.perf_counter()
            ref = oracle.encoder_forward(sub, params, xs)
            dt += time.perf_counter() - t0
            ok = ok and bool(np.array_equal(ref, y_host[done:done + 1]))
            done += 1
        cpu = {"value": done * net.Tin / dt, "unit": "frames/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"batch items 0..{done - 1} of the same workload, one at a time ({done * net.Tin} frames, "
                         f"{done * W.net_macs(sub) / 1e9:.1f} GMAC) in {dt:.2f} s",
               "gpu_output_matches": ok}

    total_macs = W.net_macs(net)
    out = {
        "metric": "INT8 encoder frames/sec", "value": value, "unit": "frames/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "step_ms": step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"{workload_label} {net.name} B={net.B} T_in={net.Tin} ({len(net.ops)} ops)",
                   "seed": args.seed, "parallelism": "single GPU",
                   "launch": "separate kernel launches" if args.eager else "HIP graph replay (one launch per step)"},
        "ms_per_step_separate_launches": other_ms,
        "launch_floor": None if floor_ms is None else {
            "ms_per_step": floor_ms, "kernels": n_launch,
            "what": "graph replay of that many dependent one-element kernels"},
        "int8_TOPS_useful": 2 * total_macs / (ms_per_step * 1e-3) / 1e12,
        "int8_TOPS_frac_of_peak": 2 * total_macs / (ms_per_step * 1e-3) / 1e12 / INT8_PEAK_TOPS,
        "int8_TOPS_frac_of_measured_loop": 2 * total_macs / (ms_per_step * 1e-3) / 1e12 / ceilings["int8_mfma_TOPs"],
        "roofline": roofline, "ceilings": ceilings, "stages": stages, "stages_cold": stages_cold,
        "cpu_baseline": cpu, "cpu_baseline_1thread": cpu_1t,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
