#!/usr/bin/env python3
"""Benchmark of the Rudra parameter-server update path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one applyUpdate of the 72M-parameter 1-softsync workload (C4: lambda = 18 learners, c = 18
gradients per update, momentum 0.9, staleness-modulated rate): 18 pushGradient calls through the C ABI
(staleness, vector clock, rate on the host) and the fused sumGradients+applyUpdate kernel they trigger.
Gradients are synthetic (seeded; 64 distinct 288 MB vectors pre-generated in HBM and cycled, far beyond
the 256 MB Infinity Cache) and already resident when the timed region starts; the arrival order is the
workload's seeded Exp(1) trace.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "PS applyUpdates/sec and absorbed gradient GB/s (% HBM peak), 72M fp32 params"
HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, vendor figure

# HBM bytes per applyUpdate launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE), each scaled by
# the same counter's reading for a plain copy of known size (factors 1.99980 and 1.0); figures and commands in
# profiles/apply_update_kernel_C4_C5_72M_hbm_traffic.md.  A measured constant, not recomputed at run time.
MEASURED_TRAFFIC_BYTES = {"C4": 6.3355e9, "C5": 1.43995e9}
MEASURED_TRAFFIC_BYTES_BATCH8 = {"C5": 3.4558e9}   # same files: C5 with 8 messages per call


def algorithmic_bytes_per_update(w) -> int:
    """Each of the c gradients read once, theta read+written once, v read+written once when there is momentum."""
    second_state = w.momentum != 0 or w.optimizer == "adagrad"      # velocity, or AdaGrad's accumulator
    return w.n_params * (4 * w.c + 8 + (8 if second_state else 0))


def run_gpu(w, steps, warmup, ring=64, flags=0, batch=1, **launch):
    """Replays (warmup+steps)*c pushes of the workload's arrival trace; returns timings of the last `steps` updates.
    batch > 1: the messages are handed over `batch` at a time (rudra_ps_push_batch; a learner pulls after the call
    that held its push), so consecutive updates share a launch."""
    import torch
    from synth.learners import HipServer

    c = w.c
    learner, step = w.arrival_trace((warmup + steps) * c)
    hip = HipServer(w, flags=flags, pregenerated=max(ring, c + 1), **launch)
    ps, bufs = hip.ps, [b.data_ptr() for b in hip.ring]
    nbuf = len(bufs)
    learner_ts = [0] * w.n_learners
    hard = w.protocol == "hardsync"
    learner = [int(x) for x in learner]

    def run_range(lo, hi):
        nonlocal learner_ts
        push = ps.push_gradient
        for i in range(lo, hi):
            l = learner[i]
            rc, res = push(bufs[i % nbuf], learner_ts[l], l)
            if rc != 0:
                raise RuntimeError(f"push {i} rejected: {rc}")
            if hard and res.applied:
                learner_ts = [res.ts_after] * w.n_learners
            else:
                learner_ts[l] = res.ts_after

    def run_range_batched(lo, hi):
        for i in range(lo, hi, batch):
            m = min(batch, hi - i)
            ls = learner[i:i + m]
            # hardsync: a gradient must carry the timestamp current at its arrival = the number of completed rounds
            ts = [(i + j) // c for j in range(m)] if hard else [learner_ts[l] for l in ls]
            rc, handled, res = ps.push_batch([bufs[(i + j) % nbuf] for j in range(m)], ts, ls)
            if rc != 0 or handled != m:
                raise RuntimeError(f"batch at push {i} rejected: {rc}")
            now = res[-1].ts_after
            for l in ls:
                learner_ts[l] = now

    if batch > 1:
        assert nbuf >= batch + c
        run_range = run_range_batched
    run_range(0, warmup * c)
    ps.sync()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    launches_before = 0 if flags & 8 else ps.stats().n_apply_launches     # (with the kernel timer on, stats() would wait)
    e0.record(hip.stream)
    t0 = time.perf_counter()
    run_range(warmup * c, (warmup + steps) * c)
    e1.record(hip.stream)
    ps.sync()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)
    st = ps.stats()
    assert st.n_updates == warmup + steps, (st.n_updates, warmup + steps)
    out = dict(wall_s=wall, event_ms=ev_ms, updates=steps, pushes=steps * c, sigma_mean=st.sigma_mean,
               kernel_ms=st.kernel_ms, kernel_launches=st.kernel_launches, timed_launches=st.n_apply_launches - launches_before)
    # sanity: the state is finite and moved
    chk = hip.weights()
    out["theta_absmax"] = float(chk.abs().max())
    assert bool(torch.isfinite(chk).all())
    hip.close()
    del hip, chk
    torch.cuda.empty_cache()
    return out


def run_gpu_tree(w, fan_in, steps, warmup, ring=64):
    """The same replay through a two-level server tree (Sec. 3.3): every `fan_in` gradients of a node are averaged on
    the device (rudra_ps_leaf_mean) and the average is relayed to the root (rudra_ps_push_aggregate)."""
    import torch
    from paper_1509_04210_amd import binding as B
    from synth.learners import HipServer

    n_msgs = w.c // fan_in                                   # relayed messages per update (c divisible by fan_in here)
    hip = HipServer(w, pregenerated=ring, avg_ring=n_msgs + 4, max_aggregate=fan_in)
    ps, bufs, avgs = hip.ps, [b.data_ptr() for b in hip.ring], [b.data_ptr() for b in hip.avg_ring]
    P, sh = w.n_params, hip.sh
    state = dict(g=0, a=0, ts=0)

    def run_updates(n):
        for _ in range(n * n_msgs):
            ptrs = [bufs[(state["g"] + j) % len(bufs)] for j in range(fan_in)]
            state["g"] += fan_in
            avg = avgs[state["a"] % len(avgs)]
            state["a"] += 1
            B.leaf_mean(ptrs, P, avg, 0, sh)
            rc, res = ps.push_aggregate(avg, [state["ts"]] * fan_in)
            if rc != 0:
                raise RuntimeError(f"relayed message rejected: {rc}")
            state["ts"] = res.ts_after                       # learners re-pull after every push (zero-latency tree)

    run_updates(warmup)
    ps.sync()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(hip.stream)
    t0 = time.perf_counter()
    run_updates(steps)
    e1.record(hip.stream)
    ps.sync()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)
    assert ps.stats().n_updates == warmup + steps
    hip.close()
    torch.cuda.empty_cache()
    return dict(wall_s=wall, event_ms=ev_ms, updates=steps, pushes=steps * w.c)


def run_copy_ceiling(n_params, reps=20):
    """What a plain device-to-device copy of one parameter vector reaches on this machine (read + write bytes over time):
    context for the roofline fraction, not a target."""
    import torch
    src = torch.empty(n_params, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del src, dst
    torch.cuda.empty_cache()
    return 8 * n_params / (ms * 1e-3) / 1e9


def run_cpu_oracle(w, n_updates=30, n_distinct=3):
    """The CPU oracle as it stands, single thread, on the full-size vector: `n_updates` applyUpdates of the same
    workload.  Gradient materialisation is excluded from the timing (as on the GPU)."""
    import numpy as np
    import torch
    from oracle.adapter import LR_MODE, PROTOCOL
    from oracle import OraclePS
    from synth import gradgen

    P = w.n_params
    dev = torch.device("cuda", 0)
    buf = torch.empty(P, dtype=torch.float32, device=dev)

    def device_vector(key, std, tail_per):
        gradgen.fill_device(buf.data_ptr(), P, key, std, tail_per, w.tail_factor, stream=0)
        torch.cuda.synchronize()
        return buf.cpu().numpy()

    init = device_vector(w.init_key(), w.init_std, 0)
    grads = [device_vector(w.grad_key(l, 0), w.grad_std, w.tail_per) for l in range(n_distinct)]
    ps = OraclePS(init, w.n_learners, w.n_split, PROTOCOL[w.protocol], LR_MODE[w.lr_mode], w.alpha0, w.lr_scale,
                  w.momentum, w.weight_decay, w.c_override)
    learner, _ = w.arrival_trace(n_updates * w.c)
    learner_ts = [0] * w.n_learners
    t0 = time.perf_counter()
    for i, l in enumerate(learner):
        rc, res = ps.push(grads[i % n_distinct], learner_ts[int(l)], int(l))
        assert rc == 0
        learner_ts[int(l)] = res.ts_after
    dt = time.perf_counter() - t0
    assert ps.ts == n_updates
    return dict(value=n_updates / dt, seconds=dt, updates=n_updates)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4",
                    help="C4 (default, the headline) or any other key of synth.configs.ALL; the small workloads (C1-C3) are "
                         "cache-resident and launch-bound: read their applyUpdates/s, not their roofline fraction")
    ap.add_argument("--ring", type=int, default=64)
    ap.add_argument("--block", type=int, default=0)
    ap.add_argument("--unroll", type=int, default=0)
    ap.add_argument("--vec", type=int, default=0)
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--double-buffer", action="store_true", help="run the server with RUDRA_FLAG_DOUBLE_BUFFER")
    ap.add_argument("--batch", type=int, default=1,
                    help="hand the messages over this many at a time (rudra_ps_push_batch): consecutive updates share a launch; "
                         "the headline is measured with 1 (every update its own launch)")
    ap.add_argument("--waves", type=int, default=0, help="launch_waves_per_cu")
    ap.add_argument("--params", type=int, default=0, help="run the workload's recipe at another vector length (size sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-kernel event pass and the second workload")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="also run this many plain device copies of P floats (known size: 4P bytes read, 4P written) so that "
                         "a rocprofv3 --pmc run of this command has a reference reading for FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (the parameter-server update path does not span GPUs here); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()          # loads what is built; builds only on a fresh checkout
    from paper_1509_04210_amd import binding as B
    from synth import configs
    B.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    launch = dict(launch_block=args.block, launch_unroll=args.unroll, launch_vec=args.vec, launch_grid=args.grid,
                  launch_waves_per_cu=args.waves)
    w = configs.ALL[args.workload]
    if args.params:
        w = w.scaled(n_params=args.params, name=f"{w.name}@{args.params}")
    base_flags = B.FLAG_DOUBLE_BUFFER if args.double_buffer else 0
    r = run_gpu(w, args.steps, args.warmup, ring=args.ring, flags=base_flags, batch=args.batch, **launch)
    bytes_upd = algorithmic_bytes_per_update(w)
    if args.batch > 1:      # per launch: every gradient of its updates once, theta (and the second state vector) once
        bytes_upd = (r["pushes"] * 4 * w.n_params + r["timed_launches"] * (bytes_upd - 4 * w.c * w.n_params)) // r["timed_launches"]
    ups = r["updates"] / r["wall_s"]
    kernel_ms = r["event_ms"] / r["timed_launches"]     # the timed region is back-to-back applyUpdate launches only
    achieved = bytes_upd / (kernel_ms * 1e-3) / 1e9
    traffic = (None if args.params else MEASURED_TRAFFIC_BYTES.get(args.workload) if args.batch == 1 else
               MEASURED_TRAFFIC_BYTES_BATCH8.get(args.workload) if args.batch == 8 else None)
    line = {
        "metric": METRIC, "value": ups, "unit": "applyUpdates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * r["wall_s"] / r["updates"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: P={w.n_params} fp32, lambda={w.n_learners}, {w.n_split}-softsync (c={w.c}), "
                               f"momentum={w.momentum}, wd={w.weight_decay}, lr=alpha0/max(1,<sigma>), "
                               f"ring of {max(args.ring, w.c + 1)} pre-generated gradients",
                   "pushes_per_step": w.c, "launch": {k: v for k, v in launch.items() if v},
                   "double_buffer": bool(args.double_buffer), "messages_per_call": args.batch},
        "absorbed_gradient_GBps": r["pushes"] * 4 * w.n_params / r["wall_s"] / 1e9,
        "pushes_per_s": r["pushes"] / r["wall_s"],
        "mean_staleness": r["sigma_mean"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "apply_update_kernel" if args.batch == 1 else "apply_update_batch_kernel", "bytes_per_launch": bytes_upd, "avg_launch_ms": kernel_ms},
    }
    if args.calibration_copies:
        src = torch.empty(w.n_params, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copies):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_extra:
        line["roofline"]["device_copy_GBps"] = run_copy_ceiling(w.n_params)
        # per-launch HIP events around every applyUpdate (library flag), same workload
        rt = run_gpu(w, min(args.steps, 100), args.warmup, ring=args.ring, flags=base_flags | B.FLAG_TIME_KERNELS, **launch)
        k_ms = rt["kernel_ms"] / max(1, rt["kernel_launches"])
        line["roofline"]["per_launch_event_ms"] = k_ms
        line["roofline"]["per_launch_event_GBps"] = bytes_upd / (k_ms * 1e-3) / 1e9
        # the other 72M workloads, same protocol of measurement: the lambda-softsync stress case (c = 1, momentum +
        # weight penalty) and the 1-softsync case under AdaGrad (what the paper ran for ImageNet 1-softsync, Sec. 5.5)
        line["extra"] = {}
        for other in ([configs.C5] if args.workload == "C4" else [configs.C4]) + [configs.C4_ADAGRAD]:
            ro = run_gpu(other, 1000 if other.c == 1 else 200, 10, ring=args.ring, flags=base_flags, **launch)
            bo = algorithmic_bytes_per_update(other)
            o_ms = ro["event_ms"] / ro["updates"]
            line["extra"][other.name] = {
                "applyUpdates_per_s": ro["updates"] / ro["wall_s"],
                "absorbed_gradient_GBps": ro["pushes"] * 4 * other.n_params / ro["wall_s"] / 1e9,
                "avg_launch_ms": o_ms, "achieved_GBps": bo / (o_ms * 1e-3) / 1e9,
                "frac": bo / (o_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "bytes_per_launch": bo,
                "mean_staleness": ro["sigma_mean"]}
    if not args.no_extra and args.batch == 1:
        # C5 again with the messages handed over 8 at a time (rudra_ps_push_batch): 8 updates per launch, theta and v
        # touched once per launch: P*(4*8 + 16) bytes instead of 8*P*20
        rb = run_gpu(configs.C5, 1024, 64, ring=max(args.ring, 64), flags=base_flags, batch=8, **launch)
        bb = (rb["pushes"] * 4 + rb["timed_launches"] * 16) * configs.C5.n_params // rb["timed_launches"]
        b_ms = rb["event_ms"] / rb["timed_launches"]
        line["extra"]["C5-8-messages-per-call"] = {
            "applyUpdates_per_s": rb["updates"] / rb["wall_s"], "absorbed_gradient_GBps": rb["pushes"] * 4 * configs.C5.n_params / rb["wall_s"] / 1e9,
            "avg_launch_ms": b_ms, "updates_per_launch": rb["updates"] / rb["timed_launches"], "bytes_per_launch": bb,
            "achieved_GBps": bb / (b_ms * 1e-3) / 1e9, "frac": bb / (b_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "kernel": "apply_update_batch_kernel"}
    if not args.no_extra:
        # 54 learners, 1-softsync (the shape of the paper's Rudra-adv ImageNet run, Table 4): flat, and as a tree with nodes of 3
        from dataclasses import replace
        w54 = replace(configs.C4, name="C4-54-learners-flat", n_learners=54)
        rf = run_gpu(w54, 60, 5, ring=args.ring, flags=base_flags, **launch)
        bf = algorithmic_bytes_per_update(w54)
        line["extra"][w54.name] = {"applyUpdates_per_s": rf["updates"] / rf["wall_s"], "avg_launch_ms": rf["event_ms"] / rf["updates"],
                                   "absorbed_gradient_GBps": rf["pushes"] * 4 * w54.n_params / rf["wall_s"] / 1e9,
                                   "achieved_GBps": bf / (rf["event_ms"] / rf["updates"] * 1e-3) / 1e9, "bytes_per_launch": bf}
        rt3 = run_gpu_tree(w54, 3, 60, 5, ring=args.ring)
        # per update: 18 node launches of (3 reads + 1 write) and the root launch over 18 relayed averages + theta, v
        bt = w54.n_params * ((w54.c // 3) * 16 + 4 * (w54.c // 3) + 16)
        line["extra"]["C4-54-learners-tree-of-3"] = {
            "applyUpdates_per_s": rt3["updates"] / rt3["wall_s"], "ms_per_update": rt3["event_ms"] / rt3["updates"],
            "absorbed_gradient_GBps": rt3["pushes"] * 4 * w54.n_params / rt3["wall_s"] / 1e9,
            "achieved_GBps": bt / (rt3["event_ms"] / rt3["updates"] * 1e-3) / 1e9, "bytes_per_update": bt,
            "launches_per_update": w54.c // 3 + 1}
    if not args.no_cpu_baseline:
        cb = run_cpu_oracle(w)
        line["cpu_baseline"] = {"value": cb["value"], "unit": "applyUpdates/s", "cores": 1, "kind": "oracle",
                                "sample": f"{cb['updates']} applyUpdates ({cb['updates'] * w.c} pushes) of the same workload on the full "
                                          f"{w.n_params}-element vector, single thread, {cb['seconds']:.1f} s, gradients pre-materialised",
                                "GBps": cb["value"] * bytes_upd / 1e9}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
