#!/usr/bin/env python3
"""Benchmark of the Rudra parameter-server update path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one applyUpdate of the 72M-parameter 1-softsync workload (C4: lambda = 18 learners, c = 18
gradients per update, momentum 0.9, staleness-modulated rate): 18 pushGradient calls through the C ABI
(staleness, vector clock, rate on the host) and the fused sumGradients+applyUpdate kernel they trigger.
Gradients are synthetic (seeded; 64 distinct 288 MB vectors pre-generated in HBM and cycled, far beyond
the 256 MB Infinity Cache) and already resident when the timed region starts; the arrival order is the
workload's seeded Exp(1) trace.  After W warm-up steps the window of exactly K steps is timed --windows
times (default 3) back to back; the headline is the median window.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "PS applyUpdates/sec and absorbed gradient GB/s (% HBM peak), 72M fp32 params"
HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, vendor figure

# HBM bytes per applyUpdate launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE), each scaled by
# the same counter's reading for a plain copy of known size; figures, commands and the commit they were taken at are in
# profiles/apply_update_kernel_C4_C5_72M_hbm_traffic.md.  Measured constants, not recomputed at run time; a test
# (tests/test_bench_constants.py) fails when one of them is more than 1 % away from the algorithmic bytes of its launch.
MEASURED_TRAFFIC_BYTES = {"C4": 6.3355e9, "C5": 1.43995e9}
MEASURED_TRAFFIC_BYTES_BATCH8 = {"C5": 3.4558e9}   # same files: C5 with 8 messages per call


def algorithmic_bytes_per_update(w) -> int:
    """Each of the c gradients read once, theta read+written once, v read+written once when there is momentum."""
    second_state = w.momentum != 0 or w.optimizer == "adagrad"      # velocity, or AdaGrad's accumulator
    return w.n_params * (4 * w.c + 8 + (8 if second_state else 0))


def run_gpu(w, steps, warmup, ring=64, flags=0, batch=1, windows=3, **launch):
    """Replays (warmup + windows*steps)*c pushes of the workload's arrival trace; after the warm-up, `windows` windows of
    exactly `steps` updates are timed back to back (host wall clock from the first push of the window to stream idle, and
    HIP events on the server's stream around the window's launches); medians and minima over the windows are returned.
    batch > 1: the messages are handed over `batch` at a time (rudra_ps_push_batch; a learner pulls after the call that
    held its push), so consecutive updates share a launch."""
    import torch
    from synth.learners import HipServer

    c = w.c
    learner, step = w.arrival_trace((warmup + windows * steps) * c)
    hip = HipServer(w, flags=flags, pregenerated=max(ring, c + 1, batch + c if batch > 1 else 0), **launch)   # a buffer is reused only after its update
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
    timer_on = bool(flags & 8)              # (with the kernel timer on, stats() would wait for the launches)
    wall, ev_ms, launches = [], [], []
    for k in range(windows):
        lo = (warmup + k * steps) * c
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        before = 0 if timer_on else ps.stats().n_apply_launches
        e0.record(hip.stream)
        t0 = time.perf_counter()
        run_range(lo, lo + steps * c)
        e1.record(hip.stream)
        ps.sync()
        torch.cuda.synchronize()
        wall.append(time.perf_counter() - t0)
        ev_ms.append(e0.elapsed_time(e1))
        launches.append(0 if timer_on else ps.stats().n_apply_launches - before)
    st = ps.stats()
    assert st.n_updates == warmup + windows * steps, (st.n_updates, warmup, windows, steps)
    n_launches = sum(launches) / len(launches)          # (batched hand-over: windows can differ by one launch)
    out = dict(wall_s=statistics.median(wall), wall_s_min=min(wall), wall_windows=wall, event_ms=statistics.median(ev_ms),
               event_ms_min=min(ev_ms), updates=steps, pushes=steps * c, sigma_mean=st.sigma_mean, kernel_ms=st.kernel_ms,
               kernel_launches=st.kernel_launches, timed_launches=n_launches, windows=windows)
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


def run_gpu_pulls(w, steps, warmup, overlap, ring=64, n_reader_streams=2, broadcast=False):
    """A workload with the pullWeights traffic of its learners: after every applyUpdate each of the lambda learners fetches
    the new weights (a device copy of the vector each).  overlap = False: rudra_ps_pull_weights, i.e. the copies queue on
    the server's stream between the updates.  overlap = True: two weight buffers (RUDRA_FLAG_DOUBLE_BUFFER) and
    rudra_ps_pull_weights_on: the copies run on reader streams, concurrently with the next update, and the update after
    that one waits for them (Sec. 3.3: computation and communication buffers with a pointer swap).  broadcast = True: the
    lambda copies of one update go out as ONE rudra_ps_broadcast_weights launch (weights read once, written lambda times),
    on the server's stream or, with overlap, on a reader stream."""
    import torch
    from paper_1509_04210_amd import binding as B
    from synth.learners import HipServer

    c, lam, P = w.c, w.n_learners, w.n_params
    learner, _ = w.arrival_trace((warmup + steps) * c)
    learner = [int(x) for x in learner]
    hip = HipServer(w, flags=B.FLAG_DOUBLE_BUFFER if overlap else 0, pregenerated=max(ring, c + 1))
    ps, bufs = hip.ps, [b.data_ptr() for b in hip.ring]
    dsts = [torch.empty(P, dtype=torch.float32, device=hip.dev) for _ in range(lam if broadcast else 4)]      # where the learners' copies land
    readers = [torch.cuda.Stream(device=hip.dev) for _ in range(n_reader_streams)]
    torch.cuda.synchronize()
    learner_ts = [0] * lam
    n_copies = 0

    def all_learners_pull():
        nonlocal n_copies
        if broadcast:
            ps.broadcast_weights([d.data_ptr() for d in dsts], readers[0].cuda_stream if overlap else hip.sh)
            n_copies += lam
            return
        if not overlap:
            for l in range(lam):
                ps.pull_weights(dsts[l % len(dsts)].data_ptr())
                n_copies += 1
            return
        for l in range(lam):
            ps.pull_weights_on(dsts[l % len(dsts)].data_ptr(), readers[l % len(readers)].cuda_stream)
            n_copies += 1

    def run_range(lo, hi):
        for i in range(lo, hi):
            l = learner[i]
            rc, res = ps.push_gradient(bufs[i % len(bufs)], learner_ts[l], l)
            if rc != 0:
                raise RuntimeError(f"push {i} rejected: {rc}")
            learner_ts[l] = res.ts_after
            if res.applied:
                all_learners_pull()
                if w.protocol == "hardsync":       # the barrier: every learner starts the next step from the new weights
                    learner_ts[:] = [res.ts_after] * lam

    run_range(0, warmup * c)
    ps.sync()
    torch.cuda.synchronize()
    n_copies = 0
    t0 = time.perf_counter()
    run_range(warmup * c, (warmup + steps) * c)
    ps.sync()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    st = ps.stats()
    hip.close()
    del dsts
    torch.cuda.empty_cache()
    return dict(wall_s=wall, updates=steps, copies=n_copies, reader_waits=st.n_reader_waits)


def run_stream_ceilings(n, ptrs, sink_ptr, stream=0):
    """What plain streaming kernels reach on this machine over buffers of the same size (the harness's own kernels, synth/csrc/
    streambench.hip; not the product): read-only passes over 3 and 20 vectors (the stream counts of the c = 1 and c = 18
    launches) and a copy; best of two disjoint buffer sets each."""
    from synth import streambench
    out = {}
    for k in (3, 20):
        out[f"read_{k}_streams"] = max(streambench.read_gbps(ptrs[j * k:(j + 1) * k], n, sink_ptr, reps=10, stream=stream) for j in range(2))
    out["copy"] = max(streambench.copy_gbps(ptrs[2 * j], ptrs[2 * j + 1], n, reps=20, stream=stream) for j in range(2))
    return out


def run_cpu_oracle(w, n_updates=30, n_distinct=3):
    """The CPU oracle as it stands on the full-size vector, `n_updates` applyUpdates of the same workload, twice: on one
    thread, and with the element range cut into one contiguous slice per host core, each slice replayed by its own
    instance of the same oracle on its own thread (the update is elementwise, so every element sees the same operations
    in the same order: the results are asserted bit-identical).  Gradient materialisation is excluded (as on the GPU)."""
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
    del buf
    learner, _ = w.arrival_trace(n_updates * w.c)
    learner = [int(x) for x in learner]

    def replay(lo, hi):
        ps = OraclePS(init[lo:hi], w.n_learners, w.n_split, PROTOCOL[w.protocol], LR_MODE[w.lr_mode], w.alpha0, w.lr_scale,
                      w.momentum, w.weight_decay, w.c_override)
        sl = [g[lo:hi] for g in grads]
        learner_ts = [0] * w.n_learners
        t0 = time.perf_counter()
        for i, l in enumerate(learner):
            rc, res = ps.push(sl[i % n_distinct], learner_ts[l], l)
            assert rc == 0
            learner_ts[l] = res.ts_after
        dt = time.perf_counter() - t0
        assert ps.ts == n_updates
        return ps, dt

    ps1, dt1 = replay(0, P)
    theta1 = ps1.theta
    ps1.close()
    cores = max(1, min(16, len(os.sched_getaffinity(0))))       # a one-GPU machine's share of host cores is 16
    bounds = [P * k // cores for k in range(cores + 1)]
    parts = [None] * cores

    def work(k):
        parts[k] = replay(bounds[k], bounds[k + 1])

    threads = [threading.Thread(target=work, args=(k,)) for k in range(cores)]
    t0 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    dtn = time.perf_counter() - t0
    assert all(p is not None for p in parts)
    for k, (ps, _) in enumerate(parts):
        assert np.array_equal(ps.theta, theta1[bounds[k]:bounds[k + 1]]), "sliced oracle differs from the single-thread oracle"
        ps.close()
    return dict(updates=n_updates, single_value=n_updates / dt1, single_seconds=dt1, cores=cores, value=n_updates / dtn, seconds=dtn)


def _extra_entry(r, bytes_per_launch, n_params):
    ms = r["event_ms"] / r["timed_launches"]
    return {"applyUpdates_per_s": r["updates"] / r["wall_s"], "absorbed_gradient_GBps": r["pushes"] * 4 * n_params / r["wall_s"] / 1e9,
            "avg_launch_ms": ms, "updates_per_launch": r["updates"] / r["timed_launches"], "bytes_per_launch": bytes_per_launch,
            "achieved_GBps": bytes_per_launch / (ms * 1e-3) / 1e9, "frac": bytes_per_launch / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "mean_staleness": r["sigma_mean"], "timed_windows": r["windows"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--windows", type=int, default=3, help="how many times the window of --steps updates is timed (the median is the headline)")
    ap.add_argument("--workload", default="C4",
                    help="C4 (default, the headline) or any other key of synth.configs.ALL; the small workloads (C1-C3) are "
                         "cache-resident and launch-bound: read their applyUpdates/s, not their roofline fraction")
    ap.add_argument("--ring", type=int, default=64)
    ap.add_argument("--block", type=int, default=0)
    ap.add_argument("--unroll", type=int, default=0)
    ap.add_argument("--vec", type=int, default=0)
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--learners", type=int, default=0, help="run the workload's recipe with this many learners (under 1-softsync c = lambda)")
    ap.add_argument("--double-buffer", action="store_true", help="run the server with RUDRA_FLAG_DOUBLE_BUFFER")
    ap.add_argument("--batch", type=int, default=1,
                    help="hand the messages over this many at a time (rudra_ps_push_batch): consecutive updates share a launch; "
                         "the headline is measured with 1 (every update its own launch)")
    ap.add_argument("--waves", type=int, default=0, help="launch_waves_per_cu")
    ap.add_argument("--state-loads", type=int, default=0, help="launch_state_loads")
    ap.add_argument("--phased", action="store_true", help="launch_phased = 2: the phase-aligned kernel (opt-in; for many gradients per update)")
    ap.add_argument("--params", type=int, default=0, help="run the workload's recipe at another vector length (size sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the bandwidth probes, the per-kernel event pass and the other workloads")
    ap.add_argument("--probes-only", action="store_true",
                    help="run only the harness's streaming probes (read-only over 3 and 20 vectors, copy) and print their GB/s: "
                         "the reference launches for counter runs")
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
    __graft_entry__.ensure_built()          # loads what is built; rebuilds only what is missing or older than its sources
    from dataclasses import replace
    from paper_1509_04210_amd import binding as B
    from synth import configs
    B.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.probes_only:
        n = configs.ALL[args.workload].n_params // 4 * 4
        pool = [torch.empty(n, dtype=torch.float32, device="cuda").normal_(std=1e-4) for _ in range(40)]
        sink = torch.zeros(1024, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        print(json.dumps({"stream_probes_GBps": run_stream_ceilings(n, [t.data_ptr() for t in pool], sink.data_ptr()), "n_floats": n}))
        return
    launch = dict(launch_block=args.block, launch_unroll=args.unroll, launch_vec=args.vec, launch_grid=args.grid,
                  launch_waves_per_cu=args.waves, launch_state_loads=args.state_loads, launch_phased=2 if args.phased else 0)
    w = configs.ALL[args.workload]
    if args.params:
        w = w.scaled(n_params=args.params, name=f"{w.name}@{args.params}")
    if args.learners:
        w = replace(w, name=f"{w.name}-{args.learners}-learners", n_learners=args.learners)
    base_flags = B.FLAG_DOUBLE_BUFFER if args.double_buffer else 0
    r = run_gpu(w, args.steps, args.warmup, ring=args.ring, flags=base_flags, batch=args.batch, windows=args.windows, **launch)
    bytes_upd = algorithmic_bytes_per_update(w)
    if args.batch > 1:      # per launch: every gradient of its updates once, theta (and the second state vector) once
        bytes_upd = int((r["pushes"] * 4 * w.n_params + r["timed_launches"] * (bytes_upd - 4 * w.c * w.n_params)) / r["timed_launches"])
    ups = r["updates"] / r["wall_s"]
    kernel_ms = r["event_ms"] / r["timed_launches"]     # the timed region is back-to-back applyUpdate launches only
    achieved = bytes_upd / (kernel_ms * 1e-3) / 1e9
    plain = not (args.params or args.learners or args.double_buffer)
    traffic = (None if not plain else MEASURED_TRAFFIC_BYTES.get(args.workload) if args.batch == 1 else
               MEASURED_TRAFFIC_BYTES_BATCH8.get(args.workload) if args.batch == 8 else None)
    line = {
        "metric": METRIC, "value": ups, "unit": "applyUpdates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * r["wall_s"] / r["updates"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: P={w.n_params} fp32, lambda={w.n_learners}, {w.n_split}-softsync (c={w.c}), "
                               f"momentum={w.momentum}, wd={w.weight_decay}, lr=alpha0/max(1,<sigma>), "
                               f"ring of {max(args.ring, w.c + 1)} pre-generated gradients",
                   "pushes_per_step": w.c, "launch": {k: v for k, v in launch.items() if v},
                   "double_buffer": bool(args.double_buffer), "messages_per_call": args.batch,
                   "timed_windows": args.windows, "headline": "median of the timed windows of `steps` steps each"},
        "ms_per_step_min": 1e3 * r["wall_s_min"] / r["updates"],
        "ms_per_step_windows": [1e3 * x / r["updates"] for x in r["wall_windows"]],
        "absorbed_gradient_GBps": r["pushes"] * 4 * w.n_params / r["wall_s"] / 1e9,
        "pushes_per_s": r["pushes"] / r["wall_s"],
        "mean_staleness": r["sigma_mean"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "apply_update_kernel" if args.batch == 1 else "apply_update_batch_kernel", "bytes_per_launch": bytes_upd,
                     "avg_launch_ms": kernel_ms, "avg_launch_ms_min": r["event_ms_min"] / r["timed_launches"]},
    }
    if args.calibration_copies:
        src = torch.empty(w.n_params, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copies):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_extra:
        # what plain streaming kernels reach over buffers of the same size on this machine (harness kernels, not the product)
        n = w.n_params // 4 * 4
        pool = [torch.empty(n, dtype=torch.float32, device="cuda").normal_(std=1e-4) for _ in range(40)]
        sink = torch.zeros(1024, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        ceil = run_stream_ceilings(n, [t.data_ptr() for t in pool], sink.data_ptr())
        line["roofline"]["stream_read_GBps"] = {"3_streams": ceil["read_3_streams"], "20_streams": ceil["read_20_streams"]}
        line["roofline"]["stream_copy_GBps"] = ceil["copy"]
        del pool, sink
        torch.cuda.empty_cache()
        # per-launch HIP events around every applyUpdate (library flag), same workload
        rt = run_gpu(w, min(args.steps, 100), args.warmup, ring=args.ring, flags=base_flags | B.FLAG_TIME_KERNELS, windows=1, **launch)
        k_ms = rt["kernel_ms"] / max(1, rt["kernel_launches"])
        line["roofline"]["per_launch_event_ms"] = k_ms
        line["roofline"]["per_launch_event_GBps"] = bytes_upd / (k_ms * 1e-3) / 1e9
        # the other 72M workloads, same protocol of measurement: the lambda-softsync stress case (c = 1, momentum +
        # weight penalty) and the 1-softsync case under AdaGrad (what the paper ran for ImageNet 1-softsync, Sec. 5.5)
        line["extra"] = {}
        for other in ([configs.C5] if args.workload == "C4" else [configs.C4]) + [configs.C4_ADAGRAD]:
            ro = run_gpu(other, 1000 if other.c == 1 else 200, 10, ring=args.ring, flags=base_flags, **launch)
            line["extra"][other.name] = _extra_entry(ro, algorithmic_bytes_per_update(other), other.n_params)
        if not args.double_buffer:      # both again with two weight buffers (Sec. 3.3 pointer swap): same bytes per launch
            for other in (configs.C4, configs.C5):
                ro = run_gpu(other, 1000 if other.c == 1 else 200, 10, ring=args.ring, flags=B.FLAG_DOUBLE_BUFFER, **launch)
                line["extra"][other.name + "-double-buffer"] = _extra_entry(ro, algorithmic_bytes_per_update(other), other.n_params)
    if not args.no_extra and args.batch == 1:
        # C5 again with the messages handed over 8, 16 and 64 at a time (rudra_ps_push_batch): k updates per launch, theta
        # and v touched once per launch: P*(4k + 16) bytes instead of k*P*20
        for k in (8, 16, 64):
            rb = run_gpu(configs.C5, 1024 if k < 64 else 1280, 64, ring=max(args.ring, k + 2), flags=base_flags, batch=k, **launch)
            bb = int((rb["pushes"] * 4 + rb["timed_launches"] * 16) * configs.C5.n_params / rb["timed_launches"])
            e = _extra_entry(rb, bb, configs.C5.n_params)
            e["kernel"] = "apply_update_batch_kernel"
            line["extra"][f"C5-{k}-messages-per-call"] = e
    if not args.no_extra:
        # more learners, 1-softsync, flat: c = 30 (the CIFAR10 runs' learner count, at ImageNet size) and c = 54 (the shape of
        # the paper's Rudra-adv ImageNet run, Table 4); c = 54 also as a tree with nodes of 3
        for lam in (30, 54):
            wl = replace(configs.C4, name=f"C4-{lam}-learners-flat", n_learners=lam)
            rf = run_gpu(wl, 60, 5, ring=max(args.ring, lam + 10), flags=base_flags, **launch)
            line["extra"][wl.name] = _extra_entry(rf, algorithmic_bytes_per_update(wl), wl.n_params)
        w54 = replace(configs.C4, name="C4-54-learners-flat", n_learners=54)
        rt3 = run_gpu_tree(w54, 3, 60, 5, ring=args.ring)
        # per update: 18 node launches of (3 reads + 1 write) and the root launch over 18 relayed averages + theta, v
        bt = w54.n_params * ((w54.c // 3) * 16 + 4 * (w54.c // 3) + 16)
        line["extra"]["C4-54-learners-tree-of-3"] = {
            "applyUpdates_per_s": rt3["updates"] / rt3["wall_s"], "ms_per_update": rt3["event_ms"] / rt3["updates"],
            "absorbed_gradient_GBps": rt3["pushes"] * 4 * w54.n_params / rt3["wall_s"] / 1e9,
            "achieved_GBps": bt / (rt3["event_ms"] / rt3["updates"] * 1e-3) / 1e9, "bytes_per_update": bt,
            "launches_per_update": w54.c // 3 + 1}
        # C4 with its learners' pullWeights traffic (18 copies of the weights per update): queued on the server's stream,
        # or overlapped with the next update from the second weight buffer (Sec. 3.3)
        pulls = {}
        for name, overlap, bc in (("serialized_on_the_server_stream", False, False), ("overlapped_from_the_second_buffer", True, False),
                                  ("one_broadcast_launch_on_the_server_stream", False, True), ("one_broadcast_launch_overlapped", True, True)):
            rp = run_gpu_pulls(configs.C4, 40, 4, overlap, broadcast=bc)
            moved = rp["updates"] * algorithmic_bytes_per_update(configs.C4) + (rp["copies"] * 4 + (rp["updates"] * 4 if bc else rp["copies"] * 4)) * configs.C4.n_params
            pulls[name] = {"applyUpdates_per_s": rp["updates"] / rp["wall_s"], "ms_per_update": 1e3 * rp["wall_s"] / rp["updates"],
                           "weight_copies_per_update": rp["copies"] / rp["updates"], "HBM_GBps_updates_plus_copies": moved / rp["wall_s"] / 1e9,
                           "launches_made_to_wait_for_readers": rp["reader_waits"]}
        line["extra"]["C4-with-18-weight-pulls-per-update"] = pulls
        # the short-vector workloads (131k and 1.0M parameters: cache-resident, one generation of waves per launch; read
        # their applyUpdates/s and the time per launch, not a roofline fraction), singly and with 64 messages per call
        short = {}
        for key, k in (("C1", 1), ("C2", 1), ("C3-n1", 1), ("C3-n2", 1), ("C3-n4", 1), ("C3-n30", 1), ("C1", 64), ("C3-n30", 64)):
            ws = configs.ALL[key]
            rs = run_gpu(ws, 2048 if k > 1 else 2000, 64, ring=max(args.ring, k + ws.c + 1), flags=base_flags, batch=k, **launch)
            short[ws.name + (f"-{k}-messages-per-call" if k > 1 else "")] = {
                "applyUpdates_per_s": rs["updates"] / rs["wall_s"], "n_params": ws.n_params, "gradients_per_update": ws.c,
                "avg_launch_us": 1e3 * rs["event_ms"] / rs["timed_launches"], "updates_per_launch": rs["updates"] / rs["timed_launches"]}
        # hardsync ends every step with all learners fetching the new weights (Sec. 3.1): C2 with 30 pulls per update, and
        # with the one broadcast launch instead
        for name, bc in (("C2-with-30-weight-pulls-per-update", False), ("C2-with-one-broadcast-launch-per-update", True)):
            rp = run_gpu_pulls(configs.C2, 1000, 50, False, broadcast=bc)
            short[name] = {"applyUpdates_per_s": rp["updates"] / rp["wall_s"], "us_per_update": 1e6 * rp["wall_s"] / rp["updates"],
                           "weight_copies_per_update": rp["copies"] / rp["updates"]}
        line["extra"]["short-vector-workloads"] = short
    if not args.no_cpu_baseline:
        cb = run_cpu_oracle(w)
        line["cpu_baseline"] = {"value": cb["value"], "unit": "applyUpdates/s", "cores": cb["cores"], "kind": "oracle",
                                "sample": f"{cb['updates']} applyUpdates ({cb['updates'] * w.c} pushes) of the same workload on the full "
                                          f"{w.n_params}-element vector, gradients pre-materialised; the element range cut into "
                                          f"{cb['cores']} slices, one instance of the oracle and one thread per slice, {cb['seconds']:.1f} s "
                                          f"(bit-identical to the single-thread run, which took {cb['single_seconds']:.1f} s)",
                                "GBps": cb["value"] * bytes_upd / 1e9,
                                "single_thread": {"value": cb["single_value"], "cores": 1, "GBps": cb["single_value"] * bytes_upd / 1e9}}
        if args.workload == "C4" and plain and not args.no_extra:      # the other 72M workload beside it: 120 single-gradient updates
            c5 = run_cpu_oracle(configs.C5, n_updates=120)
            b5 = algorithmic_bytes_per_update(configs.C5)
            line["cpu_baseline"]["other_workloads"] = {configs.C5.name: {
                "value": c5["value"], "unit": "applyUpdates/s", "cores": c5["cores"], "GBps": c5["value"] * b5 / 1e9,
                "sample": f"{c5['updates']} applyUpdates of one gradient each on the full vector, {c5['seconds']:.1f} s; single thread {c5['single_seconds']:.1f} s",
                "single_thread": {"value": c5["single_value"], "cores": 1, "GBps": c5["single_value"] * b5 / 1e9}}}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
