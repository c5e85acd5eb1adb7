"""Benchmark: full ASNN activation on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--flags 0] [--no-cpu]

A step is one asnn_activate call: every level of the packed network for the
whole batch (input staging, gather-FMA-sigmoid per level, output extraction),
graph and inputs resident in HBM.  Prints ONE JSON line: whole-job throughput
in G edge*samples/s, the roofline of the dominant kernel from HIP-event
timings of the level launches, and the CPU oracle timed on this host.
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

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth


def algorithmic_bytes(n_nodes, n_edges, n_inputs, B):
    """Gather model of one activation: every connection fetches one fp32 of
    its source per sample and its (col, w) pair once; every node value is
    written once; row_ptr is read once; the inputs are read once."""
    gather = 4.0 * n_edges * B
    store = 4.0 * n_nodes * B
    csr = 8.0 * n_edges + 4.0 * n_nodes
    inputs = 4.0 * n_inputs * B
    return gather + store + csr + inputs


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown CPU"


KERNEL_SOURCES = ("paper_2005_04347_amd/csrc/activate.hip", "paper_2005_04347_amd/csrc/asnn_common.h")


def kernel_source_sha256():
    """Fingerprint of the sources the activation kernels are built from (ties a counter summary to the code it measured)."""
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, rel), "rb").read())
    return h.hexdigest()


def measured_traffic(config, flags):
    """L2<->fabric bytes per launch (reads + writes, Infinity-Cache hits included) from the committed
    rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this workload: counter runs cannot be made from inside this
    process.  None when no summary covers the workload, or when the summary was taken from other kernel
    sources than the ones in this tree (it names the fingerprint of the sources it measured)."""
    import glob
    paths = glob.glob(os.path.join(ROOT, "profiles", f"*_config{config}_hbm_traffic.md"))
    if flags != 0 or not paths:
        return None
    traffic, sha = None, None
    for line in open(paths[0]):
        if line.startswith("traffic_bytes_per_launch:"):
            traffic = float(line.split(":")[1])
        if line.startswith("kernel_source_sha256:"):
            sha = line.split(":")[1].strip()
    return traffic if sha == kernel_source_sha256() else None


def paper_regime(flags=0, quick=False):
    """The paper's own experiment on this machine: ONE input vector per activation, time against the
    number of connections for shallow and deep networks, GPU (10 runs averaged, as in the paper's
    experimental setup) against the sequential oracle (5 runs averaged).  Prints one JSON line per network.

    GPU figures, all with the network resident: "resident" = 10 activations enqueued back to back through
    a call whose arguments were marshalled once (Network.bind), between two events; "graph replay" = the
    same 10 activations captured in a HIP graph and replayed (no host call between two kernels: what the
    device itself needs per activation, kernel plus hand-over); "binding" = the same through the general
    Python entry point, which marshals thirteen arguments and looks the stream up on every call; "with
    host copies" = host X in, host Y out around every activation, as the paper timed it; "pinned I/O" =
    X and Y in pinned host memory that the kernels read and write in place."""
    import numpy as np
    import torch

    import oracle
    import paper_2005_04347_amd as amd
    from workloads import layered_skip

    amd.load()
    torch.empty(16, pin_memory=True)        # (the first pinned allocation of a process sets up the host allocator)
    # connections swept at two depths, then depth swept at a fixed number of connections
    sweep = [(L, E) for L in (5, 40) for E in (1000, 2000, 4000, 8000, 16000, 30000, 70000, 150000, 300000)]
    sweep += [(L, 16000) for L in (3, 10, 20, 80, 160)]
    if quick:
        sweep = [(5, 1000), (5, 16000), (40, 4000)]

    def events_around(fn, reps=10):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    for index, (n_levels, n_edges) in enumerate(sweep[:1] + sweep):     # the first network once more, unreported: first-use costs
        n_nodes = max(n_edges // 10, 3 * n_levels)
        n_io = max(4, n_nodes // 50)
        wl = layered_skip(seed=1, n_nodes=n_nodes, n_inputs=n_io, n_outputs=n_io, n_levels=n_levels, B=1,
                          mean_extra_degree=n_edges / (n_nodes - n_io) - 1.0)
        net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
        X = torch.from_numpy(wl.X).cuda()
        V = torch.empty((wl.n_nodes, 1), device="cuda")
        Y = torch.empty((len(wl.output_ids), 1), device="cuda")
        bound = net.bind(X, V=V, Y=Y, flags=flags)
        for _ in range(5):
            bound.launch()
        torch.cuda.synchronize()
        gpu_us = min(events_around(bound.launch) for _ in range(3))
        binding_us = min(events_around(lambda: net.activate(X, V=V, Y=Y, flags=flags)) for _ in range(3))
        # ten activations in one HIP graph (captured on a side stream), replayed
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            side_bound = net.bind(X, V=V, Y=Y, flags=flags)
            side_bound.launch()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(10):
                    side_bound.launch()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        graph_us = min(events_around(graph.replay, reps=3) for _ in range(3)) / 10
        t0 = time.perf_counter()
        for _ in range(10):
            Xd = torch.from_numpy(wl.X).cuda()
            net.activate(Xd, V=V, Y=Y, flags=flags)
            y_host = Y.cpu()
        copy_us = (time.perf_counter() - t0) * 1e6 / 10
        # the same without copies: X and Y live in pinned host memory and the kernels read and write them in place
        Xp = torch.empty(wl.X.shape, dtype=torch.float32, pin_memory=True)
        Yp = torch.empty((len(wl.output_ids), 1), dtype=torch.float32, pin_memory=True)
        x_host = torch.from_numpy(wl.X)
        pinned = net.bind(Xp, V=V, Y=Yp, flags=flags)
        for _ in range(5):
            pinned.launch()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            Xp.copy_(x_host)
            pinned.launch()
            torch.cuda.synchronize()
            y_host = Yp.clone()
        pinned_us = (time.perf_counter() - t0) * 1e6 / 10
        assert torch.equal(y_host, Y.cpu())
        oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
        cpu_us = 0.0
        for _ in range(5):          # the node loop only: the paper times activation after its preprocessing
            tm = {}
            ref = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X, timing=tm)
            cpu_us += tm["activation_seconds"] * 1e6 / 5
        err = float(np.abs(net.values_original_order(V).cpu().numpy().astype(np.float64) - ref).max())
        if index == 0:
            continue
        print(json.dumps({"regime": "paper: batch 1", "connections": wl.n_edges, "nodes": wl.n_nodes,
                          "levels": net.n_levels,
                          "schedule_taken": amd.asnn_activate_schedule(net.graph, 1, True, flags),
                          "gpu_us_resident": round(gpu_us, 1), "gpu_us_graph_replay": round(graph_us, 1),
                          "gpu_us_resident_through_binding": round(binding_us, 1),
                          "gpu_us_with_host_copies": round(copy_us, 1),
                          "gpu_us_pinned_host_io": round(pinned_us, 1), "cpu_oracle_us": round(cpu_us, 1),
                          "speedup_resident": round(cpu_us / gpu_us, 2),
                          "speedup_with_host_copies": round(cpu_us / copy_us, 2),
                          "speedup_pinned_host_io": round(cpu_us / pinned_us, 2), "max_abs_err": err}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--flags", type=int, default=0, help="asnn_activate flags (2 = fp32 accumulate)")
    ap.add_argument("--schedule", choices=["auto", "levels", "dataflow", "workgroup"], default="auto",
                    help="level launches, persistent dataflow launch, or the library's own choice")
    ap.add_argument("--graph", action="store_true", help="capture one asnn_activate in a HIP graph and time replays")
    ap.add_argument("--no-cpu", action="store_true",
                    help="the timed activation and its yardsticks only: skip the cpu_baseline leg and the fp32-sum side timing")
    ap.add_argument("--regime-quick", action="store_true", help="with --paper-regime: three networks only (for profiling)")
    ap.add_argument("--paper-regime", action="store_true",
                    help="batch-1 latency against connections, as in the paper's figures (prints one line per network)")
    args = ap.parse_args()
    if args.paper_regime:
        paper_regime({"auto": 0, "levels": 4, "dataflow": 8, "workgroup": 16}[args.schedule], quick=args.regime_quick)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (batch columns and networks of a population would shard "
              "without any exchange step, but no multi-GPU figure is produced here). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2005_04347_amd as amd
    from workloads import make_config

    amd.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    wl = make_config(args.config, "full")
    t0 = time.perf_counter()
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids, device=dev)
    torch.cuda.synchronize()
    prep_ms = (time.perf_counter() - t0) * 1e3
    # the two preprocess calls once more, now warm, timed apart (host wall clock around each: both block)
    t0 = time.perf_counter()
    level, n_levels = amd.asnn_build_levels(wl.n_nodes, net.src, net.dst, net.input_ids)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    amd.asnn_pack_csr(wl.n_nodes, n_levels, net.src, net.dst, net.w_edges, level)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    levels_ms, pack_ms = (t1 - t0) * 1e3, (t2 - t1) * 1e3
    del level
    X = torch.from_numpy(wl.X).to(dev)
    B = wl.B
    V = torch.empty((wl.n_nodes, B), dtype=torch.float32, device=dev)
    Y = torch.empty((len(wl.output_ids), B), dtype=torch.float32, device=dev)

    flags = args.flags | {"auto": 0, "levels": amd.FLAG_LEVEL_LAUNCHES, "dataflow": amd.FLAG_DATAFLOW,
                          "workgroup": amd.FLAG_WORKGROUP}[args.schedule]

    # one asnn_activate call with its arguments marshalled once (at one input vector the marshalling of the
    # general Python entry point costs more than the kernel)
    step = net.bind(X, V=V, Y=Y, flags=flags).launch

    if args.graph:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            side_step = net.bind(X, V=V, Y=Y, flags=flags).launch        # (bound to the capture stream)
            side_step()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                side_step()
        torch.cuda.synchronize()
        step = graph.replay

    # yardsticks: what a plain streaming copy (read + write bytes), a plain streaming read and a random
    # row gather in the launch shape of this workload's levels sustain on this device
    def timed(fn, reps):
        for _ in range(2):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    n_copy = 256 * 1024 * 1024
    ca = torch.empty(n_copy, dtype=torch.float32, device=dev)
    cb = torch.empty(n_copy, dtype=torch.float32, device=dev)
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    copy_gbps = 2.0 * 4.0 * n_copy / timed(lambda: amd.asnn_device_copy(cb, ca), 5) / 1e9
    read_gbps = 4.0 * n_copy / timed(lambda: amd.asnn_device_read(ca, sink), 5) / 1e9
    del ca, cb
    gather_gbps = None
    gather_store_gbps = None
    n_upper = wl.n_nodes - int(net.graph.level_ptr_host[3])          # rows above level 0
    if B % 64 == 0 and net.n_levels > 1 and n_upper > 0:
        # the value matrix itself is the buffer (its size and row length are the workload's); one launch per
        # level with that level's number of rows, every row gathering the average in-degree from random rows
        # BELOW its level (a level only reads lower levels, so early levels gather from a small, cached prefix)
        lp = net.graph.level_ptr_host
        gathers = max(1, round(wl.n_edges / n_upper))
        shape = [(int(lp[3 * l]), int(lp[3 * l + 3] - lp[3 * l])) for l in range(1, net.n_levels)]
        V.uniform_(0.0, 1.0)

        def gather_step():
            for lvl, (below, rows) in enumerate(shape):
                amd.asnn_device_gather(V[:below], rows, gathers, lvl, sink)
        gather_gbps = sum(rows for _, rows in shape) * gathers * B * 4.0 / timed(gather_step, 5) / 1e9
        # the same gathers with every row of the level stored as well (to a second matrix, so that V stays the
        # read-only source): the traffic of a level without its arithmetic and without its graph
        V2 = torch.empty_like(V)

        def gather_store_step():
            for lvl, (below, rows) in enumerate(shape):
                amd.asnn_device_gather_store(V[:below], gathers, lvl, V2[below:below + rows])
        gather_store_gbps = (sum(rows for _, rows in shape) * (gathers + 1) * B * 4.0
                             / timed(gather_store_step, 5) / 1e9)
        del V2

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # whole-step timing: wall clock around K steps bracketed by synchronisation
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # kernel-only timing with HIP events on the launch stream (same stream the
    # library launches on): events bracket each step, so the figure is the
    # device time of all level launches of one activation, launch gaps included
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in ev:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    net.check(B)                                    # raises if a dataflow wait gave up
    dev_ms = sorted(a.elapsed_time(b) for a, b in ev)
    dev_ms_med = dev_ms[len(dev_ms) // 2]

    # beside it, not as the result: the same activation with fp32 sums (the paper's Float; the mode keeps the
    # parity bound on the 100k-node workload only, see tests/test_gpu_parity.py)
    fp32_ms = None
    if (flags & amd.FLAG_ACC_F32) == 0 and not args.graph and not args.no_cpu:
        fast_step = net.bind(X, V=V, Y=Y, flags=flags | amd.FLAG_ACC_F32).launch
        for _ in range(3):
            fast_step()
        ev32 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for a, b in ev32:
            a.record()
            fast_step()
            b.record()
        torch.cuda.synchronize()
        net.check(B)
        fp32_ms = sorted(a.elapsed_time(b) for a, b in ev32)[len(ev32) // 2]

    edge_samples = float(wl.n_edges) * B
    value = edge_samples / (wall_ms * 1e-3) / 1e9
    alg_bytes = algorithmic_bytes(wl.n_nodes, wl.n_edges, len(wl.input_ids), B)
    achieved = alg_bytes / (dev_ms_med * 1e-3) / 1e9
    taken = amd.asnn_activate_schedule(net.graph, B, True, flags)
    # level launches: one gather launch per level above the input level; the other schedules: one launch
    launches = max(net.n_levels - 1, 1) if taken == "levels" else 1
    traffic = measured_traffic(args.config, args.flags) if args.schedule == "auto" and not args.graph else None
    avg_launch_s = dev_ms_med * 1e-3 / launches
    counter_gbps = None if traffic is None else traffic / avg_launch_s / 1e9
    out = {
        "metric": "G edge*samples/s for full ASNN activation",
        "value": round(value, 3),
        "unit": "G edge*samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if (args.flags & 2) else "f64",
        "data": "synthetic",
        "config": {"workload": f"config{args.config}:{wl.name}", "n_nodes": wl.n_nodes, "n_edges": wl.n_edges,
                   "n_levels": net.n_levels, "batch": B, "n_nets": wl.n_nets, "flags": flags, "schedule": args.schedule, "schedule_taken": taken, "hip_graph": bool(args.graph),
                   "preprocess_ms_first_call": round(prep_ms, 2),
                   "build_levels_ms": round(levels_ms, 3), "pack_csr_ms": round(pack_ms, 3),
                   "preprocess_M_connections_per_s": round(wl.n_edges / ((levels_ms + pack_ms) * 1e-3) / 1e6, 1)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "achieved_is": "algorithmic bytes of the gather model (4 B per connection and sample, whether or "
                                    "not the line came from a cache) per second of device time",
                     "traffic_is": "L2<->fabric bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (Infinity-Cache "
                                   "hits included, so an upper bound on HBM bytes); null when profiles/ holds no "
                                   "summary taken from these kernel sources",
                     "counter_GBps": None if counter_gbps is None else round(counter_gbps, 1),
                     "counter_frac": None if counter_gbps is None else round(counter_gbps / HBM_PEAK_GBPS, 4),
                     "kernel": {"dataflow": "dataflow_kernel (one persistent launch)",
                                "workgroup": "workgroup_kernel (one launch, one workgroup per batch tile)",
                                "levels": "gather_light_kernel / gather_mixed_kernel (one launch per level)"}[taken],
                     "launches_per_step": launches,
                     "algorithmic_bytes_per_launch": alg_bytes / launches,
                     "avg_launch_us": round(dev_ms_med * 1e3 / launches, 3),
                     "algorithmic_bytes_per_step": alg_bytes, "device_ms_per_step_median": round(dev_ms_med, 4),
                     "device_ms_per_step_min": round(dev_ms[0], 4),
                     "with_fp32_sums": None if fp32_ms is None else {
                         "device_ms_per_step_median": round(fp32_ms, 4),
                         "achieved": round(alg_bytes / (fp32_ms * 1e-3) / 1e9, 1),
                         "frac": round(alg_bytes / (fp32_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "is": "the same call with ASNN_FLAG_ACC_F32, timed beside the result for information: "
                               "within the parity bound on config 3 only, so never the reported value"},
                     "device_copy_GBps": round(copy_gbps, 1), "device_read_GBps": round(read_gbps, 1),
                     "device_gather_GBps": None if gather_gbps is None else round(gather_gbps, 1),
                     "device_gather_store_GBps": None if gather_store_gbps is None else round(gather_store_gbps, 1),
                     "frac_of_device_read": round(achieved / read_gbps, 4),
                     "frac_of_device_gather": None if gather_gbps is None else round(achieved / gather_gbps, 4),
                     "frac_of_device_gather_store": None if gather_store_gbps is None else round(achieved / gather_store_gbps, 4),
                     "yardsticks_are": "copy: 1 GiB read + 1 GiB written; read: 1 GiB streamed; gather: one launch per level in the "
                                       "level launches' shape, every row loading the average in-degree of random rows "
                                       "below its level from the value matrix, no arithmetic; gather_store: the same and "
                                       "every row of the level stored too (bytes loaded + bytes stored per second)"},
    }
    if not args.no_cpu:
        import oracle
        # the sequential baseline: one thread, pinned to the core it is running on
        pinned_to = None
        try:
            allowed = sorted(os.sched_getaffinity(0))
            pinned_to = allowed[len(allowed) // 2]
            os.sched_setaffinity(0, {pinned_to})
        except (AttributeError, OSError):
            pass
        # calibrate on 8 columns, then time as many columns as fit in about 15 s (columns are independent)
        probe = np.ascontiguousarray(wl.X[:, :min(B, 8)])
        oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, probe[:, :1])     # warm-up / build
        t0 = time.perf_counter()
        oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, probe)
        per_col = (time.perf_counter() - t0) / probe.shape[1]
        cols = int(max(1, min(B, 15.0 / max(per_col, 1e-9))))
        Xs = np.ascontiguousarray(wl.X[:, :cols])
        # whole passes over the sample until about 10 s of CPU work are on the clock; the figure is the
        # oracle's own clock around its node loop (activation only: the adjacency lists it builds first
        # are its preprocessing, as the levels and the packing are the GPU path's)
        cpu_s, loop_s, passes = 0.0, 0.0, 0
        while cpu_s < 10.0 and passes < 1000:
            tm = {}
            t0 = time.perf_counter()
            oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, Xs, timing=tm)
            cpu_s += time.perf_counter() - t0
            loop_s += tm["activation_seconds"]
            passes += 1
        out["cpu_baseline"] = {
            "value": round(float(wl.n_edges) * cols * passes / loop_s / 1e9, 4), "unit": "G edge*samples/s", "cores": 1,
            "kind": "oracle",
            "sample": f"the same network, first {cols} of {B} batch columns (columns are independent), "
                      f"{passes} passes, {loop_s:.2f} s in the oracle's node loop ({cpu_s:.2f} s with its adjacency "
                      f"build), single thread" + (f" pinned to core {pinned_to}" if pinned_to is not None else "") +
                      f", {os.cpu_count()} visible host cores ({cpu_model()})",
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
