#!/usr/bin/env python3
"""Benchmark of the sharded-RNG hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: the fused dropout
of workload C5 (bf16 attention probabilities, global [8,32,4096,4096], nested 2-D mesh 4x2
with the head dimension sharded on both mesh dimensions) for ONE rank's [8,4,4096,4096]
share - shard geometry and decode plan on the host, then index decode, Philox4x32-10,
mask, scale and stores in one kernel - followed by the host-side offset advance.  Inputs
are resident in HBM before the timed region.  The metric is algorithmic bytes per second
(2 B read + 2 B written + 1 B mask per element).

Prints ONE JSON line.  Only one GPU is used: --gpus above 1 is refused.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published peak HBM bandwidth


def algorithmic_bytes(op, dtype, numel):
    """Bytes the method itself must move per launch: fills write one element each; dropout
    reads x and writes y and the one-byte mask."""
    size = 4 if dtype == "f32" else 2
    return numel * (2 * size + 1 if op == "dropout" else size)


def read_traffic(workload_tag):
    """HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), taken
    from the committed profile summary, or None when no such summary exists."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload_tag)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def make_launcher(v, W, torch, w, coord, copies=1):
    """Returns (launch(k), numel, algorithmic bytes) for workload w on rank `coord`.
    `copies` distinct buffer sets are cycled so that small shards do not sit in cache."""
    sh = v.Sharding(*w.sharding_args(coord))
    shape, n = v.vesrng_local_shape(sh)
    code = v.F32 if w.dtype == "f32" else v.BF16
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    outs = [torch.empty(n, dtype=tdt, device="cuda") for _ in range(copies)]
    if w.op == "dropout":
        xs = [W.device_activations(shape, w.input_seed + k, w.input_kind, w.dtype).reshape(-1) for k in range(copies)]
        masks = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(copies)]
    state = {"offset": w.offset}

    def launch(k):
        i = k % copies
        off = state["offset"]
        if w.op == "uniform":
            v.vesrng_uniform(sh, code, w.params["low"], w.params["high"], w.seed, off, outs[i])
        elif w.op == "normal":
            v.vesrng_normal(sh, code, w.params["mean"], w.params["std"], w.seed, off, outs[i])
        else:
            v.vesrng_dropout(sh, code, w.params["p"], w.seed, off, xs[i], outs[i], masks[i])
        state["offset"] = v.vesrng_advance_offset(sh, off)   # every rank steps by the global size

    return launch, n, algorithmic_bytes(w.op, w.dtype, n)


def time_kernel(torch, launch, steps, warmup):
    """Average launch duration from HIP events recorded on the launch stream around each call."""
    for k in range(warmup):
        launch(k)
    torch.cuda.synchronize()
    pairs = []
    for k in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        launch(k)
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in pairs)
    return sum(ms) / len(ms), ms[len(ms) // 2], ms[0]


def time_batch(torch, launch, reps, warmup):
    """Average duration of back-to-back launches (one event pair around the whole batch):
    for kernels of a few microseconds, where a per-launch event pair would dominate."""
    for k in range(warmup):
        launch(k)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for k in range(reps):
        launch(k)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def time_graph(torch, launch, reps):
    """Per-launch time of `reps` back-to-back launches replayed from a captured HIP graph: the
    GPU-side cost without the host's issue rate (the library only enqueues kernels, so its calls
    can be captured)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        launch(0)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for k in range(reps):
                launch(k)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        graph.replay()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) / reps)
    return sorted(times)[len(times) // 2]


def measured_ceilings(B, torch):
    """Rates of the plain probe kernels on this machine, in this run: what bare 128-bit stores,
    a 16-byte copy, the dropout kernel's access pattern without arithmetic, and the generator
    alone can reach.  1 GiB buffers (beyond the 256 MB last-level cache)."""
    nbytes = 1 << 30
    units = nbytes // 16
    a = torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    m = torch.empty(nbytes // 8, dtype=torch.int32, device="cuda")
    blocks = 1 << 30

    def med(fn):
        return time_kernel(torch, lambda _k: fn(), 20, 3)[1] * 1e-3

    t_store = med(lambda: B.vesrng_bench_probe(B.PROBE_STORE, units, None, a))
    t_copy = med(lambda: B.vesrng_bench_probe(B.PROBE_COPY, units, a, b))
    t_mix = med(lambda: B.vesrng_bench_probe(B.PROBE_DROPOUT_TRAFFIC, units, a, b, m))
    t_gen = med(lambda: B.vesrng_bench_probe(B.PROBE_PHILOX, blocks, None, a))
    return {"store_only_gb_per_s": nbytes / t_store / 1e9, "copy_gb_per_s": 2 * nbytes / t_copy / 1e9,
            "dropout_traffic_gb_per_s": 2.5 * nbytes / t_mix / 1e9,
            "philox_only_gblocks_per_s": blocks / t_gen / 1e9,
            "note": "plain probe kernels of libvesrng_bench.so (vesrng_bench_probe), medians of 20 launches in this run"}


SETTLE = 60                        # untimed launches before the timed region, at least (see main)
VALU_PEAK = 256 * 4 * 32 * 2.4e9   # lane-operations/s: 256 CUs x 4 SIMDs x 32 lanes/cycle x 2.4 GHz
                                   # (= the published 157.3 TFLOP/s fp32 vector rate / 2 flops per FMA)


def steady_state(v, W, torch):
    """The operators of the small configs at 64x the shard (same shapes of run), where launch latency
    no longer dominates: C2's ragged fp32 normal fill (at this size the library stages it through LDS
    with the large tile instead of using C2's own ragged kernel) and C3's bf16 normal fill (same
    kernel as C3).  The bf16 fill is ALU-bound; its roofline is the vector issue rate (VALU
    instructions per element from profiles/counters_bench_kernels.txt)."""
    import copy
    res = {}
    for wl, scale_dim, valu_per_elem in ((W.C2, 0, None), (W.C3, 0, 161.0 / 8)):
        big = copy.deepcopy(wl)
        big.global_shape = list(wl.global_shape)
        big.global_shape[scale_dim] *= 64
        launch, numel, nb = make_launcher(v, W, torch, big, wl.bench_coord, 1)
        avg, med, mn = time_kernel(torch, launch, 20, 3)
        gbs = nb / (med * 1e-3) / 1e9
        r = {"workload": "%s with dim %d x64 (beyond the 256 MB last-level cache): shard of %d elements" % (wl.name, scale_dim, numel),
             "median_launch_us": med * 1e3, "gb_per_s": gbs, "pct_hbm_peak": 100 * gbs / HBM_PEAK_GBS,
             "gsamples_per_s": numel / (med * 1e-3) / 1e9}
        if valu_per_elem is not None:
            lane_ops = valu_per_elem * numel / (med * 1e-3)
            r.update({"valu_lane_ops_per_s": lane_ops, "pct_valu_issue_peak": 100 * lane_ops / VALU_PEAK})
        res[wl.name.split()[0] + "x64"] = r
    return res


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(torch, W, w, coord, x_dev, sample):
    """The oracle, as it stands, on the first `sample` elements of the same shard: all host threads
    (the `value`), and one thread on a 32 times smaller sample."""
    import numpy as np
    import oracle
    threads = min(16, os.cpu_count() or 1)
    args = tuple(w.sharding_args(coord))
    n = x_dev.numel()
    xh = np.zeros(n, dtype=np.uint16)    # untouched pages cost nothing; only the sample is filled
    xh[:sample] = x_dev[:sample].view(torch.int16).cpu().numpy().view(np.uint16)
    t0 = time.perf_counter()
    oracle.dropout(args, oracle.BF16, w.params["p"], w.seed, 0, xh, i_begin=0, i_end=sample, threads=threads)
    dt = time.perf_counter() - t0
    one = max(1, sample // 32)
    t0 = time.perf_counter()
    oracle.dropout(args, oracle.BF16, w.params["p"], w.seed, 0, xh, i_begin=0, i_end=one, threads=1)
    dt1 = time.perf_counter() - t0
    return {"value": algorithmic_bytes(w.op, w.dtype, sample) / dt / 1e9, "unit": "GB/s", "cores": threads,
            "kind": "oracle", "seconds": dt, "gsamples_per_s": sample / dt / 1e9,
            "sample": "first %d of %d elements of the same C5 shard (scalar C++ oracle, %d std::threads)" % (sample, n, threads),
            "single_thread": {"value": algorithmic_bytes(w.op, w.dtype, one) / dt1 / 1e9, "unit": "GB/s", "seconds": dt1,
                              "gsamples_per_s": one / dt1 / 1e9, "sample": "first %d elements, 1 thread" % one},
            "cpu_model": cpu_model(), "logical_cpus_visible": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-config side measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known size) to scale rocprofv3's byte counters")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (mesh ranks are emulated on it); --gpus above 1 is not supported")

    import torch
    import paper_2509_07003_amd as v
    from paper_2509_07003_amd import bench_binding as B
    from paper_2509_07003_amd import workloads as W
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)

    w, coord = W.C5, W.C5.bench_coord
    sh = v.Sharding(*w.sharding_args(coord))
    shape, n = v.vesrng_local_shape(sh)
    x = W.device_activations(shape, w.input_seed, w.input_kind, w.dtype).reshape(-1)
    y = torch.empty_like(x)
    mask = torch.empty(n, dtype=torch.uint8, device="cuda")
    nbytes = algorithmic_bytes(w.op, w.dtype, n)
    state = {"offset": 0}

    def step(_k=0):
        v.vesrng_dropout(sh, v.BF16, w.params["p"], w.seed, state["offset"], x, y, mask)
        state["offset"] = v.vesrng_advance_offset(sh, state["offset"])

    # The first ~20 ms of GPU work after an idle period (and the first touch of 2.5 GB of buffers)
    # run about 1.5 % slower: whatever --warmup says, at least SETTLE untimed launches come first.
    settle = max(0, SETTLE - a.warmup)
    for _ in range(settle):
        v.vesrng_dropout(sh, v.BF16, w.params["p"], w.seed, 0, x, y, mask)
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region.  Every tenth launch (at least five of them) sits between two HIP events recorded on the launch
    # stream (no host synchronisation inside the region), so the dominant kernel's duration is
    # measured on launches that are part of `value`; bracketing every launch would put two more
    # packets between each pair of kernels and cost `value` about 1.5 %.
    every = max(1, min(10, a.steps // 5))
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range((a.steps + every - 1) // every)]
    t0 = time.perf_counter()
    for k in range(a.steps):
        if k % every == 0:
            ea, eb = pairs[k // every]
            ea.record()
            step()
            eb.record()
        else:
            step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / a.steps
    value = nbytes / (wall / a.steps) / 1e9
    launch_ms = sorted(ea.elapsed_time(eb) for ea, eb in pairs)
    avg_ms, med_ms, min_ms = sum(launch_ms) / len(launch_ms), launch_ms[len(launch_ms) // 2], launch_ms[0]
    achieved = nbytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "vesrng::aligned_kernel<3 (dropout), 1 (bf16), unsigned int, 1 run axis>", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic("c5_dropout_bf16"),
                "avg_launch_ms": avg_ms, "median_launch_ms": med_ms, "min_launch_ms": min_ms,
                "algorithmic_bytes_per_launch": nbytes}

    out = {"metric": "sharded RNG fill / fused dropout GB/s per MI355X and % of HBM peak", "value": value,
           "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u32 Philox + f32 scale, bf16 in/out, u8 mask", "data": "synthetic",
           "config": {"workload": w.name, "rank": coord, "local_shape": shape, "elements": n, "settle_launches": settle,
                      "gsamples_per_s": n / (wall / a.steps) / 1e9, "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBS},
           "roofline": roofline}

    props = torch.cuda.get_device_properties(0)
    dev = {"name": props.name, "compute_units": props.multi_processor_count,
           "hbm_gib": round(props.total_memory / 2 ** 30, 1)}
    cus, sclk_khz, mem_khz, bus_bits, wall_khz = B.vesrng_bench_device_info()
    # HBM3E at 8 Gb/s per pin makes four transfers per reported memory clock (2 GHz on MI355X).
    dev.update({"shader_clock_mhz": sclk_khz / 1e3, "memory_clock_mhz": mem_khz / 1e3, "memory_bus_bits": bus_bits,
                "hbm_peak_at_4_transfers_per_clock_gb_per_s": 4 * mem_khz * 1e3 * bus_bits / 8 / 1e9,
                "valu_lanes": cus * 4 * 16})
    out["device"] = dev

    if a.calibrate_copy:
        for _ in range(3):
            y.copy_(x)   # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()

    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, W, w, coord, x, sample=n)

    if not a.no_extra:
        del x, y, mask
        ceil = measured_ceilings(B, torch)
        out["ceilings"] = ceil
        roofline["frac_of_measured_traffic_ceiling"] = achieved / ceil["dropout_traffic_gb_per_s"]
        roofline["frac_of_measured_generator_ceiling"] = (n / 4 / (avg_ms * 1e-3) / 1e9) / ceil["philox_only_gblocks_per_s"]
        extra = {}
        for wl, copies in ((W.C1, 256), (W.C2, 16), (W.C3, 32), (W.C4, 8), (W.C5_INTERLEAVED, 1)):
            launch, numel, nb = make_launcher(v, W, torch, wl, wl.bench_coord, copies)
            avg = time_batch(torch, launch, max(50, a.steps), 5)
            per_launch_graph = time_graph(torch, launch, 4 * copies if copies > 1 else 8)
            extra[wl.name.split()[0] + ("i" if wl is W.C5_INTERLEAVED else "")] = {
                "graph_replay_us_per_launch": per_launch_graph * 1e3,
                "graph_replay_gb_per_s": nb / (per_launch_graph * 1e-3) / 1e9,
                "workload": wl.name, "elements": numel, "algorithmic_bytes": nb, "avg_launch_us": avg * 1e3,
                "gb_per_s": nb / (avg * 1e-3) / 1e9, "gsamples_per_s": numel / (avg * 1e-3) / 1e9,
                "pct_hbm_peak": 100 * nb / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, "buffers_cycled": copies,
                "note": "back-to-back launches incl. host call overhead; buffers cycled to exceed the last-level cache"}
        out["per_config"] = extra
        out["steady_state"] = steady_state(v, W, torch)
        for r in out["steady_state"].values():
            r["pct_of_measured_store_ceiling"] = 100 * r["gb_per_s"] / ceil["store_only_gb_per_s"]
            r["pct_of_measured_generator_ceiling"] = 100 * (r["gsamples_per_s"] / 4) / ceil["philox_only_gblocks_per_s"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
