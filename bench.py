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

Besides the headline the line carries, per workload config C1..C5, a roofline block built from
ceilings MEASURED IN THE SAME RUN (plain store / copy / traffic-pattern kernels, the generator
alone, and the issue rate of every instruction class the kernels are made of), steady-state rates
of the operators whose own configs are too small to leave the launch-latency regime, and the CPU
oracle timed on the host's cores.  `--design-choices` instead times every retained design choice
against its alternative (same kernels, one choice flipped) and prints that as one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published peak HBM bandwidth
SETTLE_SECONDS = 0.25        # untimed launches before any timed region: the first tens of milliseconds of GPU
                             # work after an idle period run slower (clocks ramp up)

# Vector-ALU instructions per wavefront of the kernels the workload configs run, by issue class.
# Each lane of a wave produces one unit (4 fp32 or 8 bf16 elements; the staging kernel with the large
# tile: four units, "loop_iterations" passes of its generator loop).  Counts are those of the
# compiler's listing of the kernel (hipcc -S), which for the straight-line kernels is what the
# hardware counter SQ_INSTS_VALU / SQ_WAVES reads (profiles/counters_bench_kernels.txt); for the
# staging kernel the generator classes are the listing's loop body times the passes and the total is
# the counter's.  tests/test_bench_model.py recounts them from a fresh listing.  "other" = everything that
# is neither a Philox product (v_mad_u64_u32), a Philox XOR (v_bitop3_b32) nor a transcendental.
KERNEL_MIX = {
    "aligned normal bf16": {"kernel": "aligned_kernel<2, 1, unsigned int, 1, true>", "unit_elems": 8,
                            "mad_u64_u32": 38, "bitop3_b32": 40, "trans": 16, "other": 56},
    "aligned normal f32": {"kernel": "aligned_kernel<2, 0, unsigned int, 1, true>", "unit_elems": 4,
                           "mad_u64_u32": 19, "bitop3_b32": 20, "trans": 8, "other": 30},
    "aligned dropout bf16": {"kernel": "aligned_kernel<3, 1, unsigned int, 1, true>", "unit_elems": 8,
                             "mad_u64_u32": 38, "bitop3_b32": 40, "trans": 0, "other": 67},
    "aligned uniform f32": {"kernel": "aligned_kernel<1, 0, unsigned int, 0, false>", "unit_elems": 4,
                            "mad_u64_u32": 19, "bitop3_b32": 20, "trans": 0, "other": 24},
    "ragged normal f32": {"kernel": "ragged_kernel<2, 0, unsigned int, 1>", "unit_elems": 4,
                          "mad_u64_u32": 22, "bitop3_b32": 20, "trans": 8, "other": 50},
    "staged normal f32": {"kernel": "tiled_kernel<2, 0, unsigned int, 1, 4, 2>", "unit_elems": 16, "loop_iterations": 4,
                          "mad_u64_u32": 80, "bitop3_b32": 80, "trans": 32, "other": 213},
}
SIMPLE_CLASSES = ["add_u32", "fma_f32", "mul_f32", "cvt_f32_u32", "cvt_pk_bf16_f32", "lshrrev_b32", "mul_lo_u32",
                  "cmp_cndmask_b32"]
TRANS_CLASSES = ["log_f32", "sqrt_f32", "sin_f32", "cos_f32"]


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


def settle(torch, fn, seconds=SETTLE_SECONDS):
    """Runs fn() back to back until `seconds` of wall time have passed (synchronising every few
    launches); returns (launches, seconds)."""
    t0 = time.perf_counter()
    n = 0
    while True:
        for _ in range(8):
            fn()
        n += 8
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if dt >= seconds:
            return n, dt


def burst_seconds(torch, fn, reps):
    """Per-launch seconds of `reps` back-to-back launches between one HIP event pair on the current stream."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def steady_seconds(torch, fn, nbytes, bursts=5):
    """Median over `bursts` bursts (each about 10 ms of launches) after settling by time."""
    settle(torch, fn)
    reps = max(5, int(0.010 / max(nbytes / 5e12, 2e-6)))
    return sorted(burst_seconds(torch, fn, reps) for _ in range(bursts))[bursts // 2], reps


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
    """Per-launch milliseconds of `reps` back-to-back launches replayed from a captured HIP graph: the
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
    settle(torch, graph.replay, 0.1)
    times = []
    for _ in range(7):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        graph.replay()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) / reps)
    return sorted(times)[len(times) // 2]


def measured_clock(B, torch):
    """Shader clock under load from the two on-chip counters (shader ticks / constant-rate wall ticks)."""
    wall_khz = B.vesrng_bench_device_info()[4]
    ticks = torch.zeros(4, dtype=torch.int64, device="cuda")
    best = 0.0
    for _ in range(3):
        B.vesrng_bench_clock(200000, ticks)
        torch.cuda.synchronize()
        t = ticks.cpu().tolist()
        if t[1] > 0:
            best = max(best, t[0] / t[1] * wall_khz * 1e3)
    return best


def measured_ceilings(B, torch):
    """Rates of the plain probe kernels on this machine, in this run: what bare 128-bit stores (aligned and
    element-aligned), a 16-byte copy, the dropout kernel's access pattern without arithmetic, the generator
    alone and every instruction class can reach.  1 GiB buffers (beyond the 256 MB last-level cache)."""
    nbytes = 1 << 30
    units = nbytes // 16
    a = torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    m = torch.empty(nbytes // 8, dtype=torch.int32, device="cuda")
    blocks = 1 << 30

    def rate(fn, work):
        return work / steady_seconds(torch, fn, nbytes)[0] / 1e9

    out = {"store_only_gb_per_s": rate(lambda: B.vesrng_bench_probe(B.PROBE_STORE, units, None, a), nbytes),
           "store_unaligned_gb_per_s": rate(lambda: B.vesrng_bench_probe(B.PROBE_STORE_UNALIGNED, units, None, a), nbytes),
           "copy_gb_per_s": rate(lambda: B.vesrng_bench_probe(B.PROBE_COPY, units, a, b), 2 * nbytes),
           # The dropout kernel's loads and stores without its arithmetic, launched as the library launches large
           # masked dropout (at most seven resident waves per SIMD), and at the hardware's eight.
           "dropout_traffic_gb_per_s": rate(lambda: B.vesrng_bench_probe(B.PROBE_DROPOUT_TRAFFIC_7_WAVES, units, a, b, m), 2.5 * nbytes),
           "dropout_traffic_8_waves_gb_per_s": rate(lambda: B.vesrng_bench_probe(B.PROBE_DROPOUT_TRAFFIC, units, a, b, m), 2.5 * nbytes),
           "philox_only_gblocks_per_s": rate(lambda: B.vesrng_bench_probe(B.PROBE_PHILOX, blocks, None, a), blocks)}
    # Issue rates: cycles a SIMD needs per wave-instruction of each class, 16 workgroups per compute unit.
    cus, sclk_khz = B.vesrng_bench_device_info()[:2]
    clock_hz = measured_clock(B, torch) or sclk_khz * 1e3
    wgs, iters = cus * 16, 1000
    cycles = {}
    for cls, name in enumerate(B.ALU_CLASSES):
        secs = steady_seconds(torch, lambda: B.vesrng_bench_alu(cls, wgs, iters, a), 1 << 34, bursts=3)[0]
        per_simd = wgs * 4 * iters * 64 * (2 if name == "cmp_cndmask_b32" else 1) / (cus * 4)
        cycles[name] = secs * clock_hz / per_simd
    out["shader_clock_mhz_measured"] = clock_hz / 1e6
    out["issue_cycles_per_wave_instruction"] = cycles
    out["note"] = ("plain kernels of libvesrng_bench.so (vesrng_bench_probe / vesrng_bench_alu), medians of 5 bursts of about "
                   "10 ms each in this run; issue cycles are per SIMD at the measured shader clock")
    return out


def issue_model_seconds(mix, units, ceil, cus):
    """Time the vector ALUs need to issue a kernel's instructions: per wave, every class's count times its
    measured issue cycles; waves spread over all SIMDs; at the measured shader clock."""
    cyc = ceil["issue_cycles_per_wave_instruction"]
    simple = sum(cyc[c] for c in SIMPLE_CLASSES) / len(SIMPLE_CLASSES)
    trans = sum(cyc[c] for c in TRANS_CLASSES) / len(TRANS_CLASSES)
    per_wave = (mix["mad_u64_u32"] * cyc["mad_u64_u32"] + mix["bitop3_b32"] * cyc["bitop3_b32"]
                + mix["trans"] * trans + mix["other"] * simple)
    waves = (units + 63) // 64
    return waves / (cus * 4) * per_wave / (ceil["shader_clock_mhz_measured"] * 1e6), per_wave


def roofline_block(op, kernel_tag, nbytes, numel, seconds, floor_s, ceil, cus, ragged=False):
    """Per-config roofline: achieved GB/s against the HBM peak, and against a model
    t = launch floor + max(memory time at the measured ceiling of the kernel's own store / traffic
    form, issue time of its instruction mix); `bound` names the largest of the three terms."""
    mix = KERNEL_MIX[kernel_tag]
    units = (numel + mix["unit_elems"] - 1) // mix["unit_elems"]
    # Masked dropout runs at seven resident waves per SIMD from 2^23 units on, at the hardware's eight below.
    traffic = "dropout_traffic_gb_per_s" if units >= (1 << 23) else "dropout_traffic_8_waves_gb_per_s"
    mem_ceiling = (ceil[traffic] if op == "dropout"
                   else ceil["store_unaligned_gb_per_s"] if ragged else ceil["store_only_gb_per_s"])
    t_mem = nbytes / (mem_ceiling * 1e9)
    t_alu, per_wave = issue_model_seconds(mix, units, ceil, cus)
    terms = {"launch": floor_s, "hbm" if not ragged else "store-alignment": t_mem, "alu": t_alu}
    bound = max(terms, key=terms.get)
    t_model = floor_s + max(t_mem, t_alu)
    achieved = nbytes / seconds / 1e9
    return {"bound": bound, "kernel": "vesrng::" + mix["kernel"], "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "kernel_us": seconds * 1e6,
            "model_us": {"launch_floor": floor_s * 1e6, "memory_at_measured_ceiling": t_mem * 1e6, "alu_issue": t_alu * 1e6,
                         "total": t_model * 1e6},
            "memory_ceiling_gb_per_s": mem_ceiling, "issue_cycles_per_wave": per_wave,
            "frac_of_model": t_model / seconds,
            "frac_of_measured_memory_ceiling": achieved / mem_ceiling,
            "frac_of_measured_issue_model": t_alu / seconds}


def steady_state(v, W, torch, ceil, cus):
    """The operators of the small configs at 64x the shard (same shapes of run), where launch latency
    no longer dominates: C2's ragged fp32 normal fill (at this size the kernel without staging; C2 itself,
    below 2^24 elements, is staged) and C3's bf16 normal fill, each against its measured ceilings; and the
    virtual-thread layout on an unsharded tensor."""
    import copy
    res = {}
    for wl, tag, ragged in ((W.C2, "ragged normal f32", True), (W.C3, "aligned normal bf16", False)):
        big = copy.deepcopy(wl)
        big.global_shape = list(wl.global_shape)
        big.global_shape[0] *= 64
        launch, numel, nb = make_launcher(v, W, torch, big, wl.bench_coord, 1)
        secs, reps = steady_seconds(torch, lambda: launch(0), nb)
        r = {"workload": "%s with dim 0 x64 (beyond the 256 MB last-level cache): shard of %d elements" % (wl.name, numel),
             "launches_per_burst": reps, "gb_per_s": nb / secs / 1e9, "pct_hbm_peak": 100 * nb / secs / 1e9 / HBM_PEAK_GBS,
             "gsamples_per_s": numel / secs / 1e9,
             "roofline": roofline_block(wl.op, tag, nb, numel, secs, 0.0, ceil, cus, ragged=ragged)}
        r["pct_of_measured_store_ceiling"] = 100 * r["gb_per_s"] / ceil["store_only_gb_per_s"]
        r["pct_of_measured_generator_ceiling"] = 100 * (r["gsamples_per_s"] / 4) / ceil["philox_only_gblocks_per_s"]
        res[wl.name.split()[0] + "x64"] = r
    n = 1 << 28
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    for theta in (1 << 20, 0):
        sh = v.Sharding([n], [1], [("R",)], [0], None, theta)
        secs, reps = steady_seconds(torch, lambda: v.vesrng_uniform(sh, v.F32, 0.0, 1.0, 1, 0, out), 4 * n)
        res["uniform_f32_2^28_theta_%d" % theta] = {
            "workload": "fp32 uniform fill of an unsharded 2^28-element tensor, " +
                        ("Algorithm 1's virtual-thread layout with 2^20 threads" if theta else "flat stream"),
            "gb_per_s": 4 * n / secs / 1e9, "pct_hbm_peak": 100 * 4 * n / secs / 1e9 / HBM_PEAK_GBS}
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


def counters_pass(v, W, torch):
    """A lean pass for hardware-counter collection (rocprofv3 --pmc): every kernel the benchmark times is
    launched a few times, eagerly and one after the other - no graph replay, no settling loops, no probes -
    and the launches are listed in order, so that a counter row can be matched to its workload by kernel name
    and grid size."""
    import copy
    log = []

    def run(label, fn, times=3):
        for _ in range(times):
            fn()
        torch.cuda.synchronize()
        log.append({"workload": label, "launches": times})

    for wl in (W.C1, W.C2, W.C3, W.C4, W.C5, W.C5_INTERLEAVED):
        launch, numel, nb = make_launcher(v, W, torch, wl, wl.bench_coord, 1)
        run("%s: %d elements, %d algorithmic bytes" % (wl.name, numel, nb), lambda: launch(0), 5 if wl is W.C5 else 3)
        del launch
    for wl in (W.C2, W.C3):
        big = copy.deepcopy(wl)
        big.global_shape = list(wl.global_shape)
        big.global_shape[0] *= 64
        launch, numel, nb = make_launcher(v, W, torch, big, wl.bench_coord, 1)
        run("%s x64: %d elements, %d algorithmic bytes" % (wl.name.split()[0], numel, nb), lambda: launch(0))
        del launch
    n = 1 << 28
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    for theta in (1 << 20, 0):
        sh = v.Sharding([n], [1], [("R",)], [0], None, theta)
        run("fp32 uniform fill of 2^28 elements, virtual threads = %d" % theta,
            lambda: v.vesrng_uniform(sh, v.F32, 0.0, 1.0, 1, 0, out))
    return log


# ---------------------------------------------------------------- design choices ----
def design_choices(v, B, W, torch, once=False):
    """Every design choice the kernels kept, timed against its alternative in this run: the same
    kernels with one choice flipped (the variant libraries), or the plain probe kernels.  Per entry:
    median microseconds per launch of 5 bursts, after settling, and GB/s of algorithmic bytes."""
    res = {}

    def entry(name, choice, cases):
        rows = {}
        for label, fn, nbytes in cases:
            if once:      # counter collection: three eager launches, nothing timed
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                rows[label] = {"launches": 3}
                continue
            secs, reps = steady_seconds(torch, fn, nbytes)
            rows[label] = {"us_per_launch": secs * 1e6, "gb_per_s": nbytes / secs / 1e9, "launches_per_burst": reps}
        res[name] = {"choice": choice, "measured": rows}

    nbytes = 1 << 30
    units = nbytes // 16
    a = torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    m = torch.empty(nbytes // 8, dtype=torch.int32, device="cuda")
    probe = B.vesrng_bench_probe
    entry("launch shape", "one 16-byte unit per thread, one-shot grid",
          [("one-shot (kept)", lambda: probe(B.PROBE_STORE, units, None, a), nbytes),
           ("grid-stride loop, 8 workgroups per CU", lambda: probe(B.PROBE_STORE_GRID_STRIDE, units, None, a), nbytes),
           ("four units per thread", lambda: probe(B.PROBE_STORE_4_PER_THREAD, units, None, a), nbytes)])
    entry("store cache-control bits (store only)", "global_store_dwordx4 sc1 nt",
          [("sc1 nt (kept)", lambda: probe(B.PROBE_STORE, units, None, a), nbytes),
           ("nt", lambda: probe(B.PROBE_STORE_NT, units, None, a), nbytes),
           ("plain", lambda: probe(B.PROBE_STORE_PLAIN, units, None, a), nbytes),
           ("nt, element-aligned addresses", lambda: probe(B.PROBE_STORE_UNALIGNED, units, None, a), nbytes)])
    entry("dropout traffic pattern: store bits, load bits, mask store width",
          "non-temporal loads, sc1 nt stores, 8 mask bytes per thread",
          [("nt loads, sc1 nt stores, 8-byte mask stores (kept)", lambda: probe(B.PROBE_DROPOUT_TRAFFIC, units, a, b, m), 2.5 * nbytes),
           ("nt stores", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_NT, units, a, b, m), 2.5 * nbytes),
           ("ordinary loads", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_LOAD_PLAIN, units, a, b, m), 2.5 * nbytes),
           ("sc1 nt loads", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_LOAD_SC1, units, a, b, m), 2.5 * nbytes),
           ("sc0 sc1 loads", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_LOAD_SC0SC1, units, a, b, m), 2.5 * nbytes),
           ("two units per thread, 16-byte mask stores", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_WIDE_MASK, units, a, b, m), 2.5 * nbytes),
           ("kept pattern, at most seven resident waves per SIMD", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_7_WAVES, units, a, b, m), 2.5 * nbytes),
           ("kept pattern, at most six", lambda: probe(B.PROBE_DROPOUT_TRAFFIC_6_WAVES, units, a, b, m), 2.5 * nbytes)])
    blocks = 1 << 30
    entry("three-way XOR of the generator (generator only)", "v_bitop3_b32",
          [("v_bitop3_b32 (kept)", lambda: probe(B.PROBE_PHILOX, blocks, None, a), blocks * 16),
           ("two v_xor_b32", lambda: probe(B.PROBE_PHILOX_TWO_XOR, blocks, None, a), blocks * 16)])
    del a, b, m

    variants = {k: B.Variant(k) for k in ("nopin", "ntstore", "twoxor", "lanerun", "ragged", "realign", "smalltile", "bigtile", "wavetile", "longmap", "nocap", "widekernels", "loopaxes", "pairint")}
    # Aligned kernels: C5's dropout shard, a 2^28-element fp32 uniform fill, C3 x64 (bf16 normal).
    w = W.C5
    sh5 = v.Sharding(*w.sharding_args(w.bench_coord))
    shape, n5 = v.vesrng_local_shape(sh5)
    x = W.device_activations(shape, w.input_seed, w.input_kind, w.dtype).reshape(-1)
    y = torch.empty_like(x)
    mask = torch.empty(n5, dtype=torch.uint8, device="cuda")
    drop = lambda L: (lambda: L.vesrng_dropout(sh5, v.BF16, 0.1, 1234, 0, x, y, mask))
    entry("C5 fused dropout: argument-fetch pinning, store bits, resident waves", "pinned, sc1 nt, at most seven waves per SIMD",
          [("library (kept)", drop(v), 5 * n5), ("without the pinning", drop(variants["nopin"]), 5 * n5),
           ("plain non-temporal stores", drop(variants["ntstore"]), 5 * n5),
           ("eight resident waves per SIMD (no cap)", drop(variants["nocap"]), 5 * n5)])
    del x, y, mask
    n = 1 << 28
    shu = v.Sharding([n], [1], [("R",)], [0])
    o = torch.empty(n, dtype=torch.float32, device="cuda")
    uni = lambda L: (lambda: L.vesrng_uniform(shu, v.F32, 0.0, 1.0, 1, 0, o))
    entry("aligned fp32 uniform fill (2^28 elements): argument-fetch pinning, store bits", "pinned, sc1 nt",
          [("library (kept)", uni(v), 4 * n), ("without the pinning", uni(variants["nopin"]), 4 * n),
           ("plain non-temporal stores", uni(variants["ntstore"]), 4 * n)])
    sh3 = v.Sharding([4096 * 64, 14336], [2, 4], [("S", 0), ("S", 1)], [1, 2])
    n3 = v.vesrng_local_shape(sh3)[1]
    ob = torch.empty(n3, dtype=torch.bfloat16, device="cuda")
    nrm = lambda L: (lambda: L.vesrng_normal(sh3, v.BF16, 0.0, 0.02, 3, 0, ob))
    entry("C3 x64 bf16 normal fill: three-way XOR, run arithmetic", "v_bitop3_b32; run arithmetic once per wave in scalar registers",
          [("library (kept)", nrm(v), 2 * n3), ("two v_xor_b32", nrm(variants["twoxor"]), 2 * n3),
           ("run arithmetic per lane", nrm(variants["lanerun"]), 2 * n3)])
    del ob
    of3 = torch.empty(n3, dtype=torch.float32, device="cuda")
    nrm32 = lambda L: (lambda: L.vesrng_normal(sh3, v.F32, 0.0, 0.02, 3, 0, of3))
    entry("fp32 normal fill on C3 x64's shard: run arithmetic", "once per wave in scalar registers",
          [("library (kept)", nrm32(v), 4 * n3), ("run arithmetic per lane", nrm32(variants["lanerun"]), 4 * n3)])
    del of3
    # The pinning is about the latency of a workgroup's life: it shows on the small configs (GPU-side time per
    # launch, replayed from a HIP graph), not on shards that keep the chip busy for hundreds of microseconds.
    for wl, copies in ((W.C1, 256), (W.C3, 32), (W.C4, 8)):
        rows = {}
        for label, lib in (("library (kept)", v), ("without the pinning", variants["nopin"])):
            launch, numel, nb = make_launcher(lib, W, torch, wl, wl.bench_coord, 1 if once else copies)
            if once:
                for k in range(3):
                    launch(k)
                torch.cuda.synchronize()
                rows[label] = {"launches": 3}
                continue
            ms = sorted(time_graph(torch, launch, 4 * copies) for _ in range(3))[1]
            rows[label] = {"us_per_launch": ms * 1e3, "gb_per_s": nb / (ms * 1e-3) / 1e9, "launches_per_burst": 4 * copies}
        res["%s (graph replay): argument-fetch pinning" % wl.name.split()[0]] = {"choice": "pinned", "measured": rows}
    # Ragged column shards [rows, 4096] cut three ways (C2's shape of run): C2 itself and two larger sizes.  C2's own
    # shard takes a few microseconds: it is timed as the per-config blocks time it, GPU-side from a HIP-graph replay
    # over buffers that together exceed the last-level cache.
    def entry_graph(name, choice, cases, copies):
        rows = {}
        for label, fn, nbytes in cases:
            if once:
                for k in range(3):
                    fn(k)
                torch.cuda.synchronize()
                rows[label] = {"launches": 3}
                continue
            ms = sorted(time_graph(torch, fn, 4 * copies) for _ in range(3))[1]
            rows[label] = {"us_per_launch": ms * 1e3, "gb_per_s": nbytes / (ms * 1e-3) / 1e9, "launches_per_burst": 4 * copies}
        res[name + " (graph replay)"] = {"choice": choice, "measured": rows}

    for rows in (4096, 16384, 98304):
        shr = v.Sharding([rows, 4096], [3], [("S", 1)], [1])
        nr = v.vesrng_local_shape(shr)[1]
        copies = 32 if rows == 4096 else 1
        ofs = [o[k * nr:(k + 1) * nr] for k in range(copies)]
        ois = [t.view(torch.int32) for t in ofs]
        obs = [t.view(torch.bfloat16)[:nr] for t in ofs]
        for op, call, bpe in (("raw", lambda L: (lambda k=0: L.vesrng_raw_u32(shr, 1, 0, ois[k % copies])), 4),
                              ("fp32 uniform", lambda L: (lambda k=0: L.vesrng_uniform(shr, v.F32, 0.0, 1.0, 1, 0, ofs[k % copies])), 4),
                              ("fp32 normal", lambda L: (lambda k=0: L.vesrng_normal(shr, v.F32, 0.0, 1.0, 1, 0, ofs[k % copies])), 4),
                              ("bf16 uniform", lambda L: (lambda k=0: L.vesrng_uniform(shr, v.BF16, 0.0, 1.0, 1, 0, obs[k % copies])), 2)):
            if bpe == 2:
                name, choice = ("ragged %s fill, %d elements" % (op, nr),
                                "staged (small tile) from 2^21 to 2^25 elements with runs of 256 and more, else no staging")
                cases = [("library (kept)", call(v), 2 * nr), ("no staging", call(variants["ragged"]), 2 * nr),
                         ("staged, small tile", call(variants["smalltile"]), 2 * nr)]
            else:
                name, choice = ("ragged %s fill, %d elements" % (op, nr),
                                "raw and uniform: small tile below 2^22 elements, large tile from there; "
                                "normal: the same below 2^24 elements, no staging above")
                cases = [("library (kept)", call(v), 4 * nr),
                         ("no staging, element-aligned stores", call(variants["ragged"]), 4 * nr),
                         ("no staging, realigned across lanes (DPP)", call(variants["realign"]), 4 * nr),
                         ("staged, small tile", call(variants["smalltile"]), 4 * nr),
                         ("staged, large tile", call(variants["bigtile"]), 4 * nr),
                         ("library's choice with the tile map per wavefront (scalar)", call(variants["wavetile"]), 4 * nr),
                         ("library's choice with the general form of the tile map", call(variants["longmap"]), 4 * nr)]
            if copies > 1:
                entry_graph(name, choice, cases, copies)
            else:
                entry(name, choice, cases)
        # Fused bf16 dropout on the same shard (small tile): 5 bytes per element.
        xr = torch.randn(nr, dtype=torch.float32, device="cuda").to(torch.bfloat16)
        orr = torch.empty_like(xr)
        mr = torch.empty(nr, dtype=torch.uint8, device="cuda")
        drop = lambda L: (lambda: L.vesrng_dropout(shr, v.BF16, 0.1, 1, 0, xr, orr, mr))
        entry("ragged bf16 dropout, %d elements" % nr, "staged, short form of the tile map",
              [("library (kept)", drop(v), 5 * nr), ("general form of the tile map", drop(variants["longmap"]), 5 * nr),
               ("no staging", drop(variants["ragged"]), 5 * nr)])
        del xr, orr, mr
    # Shards of 2^30 elements and more: piece by piece through the 32-bit kernels against the 64-bit kernels.
    del o
    wide_out = torch.empty(1 << 31, dtype=torch.float32, device="cuda")
    for shape, what in (([1 << 17, 1 << 15], "aligned runs of 16384 elements, 2^31 elements"),
                        ([1 << 24, 200], "aligned runs of 100 elements, 1.68e9 elements"),
                        ([1 << 19, 4099], "ragged runs of 2049 elements, 1.07e9 elements")):
        shw = v.Sharding(shape, [2], [("S", 1)], [1])
        nw = v.vesrng_local_shape(shw)[1]
        wf = wide_out[:nw]
        wb = wide_out.view(torch.bfloat16)[:nw]
        entry("fp32 uniform fill, " + what, "piece by piece through the 32-bit kernels",
              [("library (kept)", lambda: v.vesrng_uniform(shw, v.F32, 0.0, 1.0, 1, 0, wf), 4 * nw),
               ("64-bit index kernels", lambda: variants["widekernels"].vesrng_uniform(shw, v.F32, 0.0, 1.0, 1, 0, wf), 4 * nw)])
        entry("bf16 normal fill, " + what, "piece by piece through the 32-bit kernels",
              [("library (kept)", lambda: v.vesrng_normal(shw, v.BF16, 0.0, 1.0, 1, 0, wb), 2 * nw),
               ("64-bit index kernels", lambda: variants["widekernels"].vesrng_normal(shw, v.BF16, 0.0, 1.0, 1, 0, wb), 2 * nw)])
    # Double-sharded tensors: two and three axes of runs (Table 5's grid), run arithmetic written out against the loop.
    xa = torch.randn(1 << 27, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    ma = torch.empty(1 << 27, dtype=torch.uint8, device="cuda")
    for shape, mesh, pls, what in (([256, 256, 8192], [2, 2], [("S", 1), ("S", 2)], "two axes of runs of 4096 elements"),
                                   ([16, 32, 128, 8192], [2, 2, 2], [("S", 1), ("S", 2), ("S", 3)], "three axes of runs of 4096 elements"),
                                   ([64, 128, 512, 200], [2, 2, 2], [("S", 1), ("S", 2), ("S", 3)], "three axes of runs of 100 elements")):
        sha = v.Sharding(shape, mesh, pls, [1] * len(mesh))
        na = v.vesrng_local_shape(sha)[1]
        af = wide_out[:na]
        ab = wide_out.view(torch.bfloat16)[:na]
        entry("fp32 uniform fill, %s, %d elements" % (what, na), "run arithmetic written out for two and three axes",
              [("library (kept)", lambda: v.vesrng_uniform(sha, v.F32, 0.0, 1.0, 1, 0, af), 4 * na),
               ("loop over the axes", lambda: variants["loopaxes"].vesrng_uniform(sha, v.F32, 0.0, 1.0, 1, 0, af), 4 * na)])
        entry("bf16 dropout, %s, %d elements" % (what, na), "run arithmetic written out for two and three axes",
              [("library (kept)", lambda: v.vesrng_dropout(sha, v.BF16, 0.1, 1, 0, xa[:na], ab, ma[:na]), 5 * na),
               ("loop over the axes", lambda: variants["loopaxes"].vesrng_dropout(sha, v.BF16, 0.1, 1, 0, xa[:na], ab, ma[:na]), 5 * na)])
    # randint (8 bytes per element): two threads per generator block against one thread with two stores.
    oi64 = wide_out.view(torch.int64)
    for shape, mesh, pls, what in (([1 << 28], [1], [("R",)], "contiguous shard of 2^28 elements"),
                                   ([1 << 15, 8192], [2], [("S", 1)], "runs of 4096 elements, 2^27 elements")):
        shi = v.Sharding(shape, mesh, pls, [p - 1 for p in mesh])
        ni = v.vesrng_local_shape(shi)[1]
        entry("randint fill, " + what, "two threads per generator block, one 16-byte store each",
              [("library (kept)", lambda: v.vesrng_randint(shi, 0, 1000, 1, 0, oi64[:ni]), 8 * ni),
               ("one thread per block, halves traded across lanes, two stores",
                lambda: variants["pairint"].vesrng_randint(shi, 0, 1000, 1, 0, oi64[:ni]), 8 * ni)])
    del wide_out, xa, ma, oi64
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-config side measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known size) to scale rocprofv3's byte counters")
    ap.add_argument("--design-choices", action="store_true",
                    help="time every retained design choice against its alternative instead of the benchmark")
    ap.add_argument("--counters-pass", action="store_true",
                    help="for rocprofv3 --pmc: launch every timed kernel a few times, eagerly, and time nothing "
                         "(with --design-choices: every choice and its alternative)")
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

    if a.design_choices:
        print(json.dumps({"design_choices": design_choices(v, B, W, torch, once=a.counters_pass)}), flush=True)
        return
    if a.counters_pass:
        print(json.dumps({"counters_pass": counters_pass(v, W, torch)}), flush=True)
        return

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

    # Settle by TIME, whatever --warmup says: at least SETTLE_SECONDS of untimed launches come first.
    settle_launches, settle_s = settle(torch, step)
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region: K steps between two HIP events recorded on the launch stream (and between two
    # host clock readings after a synchronise).  No event sits between launches - a pair around each one
    # adds packets that slow the stream - so the kernel's average duration is the events' elapsed time / K:
    # it includes the few hundred nanoseconds between consecutive kernels, i.e. it can only overstate the
    # kernel's own duration (rocprofv3's per-kernel average for the same command is slightly shorter).
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for k in range(a.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / a.steps
    value = nbytes / (wall / a.steps) / 1e9
    avg_ms = e0.elapsed_time(e1) / a.steps
    achieved = nbytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "vesrng::aligned_kernel<3 (dropout), 1 (bf16), unsigned int, 1 run axis, runs of whole waves>",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": read_traffic("c5_dropout_bf16"), "avg_launch_ms": avg_ms,
                "timing": "HIP events on the launch stream around the %d launches of the timed region, elapsed / %d "
                          "(includes the gaps between consecutive kernels)" % (a.steps, a.steps),
                "algorithmic_bytes_per_launch": nbytes}

    out = {"metric": "sharded RNG fill / fused dropout GB/s per MI355X and % of HBM peak", "value": value,
           "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u32 Philox + f32 scale, bf16 in/out, u8 mask", "data": "synthetic",
           "config": {"workload": w.name, "rank": coord, "local_shape": shape, "elements": n,
                      "settle_launches": settle_launches, "settle_seconds": settle_s,
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
        # Vector-ALU peak of this path: every instruction class the kernels use issues one wave-instruction
        # per SIMD every ~4 cycles (16 lanes per cycle; transcendentals every ~8): lanes x clock.
        ceil["valu_peak_lane_ops_per_s"] = cus * 4 * 16 * ceil["shader_clock_mhz_measured"] * 1e6
        roofline["frac_of_measured_traffic_ceiling"] = achieved / ceil["dropout_traffic_gb_per_s"]
        roofline["frac_of_measured_generator_ceiling"] = (n / 4 / (avg_ms * 1e-3) / 1e9) / ceil["philox_only_gblocks_per_s"]
        t_alu, per_wave = issue_model_seconds(KERNEL_MIX["aligned dropout bf16"], n // 8, ceil, cus)
        roofline["frac_of_measured_issue_model"] = t_alu / (avg_ms * 1e-3)
        # Launch floor: graph replay of the same entry point on a shard of one workgroup.
        tiny = v.Sharding([1024], [1], [("R",)], [0])
        tbuf = torch.empty(1024, dtype=torch.float32, device="cuda")
        floor_ms = time_graph(torch, lambda k: v.vesrng_uniform(tiny, v.F32, 0.0, 1.0, 1, 0, tbuf), 64)
        ceil["launch_floor_us"] = floor_ms * 1e3
        extra = {}
        tags = {"C1": ("aligned uniform f32", False), "C2": ("staged normal f32", False), "C3": ("aligned normal bf16", False),
                "C4": ("aligned dropout bf16", False), "C5i": ("aligned dropout bf16", False)}
        for wl, copies in ((W.C1, 256), (W.C2, 16), (W.C3, 32), (W.C4, 8), (W.C5_INTERLEAVED, 1)):
            key = wl.name.split()[0] + ("i" if wl is W.C5_INTERLEAVED else "")
            launch, numel, nb = make_launcher(v, W, torch, wl, wl.bench_coord, copies)
            avg = time_batch(torch, launch, max(50, a.steps), 5)
            per_launch_graph = time_graph(torch, launch, 4 * copies if copies > 1 else 8)
            tag, ragged = tags[key]
            extra[key] = {
                "graph_replay_us_per_launch": per_launch_graph * 1e3,
                "graph_replay_gb_per_s": nb / (per_launch_graph * 1e-3) / 1e9,
                "workload": wl.name, "elements": numel, "algorithmic_bytes": nb, "avg_launch_us": avg * 1e3,
                "gb_per_s": nb / (avg * 1e-3) / 1e9, "gsamples_per_s": numel / (avg * 1e-3) / 1e9,
                "pct_hbm_peak": 100 * nb / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, "buffers_cycled": copies,
                "note": "avg_launch_us: back-to-back launches incl. host call overhead; graph_replay: the same launches "
                        "replayed from a HIP graph (GPU-side time per launch, the roofline block's kernel time); "
                        "buffers cycled to exceed the last-level cache",
                "roofline": roofline_block(wl.op, tag, nb, numel, per_launch_graph * 1e-3, floor_ms * 1e-3, ceil, cus,
                                           ragged=ragged)}
        extra["C5"] = {"workload": w.name, "elements": n, "algorithmic_bytes": nbytes,
                       "roofline": roofline_block("dropout", "aligned dropout bf16", nbytes, n, avg_ms * 1e-3, floor_ms * 1e-3,
                                                  ceil, cus)}
        out["per_config"] = extra
        out["steady_state"] = steady_state(v, W, torch, ceil, cus)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
