#!/usr/bin/env python3
"""Benchmark of the CGBN hot path on one MI355X.

A step is one pass of the whole path -- cgbn_forward then cgbn_backward -- over
one synthetic activation tensor that is already resident in HBM.  The headline
workload is the detector stem level (16 x 64 x 400 x 672, NCHW fp32, K = 8
shards).

`value` is the effective bandwidth on the MINIMUM bytes the step has to move:
every tensor touched once (x read, y written; dy and x read, dx written = 5
tensors) divided by the step time.  No implementation can move fewer bytes, so
the figure cannot exceed what HBM delivers; for the single-launch kernels, which
keep each unit of the tensor in registers and LDS between the reductions and the
elementwise step, it is also what really moves (confirmed by FETCH_SIZE /
WRITE_SIZE, see profiles/).  The byte count of the two-pass method run as
separate sweeps (9 tensors: 3 reads + 1 write forward, 4 reads + 1 write
backward) over the same time is reported beside it as
`two_pass_equivalent_GBps`; it says how fast separate sweeps would have to be
to match, and is not a bandwidth.

Prints ONE JSON line.  `roofline` is for the dominant kernel (the single-launch
backward, or the dx sweep where that path does not apply): the bytes that
launch moves divided by its duration, from HIP events around the backward call
inside timed steps on the stream it is launched on.  `cpu_baseline` is the
float64 oracle timed on this machine's host cores on a sample of channels of
the same workload.
"""

from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_GBPS = 8000.0   # MI355X HBM3E, published
METRIC = "CGBN fwd+bwd ms/layer and effective HBM GB/s (% of MI355X peak), 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """Device buffers of one CGBN layer plus the calls that make up a step."""

    def __init__(self, wl, torch, cgbn, x, dy, gamma, beta):
        self.wl, self.cgbn, self.torch = wl, cgbn, torch
        dev = x.device
        self.x, self.dy, self.gamma, self.beta = x, dy, gamma, beta
        self.y, self.dx = torch.empty_like(x), torch.empty_like(x)
        v = lambda: torch.empty(wl.C, dtype=torch.float32, device=dev)
        self.mean, self.invstd, self.mean_lo, self.dgamma, self.dbeta = v(), v(), v(), v(), v()
        wb = cgbn.cgbn_workspace_bytes(wl.N, wl.C, wl.H, wl.W, wl.layout, wl.dtype, wl.K)
        self.ws = torch.empty(wb, dtype=torch.uint8, device=dev)
        f64 = lambda: torch.empty(wl.K * wl.C, dtype=torch.float64, device=dev)
        self.s, self.v, self.a, self.b = f64(), f64(), f64(), f64()
        self.shape = (wl.N, wl.C, wl.H, wl.W)

    def forward(self):
        wl = self.wl
        self.cgbn.cgbn_forward(self.x, *self.shape, wl.layout, wl.K, self.gamma, self.beta, wl.eps,
                               self.y, self.mean, self.invstd, wl.dtype, self.mean_lo, self.ws)

    def backward(self):
        wl = self.wl
        self.cgbn.cgbn_backward(self.dy, self.x, self.mean, self.invstd, self.gamma, self.dx,
                                self.dgamma, self.dbeta, *self.shape, wl.layout, wl.K, wl.dtype,
                                self.mean_lo, self.ws)

    def step(self):
        self.forward()
        self.backward()

    # the sweeps one at a time (same kernels as the fused entry points)
    def sweeps(self):
        wl, c, sh = self.wl, self.cgbn, self.shape
        M = wl.M
        return {
            "shard_sum": (1, lambda: c.cgbn_shard_sum(self.x, *sh, wl.layout, wl.K, wl.dtype, self.s, self.ws)),
            "shard_sqdev": (1, lambda: c.cgbn_shard_sqdev(self.x, *sh, wl.layout, wl.K, wl.dtype, self.mean,
                                                          self.mean_lo, self.v, self.ws)),
            "normalize": (2, lambda: c.cgbn_normalize(self.x, *sh, wl.layout, wl.dtype, self.mean, self.mean_lo,
                                                      self.invstd, self.gamma, self.beta, self.y)),
            "backward_shard_sums": (2, lambda: c.cgbn_backward_shard_sums(
                self.dy, self.x, *sh, wl.layout, wl.K, wl.dtype, self.mean, self.mean_lo, self.invstd,
                self.a, self.b, self.ws)),
            "backward_dx": (3, lambda: c.cgbn_backward_dx(self.dy, self.x, *sh, wl.layout, wl.dtype, self.mean,
                                                          self.mean_lo, self.invstd, self.gamma, self.dgamma,
                                                          self.dbeta, self.dx)),
        }


def device_inputs_host_recipe(wl, torch, synth, dev):
    d = synth.make_inputs(wl, threads=min(16, os.cpu_count() or 1))
    conv = lambda a: torch.from_numpy(a.view("int16") if a.dtype.name == "uint16" else a).to(dev)
    return conv(d["x"]), conv(d["dy"]), torch.from_numpy(d["gamma"]).to(dev), torch.from_numpy(d["beta"]).to(dev)


def device_inputs_fast(wl, torch, synth, dev):
    """Same distributions drawn on the device (used for the secondary workloads,
    where only timing is taken)."""
    mu, sigma, gamma, beta = (torch.from_numpy(a).to(dev) for a in synth.channel_params(wl))
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed)
    shape = (wl.N, wl.C, wl.H, wl.W) if wl.layout == "NCHW" else (wl.N, wl.H, wl.W, wl.C)
    bs = (1, -1, 1, 1) if wl.layout == "NCHW" else (1, 1, 1, -1)
    x = torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
    x.mul_(sigma.view(bs)).add_(mu.view(bs))
    if wl.x_kind == "relu":
        x.clamp_(min=0)
    dy = torch.randn(shape, generator=g, device=dev, dtype=torch.float32).mul_(wl.dy_sigma)
    if wl.dtype == "bf16":
        x, dy = x.to(torch.bfloat16).view(torch.int16), dy.to(torch.bfloat16).view(torch.int16)
    return x, dy, gamma, beta


def time_calls(torch, fn, warmup, iters):
    """Per-call durations in ms from HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    torch.cuda.synchronize()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in ev]


def time_step_halves(torch, layer, iters):
    """Forward and backward durations (ms) inside whole steps: events before, between and after the two calls."""
    ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(iters)]
    torch.cuda.synchronize()
    for a, b, c in ev:
        a.record()
        layer.forward()
        b.record()
        layer.backward()
        c.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b, _ in ev], [b.elapsed_time(c) for _, b, c in ev]


def measure_workload(layer, torch, steps, warmup):
    """Times K steps back to back (ms_per_step: wall clock between two synchronisations, no events inside),
    then the same steps again with events between the two calls."""
    wl = layer.wl
    Sb = wl.S * wl.elem_bytes
    for _ in range(warmup):
        layer.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        layer.step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    fwd_in, bwd_in = time_step_halves(torch, layer, steps)
    per_step = [f + b for f, b in zip(fwd_in, bwd_in)]
    fused_f, fused_b = (layer.cgbn.cgbn_get_tuning("last_forward_fused"), layer.cgbn.cgbn_get_tuning("last_backward_fused"))
    # bytes the step moves by design: 5 tensors when both directions run as one launch each; as separate sweeps
    # the forward moves 3 (statistics from one sweep over x, the default) or 4, the backward 5
    one_sweep = layer.cgbn.cgbn_get_tuning("one_sweep_stats")
    moved = ((2 if fused_f else (3 if one_sweep else 4)) + (3 if fused_b else 5)) * Sb
    return dict(
        workload=wl.name, ms_per_step=wall_ms, fwd_ms=statistics.median(fwd_in), bwd_ms=statistics.median(bwd_in),
        bwd_ms_mean=statistics.mean(bwd_in),
        step_ms_median=statistics.median(per_step), step_ms_min=min(per_step), step_ms_max=max(per_step),
        single_launch=dict(forward=fused_f, backward=fused_b),
        min_bytes=5 * Sb, min_bytes_GBps=5 * Sb / wall_ms / 1e6,
        pct_of_peak_on_min_bytes=5 * Sb / wall_ms / 1e6 / PEAK_GBPS * 100,
        moved_bytes_by_design=moved, moved_GBps=moved / wall_ms / 1e6,
        pct_of_peak_on_moved_bytes=moved / wall_ms / 1e6 / PEAK_GBPS * 100,
        two_pass_equivalent_GBps=9 * Sb / wall_ms / 1e6,
        fwd_min_bytes_GBps=2 * Sb / statistics.median(fwd_in) / 1e6,
        bwd_min_bytes_GBps=3 * Sb / statistics.median(bwd_in) / 1e6)


def measure_rotating(layer, torch, cgbn, steps, sets=4):
    """ms per step when consecutive steps work on different buffer sets, so that
    nothing a step left in the memory-side cache serves the next one."""
    wl = layer.wl
    layers = [layer] + [Layer(wl, torch, cgbn, layer.x.clone(), layer.dy.clone(), layer.gamma, layer.beta)
                        for _ in range(sets - 1)]
    for l in layers:
        l.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        layers[i % sets].step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def measure_graph(layer, torch, steps):
    """ms per step when forward + backward are captured once into a HIP graph and replayed:
    what a launch-latency-bound shape costs without the per-launch host work."""
    layer.step()
    torch.cuda.synchronize()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        layer.step()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def cpu_baseline(wl, synth, budget_s=12.0):
    """The float64 oracle (plain definition, forward + backward) on host cores,
    on channels of the same workload, sized to about `budget_s` seconds."""
    from oracle import cgbn_oracle as O
    workers = max(1, min(16, os.cpu_count() or 1))
    per = wl.M * wl.elem_bytes * 9

    def draw(c):
        d = synth.make_inputs(wl, channels=[c], threads=1)
        if wl.dtype == "bf16":
            d["x"], d["dy"] = O.bf16_bits_to_f64(d["x"]), O.bf16_bits_to_f64(d["dy"])
        return d

    def run(d):
        O.cgbn_forward_backward_ref(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout)

    d0 = draw(0)
    t = time.perf_counter()
    run(d0)                                             # one channel alone: sizes the sample
    t_one = time.perf_counter() - t
    rounds = max(1, min(wl.C // workers, int(budget_s / max(t_one, 1e-3))))
    chans = list(range(workers * rounds))
    # when the whole layer is too little work, go over its channels more than once (>= ~10 s of CPU work)
    reps = max(1, min(8, int(-(-10.0 // max(t_one * len(chans), 1e-3)))))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        inputs = list(ex.map(draw, chans))              # untimed
        t = time.perf_counter()
        for _ in range(reps):
            list(ex.map(run, inputs))
        wall = (time.perf_counter() - t) / reps
    return dict(value=per * len(chans) / wall / 1e9, unit="GB/s", cores=workers, kind="oracle",
                sample=f"{len(chans)} of {wl.C} channels of {wl.name}, forward+backward, float64 numpy, "
                       f"{workers} threads with one channel each, {reps} pass(es), {wall:.2f} s wall per pass",
                ms_per_layer_extrapolated=wall / len(chans) * wl.C * 1e3)


def load_traffic(name):
    """Measured HBM bytes per launch of the dominant kernel, from the committed
    rocprofv3 counter summary (profiles/traffic.txt: `name bytes` lines), or None."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split("#", 1)[0].split()
                if len(parts) == 2 and parts[0] == name:
                    return float(parts[1])
    except (OSError, ValueError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--others", default="cfg0,cfg2,cfg3,cfg4,cfg4b", help="secondary workloads timed with fewer steps ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the library's plain copy kernel over 1 GiB (for counter calibration under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the K shards are virtual devices on it); "
                 "--gpus N with N > 1 is not supported")

    import torch
    from paper_1711_07240_amd import cgbn, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cgbn.lib()                       # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = synth.WORKLOADS[args.workload]
    log(f"[bench] drawing {wl.name} on the host ({wl.S} elements x 2)")
    x, dy, gamma, beta = device_inputs_host_recipe(wl, torch, synth, dev)
    layer = Layer(wl, torch, cgbn, x, dy, gamma, beta)
    log("[bench] timing the step")
    head = measure_workload(layer, torch, args.steps, args.warmup)

    # the sweeps one at a time (the multi-sweep path's kernels), each on the bytes it moves
    Sb = wl.S * wl.elem_bytes
    sweeps = {}
    for name, (ntensors, fn) in layer.sweeps().items():
        ms = time_calls(torch, fn, 3, max(10, args.steps // 2))
        sweeps[name] = dict(ms=statistics.mean(ms), GBps=ntensors * Sb / statistics.mean(ms) / 1e6)
    if head["single_launch"]["backward"] == 1:
        # The backward is one launch that holds dy and x in registers and LDS between the device sums and
        # dx: it reads dy and x once and writes dx once, 3 tensors (`traffic`: what the counters saw move).
        # Its duration: the backward half of the timed steps (the launch itself plus the few-microsecond
        # launch that prepares its rows).  Separate sweeps would move 5 tensors for the same work; that
        # count over this time is kept as a comparison figure, it is not a bandwidth.
        ms = head["bwd_ms_mean"]
        roofline = dict(bound="hbm", kernel="nchw_fused_backward", achieved=3 * Sb / ms / 1e6, peak=PEAK_GBPS,
                        unit="GB/s", frac=3 * Sb / ms / 1e6 / PEAK_GBPS,
                        traffic=load_traffic(f"{wl.name}.nchw_fused_backward"), avg_ms=ms,
                        moved_bytes_by_design=3 * Sb,
                        two_sweep_equivalent_GBps=5 * Sb / ms / 1e6)
    else:
        dom = "backward_dx"
        roofline = dict(bound="hbm", kernel=dom, achieved=sweeps[dom]["GBps"], peak=PEAK_GBPS, unit="GB/s",
                        frac=sweeps[dom]["GBps"] / PEAK_GBPS, traffic=load_traffic(f"{wl.name}.{dom}"),
                        avg_ms=sweeps[dom]["ms"], moved_bytes_by_design=3 * Sb)

    # fixed-statistics mode on the same tensors: one sweep each way, 2*S*b bytes per launch
    fv = layer.invstd.double().pow(-2).float()                      # variances of the right size for this data
    frozen = {}
    for name, fn in (("frozen_forward", lambda: cgbn.cgbn_frozen_forward(
                          layer.x, *layer.shape, wl.layout, wl.dtype, layer.mean, fv, layer.gamma, layer.beta, wl.eps, layer.y)),
                     ("frozen_backward", lambda: cgbn.cgbn_frozen_backward(
                          layer.dy, *layer.shape, wl.layout, wl.dtype, fv, layer.gamma, wl.eps, layer.dx))):
        ms = statistics.mean(time_calls(torch, fn, 3, max(10, args.steps // 2)))
        frozen[name] = dict(ms=ms, GBps=2 * Sb / ms / 1e6, frac_of_peak=2 * Sb / ms / 1e6 / PEAK_GBPS)

    # CGBN + shortcut add + ReLU on the same tensors (y doubles as the stored output the backward masks by)
    relu = {}
    shortcut = layer.dy                                              # any tensor of the right shape
    dz = torch.empty_like(layer.x)
    for name, sc, dsc in (("relu", None, None), ("add_relu", shortcut, dz)):
        fw = lambda: cgbn.cgbn_forward_relu(layer.x, sc, *layer.shape, wl.layout, wl.K, layer.gamma, layer.beta, wl.eps,
                                            layer.y, layer.mean, layer.invstd, wl.dtype, layer.mean_lo, layer.ws)
        bw = lambda: cgbn.cgbn_backward_relu(layer.dy, layer.y, layer.x, layer.mean, layer.invstd, layer.gamma, layer.dx,
                                             dsc, layer.dgamma, layer.dbeta, *layer.shape, wl.layout, wl.K, wl.dtype,
                                             layer.mean_lo, layer.ws)
        fms = statistics.median(time_calls(torch, fw, 3, max(10, args.steps // 2)))
        bms = statistics.median(time_calls(torch, bw, 3, max(10, args.steps // 2)))
        moved_f, moved_b = (3 if sc is not None else 2), (5 if dsc is not None else 4)
        relu[name] = dict(fwd_ms=fms, bwd_ms=bms, fwd_moved_GBps=moved_f * Sb / fms / 1e6, bwd_moved_GBps=moved_b * Sb / bms / 1e6,
                          single_launch=dict(forward=cgbn.cgbn_get_tuning("last_forward_fused"),
                                             backward=cgbn.cgbn_get_tuning("last_backward_fused")))
    del dz

    # What this machine's memory system gives a plain streaming copy (the library's copy kernel, 1 GiB read + 1 GiB
    # written): context for the figures above, which mix reads and writes the same way.  Under rocprofv3 the same
    # launches calibrate the traffic counters (`--calibrate` is kept for the profile commands; it changes nothing).
    nb = 1 << 30
    a, b = torch.empty(nb, dtype=torch.uint8, device=dev), torch.empty(nb, dtype=torch.uint8, device=dev)
    copy_ms = statistics.median(time_calls(torch, lambda: cgbn.cgbn_calibration_copy(a, b, nb), 3, 10))
    streaming_copy = dict(ms=copy_ms, GBps=2 * nb / copy_ms / 1e6, frac_of_peak=2 * nb / copy_ms / 1e6 / PEAK_GBPS,
                          bytes_moved=2 * nb, kernel="calibration_copy (16-byte loads and stores, 1 read : 1 write)")
    del a, b
    roofline["achieved_over_streaming_copy"] = roofline["achieved"] / streaming_copy["GBps"]

    others = []
    del layer, x, dy
    torch.cuda.empty_cache()
    for name in [n for n in args.others.split(",") if n and n != wl.name]:
        w2 = synth.WORKLOADS[name]
        log(f"[bench] secondary workload {name}")
        l2 = Layer(w2, torch, cgbn, *device_inputs_fast(w2, torch, synth, dev))
        others.append(measure_workload(l2, torch, max(5, args.steps // 5), max(2, args.warmup // 2)))
        if not others[-1]["single_launch"]["forward"]:
            # the forward runs as separate sweeps: also with a sweep each for the sums and the squared deviations
            # (9 instead of 8 tensor sweeps per step)
            cgbn.cgbn_set_tuning("one_sweep_stats", 0)
            v = measure_workload(l2, torch, max(5, args.steps // 5), 2)
            cgbn.cgbn_set_tuning("one_sweep_stats", 1)
            others[-1]["two_sweep_statistics"] = dict(
                ms_per_step=v["ms_per_step"], fwd_ms=v["fwd_ms"], moved_bytes_by_design=v["moved_bytes_by_design"],
                moved_GBps=v["moved_GBps"], pct_of_peak_on_moved_bytes=v["pct_of_peak_on_moved_bytes"],
                pct_of_peak_on_min_bytes=v["pct_of_peak_on_min_bytes"])
        if w2.S * w2.elem_bytes <= (1 << 20):
            # launch-latency bound (the tensors live in L2): also as a replayed HIP graph
            others[-1]["ms_per_step_graph_replay"] = measure_graph(l2, torch, 200)
        elif 4 * w2.S * w2.elem_bytes <= (2 << 30):
            # tensors near the size of the memory-side cache (256 MB): the figure above re-uses one
            # buffer set ("warm"), this one rotates over four ("cold")
            others[-1]["ms_per_step_rotating_4_buffer_sets"] = measure_rotating(l2, torch, cgbn, max(8, args.steps // 5))
        del l2
        torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu_baseline:
        log("[bench] timing the float64 oracle on the host")
        cpu = cpu_baseline(wl, synth)

    out = {
        "metric": METRIC, "value": head["min_bytes_GBps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: N={wl.N} C={wl.C} H={wl.H} W={wl.W} {wl.layout} {wl.dtype} K={wl.K}",
                   "step": "cgbn_forward + cgbn_backward",
                   "value_is": "minimum bytes of a step (each of x, y, dy, x, dx touched once = 5 tensors) / step time",
                   "min_bytes": 5 * Sb, "two_pass_sweep_bytes": 9 * Sb,
                   "tuning": {k: cgbn.cgbn_get_tuning(k) for k in
                              ("chunk_bytes", "wave_plane_bytes", "tiny_planes", "piece_bytes", "map_piece_bytes", "reverse", "nt_store", "fused",
                               "big_lds", "stagger", "stagger_us", "stagger_phases", "one_sweep_stats", "cooperative", "wait_us")},
                   "single_launch": head["single_launch"]},
        "pct_of_peak_on_min_bytes": head["pct_of_peak_on_min_bytes"],
        "moved_bytes_by_design": head["moved_bytes_by_design"], "pct_of_peak_on_moved_bytes": head["pct_of_peak_on_moved_bytes"],
        "two_pass_equivalent_GBps": head["two_pass_equivalent_GBps"],
        "fwd_ms": head["fwd_ms"], "bwd_ms": head["bwd_ms"],
        "fwd_min_bytes_GBps": head["fwd_min_bytes_GBps"], "bwd_min_bytes_GBps": head["bwd_min_bytes_GBps"],
        "step_ms": {"median": head["step_ms_median"], "min": head["step_ms_min"], "max": head["step_ms_max"]},
        "sweeps": sweeps, "fixed_statistics_mode": frozen, "relu_variants": relu, "roofline": roofline, "streaming_copy_on_this_box": streaming_copy, "cpu_baseline": cpu, "other_workloads": others,
        "device": torch.cuda.get_device_name(0), "hip": torch.version.hip,
        "compute_units": torch.cuda.get_device_properties(0).multi_processor_count,
        "hbm_GiB": torch.cuda.get_device_properties(0).total_memory / 2 ** 30,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
