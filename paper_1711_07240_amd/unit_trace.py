"""Per-unit timeline of the single-launch kernels (a profiling aid, not part of the product path).

An instrumented flavour of the library (built with -DCGBN_TRACE beside the product one) makes thread 0 of
every workgroup write the device's 100 MHz wall clock into a buffer at the phase boundaries of each unit:
start, rows published ("arrived"), rows of all sibling units gathered, statistics reduced, unit written out.
This script runs one forward and one backward of a workload on that flavour and prints how a unit's time
divides into loading + partial sums, waiting for the sibling units, reducing, and writing out.

    python -m paper_1711_07240_amd.unit_trace --build          # on the CPU: compile the instrumented flavour
    python -m paper_1711_07240_amd.unit_trace cfg1 cfg3        # on the GPU
"""

from __future__ import annotations

import ctypes
import os
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
TRACE_LIB = os.path.join(PKG, "_build_trace", "libcgbn_trace.so")


def build_flavour() -> str:
    from paper_1711_07240_amd import build as b
    os.makedirs(os.path.dirname(TRACE_LIB), exist_ok=True)
    return b.build(extra_flags=["-DCGBN_TRACE"], lib=TRACE_LIB, obj_dir=os.path.join(PKG, "_build_trace"))


def main(argv) -> int:
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    if argv and argv[0] == "--build":
        print(build_flavour())
        return 0
    import numpy as np
    import torch
    from paper_1711_07240_amd import cgbn, synth
    import bench
    if not os.path.exists(TRACE_LIB):
        sys.exit(f"{TRACE_LIB} is not built: run with --build first")
    cgbn.LIB_PATH = TRACE_LIB
    lib = cgbn.lib()
    lib.cgbn_debug_set_trace.argtypes = [ctypes.c_void_p]
    lib.cgbn_debug_set_trace.restype = None
    dev = torch.device("cuda:0")
    for name in argv or ["cfg1"]:
        wl = synth.WORKLOADS[name]
        layer = bench.Layer(wl, torch, cgbn, *bench.device_inputs_fast(wl, torch, synth, dev))
        for _ in range(3):
            layer.step()
        torch.cuda.synchronize()
        for direction in ("forward", "backward"):
            slots = 1 << 18
            buf = torch.zeros(slots * 8, dtype=torch.int64, device=dev)
            lib.cgbn_debug_set_trace(ctypes.c_void_p(buf.data_ptr()))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            getattr(layer, direction)()
            e1.record()
            torch.cuda.synchronize()
            lib.cgbn_debug_set_trace(None)
            taken = cgbn.cgbn_get_tuning("last_forward_fused" if direction == "forward" else "last_backward_fused")
            if not taken:
                print(f"== {name} {direction}: runs as separate sweeps, no units to trace")
                continue
            t = buf.cpu().numpy().reshape(-1, 8)
            t = t[t[:, 0] != 0].astype(np.float64)
            t = (t - t[:, 0].min()) / 100.0                        # microseconds
            n = len(t)
            total = t[:, 7] - t[:, 0]
            print(f"== {name} {direction}: launch {e0.elapsed_time(e1) * 1e3:.0f} us, {n} units, "
                  f"last unit done at {t[:, 7].max():.0f} us, mean unit {total.mean():.1f} us")
            for label, a, b in (("load + partial sums + publish", 0, 1), ("wait for siblings + gather", 1, 2),
                                ("reduce", 2, 3), ("elementwise + write out", 3, 7)):
                d = t[:, b] - t[:, a]
                print(f"   {label:30s} mean {d.mean():6.2f} us ({100 * d.sum() / total.sum():4.1f} % of unit time)  "
                      f"p50 {np.median(d):6.2f}  p95 {np.percentile(d, 95):6.2f}  max {d.max():6.2f}")
            U = cgbn.cgbn_plan_get(wl.N, wl.C, wl.H, wl.W, wl.layout, wl.dtype, wl.K,
                                   ("fwd_U" if direction == "forward" else "bwd_U"))
            if U > 0 and n == U * wl.C:
                tc = t.reshape(wl.C, U, 8)
                spread = tc[:, :, 1].max(axis=1) - tc[:, :, 1].min(axis=1)
                lag = tc[:, :, 2].min(axis=1) - tc[:, :, 1].max(axis=1)
                print(f"   per channel ({U} units): arrivals spread over {spread.mean():.1f} us (p95 {np.percentile(spread, 95):.1f}); "
                      f"last arrival -> first sibling released {lag.mean():.1f} us (p95 {np.percentile(lag, 95):.1f})")
            # how many workgroups are in each phase as time goes by (1 us bins): the memory system has work only
            # from those that load or write out
            span = int(np.ceil(t[:, 7].max())) + 1
            occ = np.zeros((3, span + 1))
            for ph, (a, b) in enumerate(((0, 1), (1, 3), (3, 7))):
                np.add.at(occ[ph], np.floor(t[:, a]).astype(int), 1)
                np.add.at(occ[ph], np.floor(t[:, b]).astype(int), -1)
            occ = np.cumsum(occ, axis=1)[:, :span]
            busy = occ[0] + occ[2]
            steady = slice(span // 10, span - span // 10)
            print(f"   workgroups per phase, mean over the middle 80 % of the launch: loading {occ[0][steady].mean():.0f}, "
                  f"waiting/reducing {occ[1][steady].mean():.0f}, writing out {occ[2][steady].mean():.0f}; "
                  f"time with fewer than 100 workgroups loading or writing: {100 * (busy[steady] < 100).mean():.1f} %, "
                  f"fewer than 250: {100 * (busy[steady] < 250).mean():.1f} %")
            if os.environ.get("CGBN_TRACE_TIMELINE"):
                step = max(1, span // 60)
                print("   timeline (us: loading/waiting/writing): " + " ".join(
                    f"{i}:{occ[0][i]:.0f}/{occ[1][i]:.0f}/{occ[2][i]:.0f}" for i in range(0, span, step)))
            if os.environ.get("CGBN_TRACE_PLACEMENT"):
                # where the time goes by placement: workgroup b runs units b, b + G, ...; workgroups are dealt to the
                # chip's 8 dies (XCDs) in turn, and to a compute unit's residency slots in waves of 256
                G_ = int(os.environ["CGBN_TRACE_PLACEMENT"])
                full = buf.cpu().numpy().reshape(-1, 8).astype(np.float64)
                idx = np.nonzero(full[:, 0])[0]
                load = (full[idx, 1] - full[idx, 0]) / 100.0
                wait = (full[idx, 2] - full[idx, 1]) / 100.0
                b = idx % G_
                for label, key in (("die (b % 8)", b % 8), ("slot (b // 256)", b // 256)):
                    print(f"   by {label}: " + "  ".join(
                        f"{k}: load {load[key == k].mean():.1f} wait {wait[key == k].mean():.1f}" for k in np.unique(key)))
        del layer
        torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
