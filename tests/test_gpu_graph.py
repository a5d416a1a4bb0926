"""The library under HIP graph capture: cgbn_forward + cgbn_backward allocate nothing,
never synchronise and clear their scratch with a kernel (not a memset node), so a
captured step must replay to exactly the eager result, every time."""

import dataclasses

import pytest
import torch

import gpu_harness as G
from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth

pytestmark = pytest.mark.gpu

BASE = synth.WORKLOADS["cfg1"]
CASES = [
    ("cfg0", synth.WORKLOADS["cfg0"]),                                                    # launch-latency bound
    ("single-launch-tiles", dataclasses.replace(BASE, name="g1", N=2, C=3, H=200, W=200, K=2)),
    ("single-launch-small-planes", dataclasses.replace(BASE, name="g2", N=8, C=24, H=25, W=42, K=4)),
    ("channels-last-sweeps", dataclasses.replace(BASE, name="g3", N=4, C=24, H=31, W=17, K=4, layout="NHWC", dtype="bf16")),
]


@pytest.mark.parametrize("name,wl", CASES, ids=[c[0] for c in CASES])
def test_captured_step_replays_to_the_eager_result(name, wl):
    print(f"[case] graph {name}", flush=True)
    d = synth.make_inputs(wl)
    p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
    p.forward()
    p.backward()
    torch.cuda.synchronize()
    outs = (p.y, p.dx, p.mean, p.invstd, p.mean_lo, p.dgamma, p.dbeta)
    eager = [t.clone() for t in outs]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):            # the binding launches on torch's current stream
        p.forward()
        p.backward()
    for replay in range(4):
        for t in outs:                                    # eager work between replays: wipe the outputs
            t.fill_(float("nan")) if t.dtype.is_floating_point else t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, e in zip(outs, eager):
            assert torch.equal(t, e), f"{name}: replay {replay} differs from the eager result"
    err = p.ws[L.cgbn_workspace_error_offset(*p.shape_args, wl.layout, wl.dtype, wl.K):][:4].view(torch.int32)
    assert int(err.item()) == 0


def test_two_streams_with_cooperative_launches():
    """Two layers whose single-launch kernels may overlap on two streams: with the "cooperative" knob the
    results equal those of running them one after the other."""
    wls = [dataclasses.replace(BASE, name="s0", N=4, C=48, H=200, W=200, K=2),
           dataclasses.replace(BASE, name="s1", N=8, C=256, H=25, W=42, K=4)]
    probs = []
    for wl in wls:
        d = synth.make_inputs(wl)
        probs.append(G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K))
    outs = lambda p: (p.y, p.dx, p.mean, p.invstd, p.dgamma, p.dbeta)
    want = []
    for p in probs:                                   # one after the other
        p.forward()
        p.backward()
        torch.cuda.synchronize()
        assert L.cgbn_get_tuning("last_forward_fused") == 1 and L.cgbn_get_tuning("last_backward_fused") == 1
        want.append([t.clone() for t in outs(p)])
        for t in outs(p):
            t.fill_(float("nan"))
    old = L.cgbn_get_tuning("cooperative")
    L.cgbn_set_tuning("cooperative", 1)
    try:
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        for rep in range(3):
            for p, s in zip(probs, streams):
                with torch.cuda.stream(s):
                    p.forward()
                    p.backward()
        torch.cuda.synchronize()
    finally:
        L.cgbn_set_tuning("cooperative", old)
    for p, w in zip(probs, want):
        for t, e in zip(outs(p), w):
            assert torch.equal(t, e)
        err = p.ws[L.cgbn_workspace_error_offset(*p.shape_args, p.layout, p.dtype, p.K):][:4].view(torch.int32)
        assert int(err.item()) == 0
