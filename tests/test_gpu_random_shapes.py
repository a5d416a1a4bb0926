"""Seeded random shapes through both paths (single-launch where the shape allows, multi-sweep),
plain and ReLU variants, against the float64 oracle: a net for shape-dependent indexing mistakes
(ragged tiles, odd planes, shard/row bookkeeping) that the hand-picked cases may miss."""

import dataclasses

import numpy as np
import pytest
import torch

import gpu_harness as G
from oracle import cgbn_oracle as O
from oracle import cgbn_relu_oracle as R
from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth

pytestmark = pytest.mark.gpu

BASE = synth.WORKLOADS["cfg1"]


def _draw_tiny(count, seed):
    """NCHW shapes for the kernels that take runs of tiny planes (C a multiple of 8, planes up to 2 KiB), and
    planes of 19-56 KB with enough images for three or four planes per workgroup."""
    r = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        dtype = "f32" if r.random() < 0.5 else "bf16"
        K = int(r.choice([1, 2, 3, 4]))
        if r.random() < 0.7:
            N = K * int(r.integers(1, 5))
            C = int(r.choice([8, 16, 24, 40, 64, 136, 264]))
            H, W = int(r.integers(1, 25)), int(r.integers(1, 25))
            if H * W * (4 if dtype == "f32" else 2) > 2048:
                continue
        else:
            N = K * int(r.integers(2, 5))
            C = int(r.integers(1, 4))
            H, W = int(r.integers(60, 130)), int(r.integers(80, 130))
        if N * C * H * W > 1_500_000:
            continue
        shapes.append(dict(N=N, C=C, H=H, W=W, K=K, layout="NCHW", dtype=dtype))
    return shapes


def _draw_shapes(count, seed, wide=False):
    r = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        layout = "NCHW" if r.random() < (0.75 if wide else 0.6) else "NHWC"
        dtype = "f32" if r.random() < 0.6 else "bf16"
        K = int(r.choice([1, 2, 3, 4, 6, 8]))
        N = K * int(r.integers(1, 4))
        if wide and r.random() < 0.3:
            N = K * int(r.integers(4, 17))          # enough images for planes in LDS and several units per channel
        if layout == "NCHW":
            C = int(r.integers(1, 9))
            H, W = int(r.integers(1, 90)), int(r.integers(1, 150))
            if wide:
                kind = int(r.integers(0, 3))
                if kind == 0:                        # mid-size planes: spilled slots, two planes per workgroup
                    H, W = int(r.integers(40, 130)), int(r.integers(60, 200))
                elif kind == 1:                      # the feature-map sizes of the detector's backbone
                    H, W = int(r.choice([13, 25, 50, 100])), int(r.choice([21, 42, 84, 168]))
        else:
            C = int(r.choice([1, 3, 8, 12, 32, 40, 64, 100, 256]))
            H, W = int(r.integers(1, 40)), int(r.integers(1, 40))
        if N * C * H * W > (1_500_000 if wide else 600_000):
            continue
        shapes.append(dict(N=N, C=C, H=H, W=W, K=K, layout=layout, dtype=dtype))
    return shapes


SHAPES = _draw_shapes(48, 20240607) + _draw_shapes(72, 20240608, wide=True) + _draw_tiny(40, 20240609)


@pytest.mark.parametrize("fused", [1, 0], ids=["fused", "sweeps"])
@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_random_shape(i, fused):
    kw = SHAPES[i]
    wl = dataclasses.replace(BASE, name=f"rnd{i}", **kw)
    print(f"[case] random {i} fused={fused}: {kw}", flush=True)
    old = L.cgbn_get_tuning("fused")
    L.cgbn_set_tuning("fused", fused)
    try:
        d = synth.make_inputs(wl)
        p = G.Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
        p.forward()
        p.backward()
        got = p.results()
        xw, dyw = G.widen(d["x"], wl.dtype), G.widen(d["dy"], wl.dtype)
        g64, b64 = d["gamma"].astype(np.float64), d["beta"].astype(np.float64)
        sum_scale = np.sqrt(wl.M) * G.rms(dyw)      # what a channel's gradient sums amount to when nothing cancels
        # with a handful of values per channel eps << var makes dx (and only dx) ill-conditioned in float:
        # (1 - xhat^2) of nearly equal terms; everything else is compared whatever M is
        skip = () if wl.M >= 8 else ("dx",)
        ref = O.cgbn_forward_backward_ref(xw, dyw, g64, b64, wl.eps, wl.layout)
        G.check_against_oracle(got, ref, wl.dtype, f"random {i}", sum_scale=sum_scale, skip=skip)
        # ReLU variant with a shortcut on the same shape
        sc_host = np.random.default_rng(i).standard_normal(d["x"].shape).astype(np.float32)
        if wl.dtype == "bf16":
            sc_host = synth.f32_to_bf16_bits(sc_host)
        sc, dz = G.to_dev(sc_host), torch.empty_like(p.x)
        L.cgbn_forward_relu(p.x, sc, *p.shape_args, wl.layout, wl.K, p.gamma, p.beta, wl.eps, p.y, p.mean, p.invstd,
                            wl.dtype, p.mean_lo, p.ws)
        L.cgbn_backward_relu(p.dy, p.y, p.x, p.mean, p.invstd, p.gamma, p.dx, dz, p.dgamma, p.dbeta, *p.shape_args,
                             wl.layout, wl.K, wl.dtype, p.mean_lo, p.ws)
        got = p.results()
        ys = got["y"]
        y_ref, m_ref, i_ref = R.cgbn_relu_forward_ref(xw, g64, b64, wl.eps, wl.layout, residual=G.widen(sc_host, wl.dtype))
        dx_ref, dg_ref, db_ref, dz_ref = R.cgbn_relu_backward_ref(dyw, ys, xw, m_ref, i_ref, g64, wl.layout)
        assert np.array_equal(G.to_host_f64(dz, wl.dtype), dz_ref)
        ref = dict(y=y_ref, mean=m_ref, invstd=i_ref, dx=dx_ref, dgamma=dg_ref, dbeta=db_ref)
        G.check_against_oracle(got, ref, wl.dtype, f"random {i} relu", sum_scale=sum_scale, skip=skip)
    finally:
        L.cgbn_set_tuning("fused", old)
