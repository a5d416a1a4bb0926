"""GPU parity under every launch-shape knob: each knob setting below runs all the small shapes of
test_gpu_parity through forward and backward and compares them with the float64 oracle element by
element.  (The knobs change how the work is cut up and launched, never what is computed.)"""

import pytest

from paper_1711_07240_amd import cgbn as L
from paper_1711_07240_amd import synth
from gpu_harness import Problem, check_against_oracle
from test_gpu_parity import SMALL, BASE, oracle_all

pytestmark = pytest.mark.gpu

KNOBS = [
    dict(cooperative=1),
    dict(stagger=0),
    dict(stagger_us=3, stagger_phases=8),
    dict(big_lds=0),
    dict(nt_store=0),
    dict(reverse=0),
    dict(tiny_planes=0),
    dict(chunk_bytes=8192, wave_plane_bytes=1024),
    dict(piece_bytes=65536, map_piece_bytes=16384),
    dict(fused_groups=48),
    dict(fused=0),
    dict(fused=0, one_sweep_stats=0),
]


@pytest.mark.parametrize("knobs", KNOBS, ids=[",".join(f"{k}={v}" for k, v in ks.items()) for ks in KNOBS])
def test_every_small_shape_under_this_setting(knobs):
    old = {k: L.cgbn_get_tuning(k) for k in knobs}
    for k, v in knobs.items():
        L.cgbn_set_tuning(k, v)
    try:
        for name, kw in SMALL:
            wl = BASE.scaled(name=name, **kw)
            d = synth.make_inputs(wl)
            p = Problem(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype, wl.K)
            p.forward()
            p.backward()
            ref = oracle_all(d["x"], d["dy"], d["gamma"], d["beta"], wl.eps, wl.layout, wl.dtype)
            check_against_oracle(p.results(), ref, wl.dtype, f"{name} under {knobs}")
        print(f"[ok] {len(SMALL)} shapes under {knobs}", flush=True)
    finally:
        for k, v in old.items():
            L.cgbn_set_tuning(k, v)
