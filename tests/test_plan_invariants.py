"""Host-side launch planning without a GPU: for thousands of seeded shapes the numbers the
kernels trust for their indexing (pieces, tiles, units, rows, slots) must cover the tensor
exactly, fit what a workgroup can hold, and fit the workspace.  The capacities below are the
kernels' own (128 words of unit data per thread in the forward, 64 per tensor in the backward,
plus 24 / 48 / 44 words in LDS depending on the variant), restated here from their definition."""

import os
import re

import numpy as np
import pytest

from paper_1711_07240_amd import cgbn as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
THREADS, WAVE = 256, 64
MAX_ROWS, MAX_SHARDS = 2048, 512
BIG_ROWS, BIG_SHARDS_LARGE, BIG_SHARDS_SMALL = 384, 48, 128


def _built():
    """(LB, LPPC) pairs the single-launch kernels are instantiated for, from the list header (a list may be
    made of other lists)."""
    text = open(os.path.join(ROOT, "paper_1711_07240_amd", "csrc", "cgbn_fused_list.h")).read()
    text = text.replace("\\\n", " ")
    bodies = dict(re.findall(r"#define CGBN_FUSED_(\w+)\(X\)(.*)", text))

    def pairs(name):
        body = bodies[name]
        out = {(int(a), int(b)) for a, b in re.findall(r"\bX\((\d+),\s*(-?\d+)\)", body)}
        for sub in re.findall(r"CGBN_FUSED_(\w+)\(X\)", body):
            out |= pairs(sub)
        return out

    return {name: pairs(name) for name in ("COMMON", "FORWARD_ONLY", "BACKWARD_ONLY", "BIG_SMALL", "RELU_BWD_F32_NARROW",
                                           "WGP_FORWARD", "WGP_BACKWARD")}


BUILT = _built()


def _slot_counts():
    text = open(os.path.join(ROOT, "paper_1711_07240_amd", "csrc", "cgbn_fused_list.h")).read()
    body = re.search(r"kCgbnSlotCounts\[\]\s*=\s*\{([^}]*)\}", text).group(1)
    return [int(v) for v in body.split(",")]


SLOT_COUNTS = _slot_counts()


def _full_slots(lppc, R):
    """Leading slots of every plane the kernels of a variant treat as full without looking (restated from the
    rule: the host takes the smallest admissible slot count, so a plane is longer than the next smaller one)."""
    if lppc > R:
        return R
    smaller = [c for c in SLOT_COUNTS if c < lppc]
    prev = smaller[-1] if smaller else 0
    return prev if prev * 16 >= R else 0


def _ceil(a, b):
    return -(-a // b)


def _get(shape, key):
    return L.cgbn_plan_get(*shape, key)


def _check_sweeps(shape):
    N, C, H, W, layout, dtype, K = shape
    eb = 4 if dtype == "f32" else 2
    HW, ips = H * W, N // K
    g = lambda k: _get(shape, k)
    rows, rps = g("rows"), g("rps")
    assert rows == rps * K
    if layout == "NCHW":
        if g("tiny"):
            tg = g("tg")
            assert HW * eb <= 2048 and C % 8 == 0, "tiny planes: a workgroup's run must start and end on 16 bytes"
            assert tg in (8, 16, 32, 64, 128, 256) and tg * HW * eb <= 16384, "the run must fit its LDS stage"
            assert tg == 256 or 2 * tg * HW * eb > 16384, "... and be the longest that does"
            assert g("L") == HW and g("sp") == 1 and not g("wave_mode")
            assert g("grid") == N * _ceil(C, tg) and rows == N
        elif g("wave_mode"):
            assert HW * eb <= 16384 and g("L") == HW and g("sp") == 1
            assert g("grid") == _ceil(N * C, 4) and rows == N
        else:
            Lc, sp = g("L"), g("sp")
            assert sp == _ceil(HW, Lc) and (sp - 1) * Lc < HW <= sp * Lc
            assert Lc == HW or Lc % (THREADS * 16 // eb) == 0
            assert g("grid") == N * C * sp and rows == N * sp and rps == ips * sp
    else:
        full = 16 // eb
        vec = full if C % full == 0 else 1
        assert g("vec") == vec and g("cv") == C // vec
        TW, ctiles, rpp = g("TW"), g("ctiles"), g("rpp")
        assert TW == min(C // vec, THREADS) and ctiles == _ceil(C // vec, TW) and rpp == THREADS // TW >= 1
        spix = ips * HW
        for pl, pp in (("PL", "pps"), ("PLm", "ppsm"), ("PLm2", "ppsm2")):
            PL, pps = g(pl), g(pp)
            assert 1 <= PL <= spix and pps == _ceil(spix, PL) and (pps - 1) * PL < spix
            assert PL == spix or PL % (4 * rpp) == 0
        assert rows == g("pps") * K and g("grid") == rows * ctiles and g("gridm") == g("ppsm") * K * ctiles and g("gridm2") == g("ppsm2") * K * ctiles
    G = g("G")
    assert G in (1, 2, 4, 8, 16, 32, 64) and G >= min(rps, WAVE) and (G == 1 or G // 2 < rps)
    return rows


def _check_fused(shape, direction):
    N, C, H, W, layout, dtype, K = shape
    eb = 4 if dtype == "f32" else 2
    HW, ips = H * W, N // K
    g = lambda k: _get(shape, direction + "_" + k)
    if not g("ok"):
        return 0
    assert layout == "NCHW" and K <= MAX_SHARDS
    words = 128 if direction == "fwd" else 64
    lds = {0: 24, 1: 48, 2: 44}
    LB, LPPC, big, U, rows = g("LB"), g("LPPC"), g("big"), g("U"), g("rows")
    assert LB in (4, 8, 16) and (HW * eb) % LB == 0 and (LB == 16 or (HW * eb) % (2 * LB) != 0)
    Wd, E = LB // 4, LB // eb
    R = words // Wd
    ldsw = lds[big] if direction == "fwd" else lds[big] // 2
    if LPPC > 0:                                     # small planes, whole, LPPC slots each
        assert big in (0, 2)
        LPP = g("LPP")
        assert LPP == _ceil(HW, WAVE * E) and LPP <= LPPC
        full = _full_slots(LPPC, R)
        assert full < LPP, "the kernels read the first `full` slots of a plane without any check"
        assert full * WAVE * LB <= HW * eb, "... so those slots must lie wholly inside the plane"
        if LPPC > R:                                 # one plane per wavefront, its last slots in LDS
            assert big == 0 and LPPC == R + ldsw // Wd and LB >= 8
            per_wave = 1
        else:
            per_wave = R // LPPC + ((ldsw // Wd) // LPPC if big == 2 else 0)
        IPU = g("IPU")
        assert 1 <= IPU <= 4 * per_wave, "a unit must fit the registers and LDS planes of its workgroup"
        assert U * IPU >= N and (U - 1) * IPU < N
        assert rows == N and g("rps") == ips
        assert IPU * C * HW * eb <= 2 ** 31 - 1
        lists = BUILT["BIG_SMALL"] if big == 2 else BUILT["COMMON"] | BUILT["FORWARD_ONLY" if direction == "fwd" else "BACKWARD_ONLY"]
        assert (LB, LPPC) in lists, "no such kernel is built"
        if big == 2:
            assert N <= BIG_ROWS and K <= BIG_SHARDS_SMALL
    elif LPPC < 0:                                   # several whole planes per workgroup, in workgroup-wide slots
        ppu = -LPPC
        assert LB == 16 and big in (0, 1) and g("tp") == 1 and N >= ppu >= 2
        spw = (R + ldsw // Wd) // ppu
        assert _ceil(HW * eb, THREADS * LB) <= spw, "each plane must fit its share of the workgroup's slots"
        assert U == _ceil(N, ppu) and rows == N and g("rps") == ips
        assert C * HW * eb <= 2 ** 32 - 1
        if big == 1:
            assert rows <= BIG_ROWS and K <= BIG_SHARDS_LARGE
        if ppu == 2:
            assert (16, -2) in BUILT["COMMON"]
        else:
            assert big == 1 and (16, LPPC) in BUILT["WGP_FORWARD" if direction == "fwd" else "WGP_BACKWARD"]
    else:                                            # large planes cut into equal tiles
        assert LB in (8, 16) and big in (0, 1)
        tp, TL = g("tp"), g("TL")
        assert TL % (THREADS * E) == 0 and tp == _ceil(HW, TL) and (tp - 1) * TL < HW
        cap = (R + (ldsw // Wd if LB == 16 else 0)) * THREADS * E
        assert TL <= cap, "a tile must fit the registers and LDS slots of its workgroup"
        assert U == N * tp == rows and g("rps") == ips * tp
        if big == 1:
            assert LB == 16 and rows <= BIG_ROWS and K <= BIG_SHARDS_LARGE
        assert (LB, 0) in BUILT["COMMON"]
    assert rows <= MAX_ROWS and g("total_units") == C * U
    G = g("G")
    assert G in (1, 2, 4, 8, 16, 32, 64) and G >= min(g("rps"), WAVE)
    return rows


def _check(shape):
    if L.cgbn_workspace_bytes(*shape) == 0:          # refused (too many workgroups or rows to index): nothing to launch
        return False
    rows = max(_check_sweeps(shape), _check_fused(shape, "fwd"), _check_fused(shape, "bwd"))
    N, C, H, W, layout, dtype, K = shape
    assert _get(shape, "part_bytes") >= C * rows * 4
    assert _get(shape, "shard_bytes") >= K * C * 8
    wb = L.cgbn_workspace_bytes(*shape)
    assert wb >= 2 * _get(shape, "part_bytes") + 2 * _get(shape, "shard_bytes") + 4 * C + 4 * (64 + 4 * C)
    off = L.cgbn_workspace_error_offset(*shape)
    assert 0 < off < wb and off % 4 == 0
    return True


def _random_shapes(count, seed):
    r = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        layout = "NCHW" if r.random() < 0.6 else "NHWC"
        dtype = "f32" if r.random() < 0.5 else "bf16"
        K = int(r.choice([1, 2, 3, 4, 7, 8, 16, 32, 48, 64, 128, 129, 256, 512, 600]))
        N = K * int(r.integers(1, 9))
        C = int(r.choice([1, 3, 7, 8, 16, 24, 64, 100, 256, 512, 1028, 2048, 4096]))
        kind = r.integers(0, 4)
        if kind == 0:
            H, W = int(r.integers(1, 8)), int(r.integers(1, 8))
        elif kind == 1:
            H, W = int(r.integers(1, 64)), int(r.integers(1, 64))
        elif kind == 2:
            H, W = int(r.integers(20, 400)), int(r.integers(20, 700))
        else:
            H, W = int(r.choice([13, 25, 50, 100, 200, 400, 800])), int(r.choice([21, 42, 84, 168, 336, 672, 1344]))
        if N * C * H * W > 2 ** 36:
            continue
        out.append((N, C, H, W, layout, dtype, K))
    return out


def test_workloads_of_the_paper():
    for shape in [(4, 16, 32, 32, "NCHW", "f32", 2), (16, 64, 400, 672, "NCHW", "f32", 8),
                  (16, 256, 200, 336, "NCHW", "f32", 8), (256, 2048, 25, 42, "NCHW", "f32", 128),
                  (64, 512, 50, 84, "NHWC", "bf16", 32), (64, 512, 50, 84, "NHWC", "f32", 32)]:
        _check(shape)
    # what the measurements quote: units per channel of the headline workloads
    assert _get((16, 64, 400, 672, "NCHW", "f32", 8), "fwd_U") == 96
    assert _get((16, 64, 400, 672, "NCHW", "f32", 8), "bwd_U") == 192
    assert _get((256, 2048, 25, 42, "NCHW", "f32", 128), "fwd_U") == 8
    assert _get((256, 2048, 25, 42, "NCHW", "f32", 128), "bwd_U") == 16


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_random_shapes(seed):
    taken = 0
    for shape in _random_shapes(1500, seed):
        try:
            taken += _check(shape)
        except AssertionError as e:
            raise AssertionError(f"{shape}: {e}") from e
    assert taken >= 1400                             # the library refuses next to none of them


@pytest.mark.parametrize("knobs", [dict(big_lds=0), dict(chunk_bytes=8192, wave_plane_bytes=1024),
                                   dict(piece_bytes=65536, map_piece_bytes=16384)])
def test_random_shapes_under_other_knobs(knobs):
    old = {k: L.cgbn_get_tuning(k) for k in knobs}
    try:
        for k, v in knobs.items():
            L.cgbn_set_tuning(k, v)
        for shape in _random_shapes(600, 11):
            if "wave_plane_bytes" in knobs and shape[4] == "NCHW":
                continue                             # (the wave-mode bound checked above is the default's)
            try:
                _check(shape)
            except AssertionError as e:
                raise AssertionError(f"{knobs} {shape}: {e}") from e
    finally:
        for k, v in old.items():
            L.cgbn_set_tuning(k, v)


def test_invalid_arguments_and_keys():
    assert L.cgbn_plan_get(4, 16, 32, 32, "NCHW", "f32", 3, "grid") == -1      # K does not divide N
    assert L.cgbn_plan_get(4, 16, 32, 32, "NCHW", "f32", 2, "no_such_key") == -1
    assert L.cgbn_plan_get(4, 16, 32, 32, "NCHW", "f32", 2, "fwd_no_such_key") == -1
