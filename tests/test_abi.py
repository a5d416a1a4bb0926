"""The C ABI without a GPU: the library loads, exports what the header declares,
sizes workspaces, and turns bad arguments into status codes before any launch."""

import os
import re

import pytest

from paper_1711_07240_amd import cgbn as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cgbn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cgbn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "cgbn_forward" in names and "cgbn_backward" in names and len(names) >= 14
    handle = L.lib()
    for n in names:
        assert hasattr(handle, n), n
    assert sorted(L.SIGNATURES) == names
    for n in names:                       # the binding has a function of the same name
        assert callable(getattr(L, n)), n


def test_status_strings():
    seen = {L.cgbn_status_string(i) for i in range(13)}
    assert len(seen) == 13 and "ok" in seen and "unknown status" not in seen
    assert L.cgbn_status_string(99) == "unknown status"


def test_workspace_bytes():
    wb = L.cgbn_workspace_bytes(4, 16, 32, 32, "NCHW", "f32", 2)
    assert wb > 0 and wb % 256 == 0
    for wl in [(16, 64, 400, 672, "NCHW", "f32", 8), (256, 2048, 25, 42, "NCHW", "f32", 128),
               (64, 512, 50, 84, "NHWC", "bf16", 32)]:
        b = L.cgbn_workspace_bytes(*wl)
        assert 0 < b < 64 << 20 and b % 256 == 0
    # invalid problems have no workspace size
    assert L.cgbn_workspace_bytes(4, 16, 32, 32, "NCHW", "f32", 3) == 0
    assert L.cgbn_workspace_bytes(0, 16, 32, 32, "NCHW", "f32", 1) == 0
    assert L.cgbn_workspace_bytes(4, 16, 32, 32, 7, "f32", 2) == 0
    assert L.cgbn_workspace_bytes(4, 16, 32, 32, "NCHW", 5, 2) == 0


P = 0x10000  # a non-null, 256-byte aligned fake address: never dereferenced on these paths
GOOD = dict(x=P, N=4, C=16, H=32, W=32, layout="NCHW", K=2, gamma=P, beta=P, eps=1e-5,
            y=P, mean=P, invstd=P, dtype="f32", mean_lo=None, workspace=P,
            workspace_bytes=1 << 20, stream=0)


def _fwd(**kw):
    a = dict(GOOD, **kw)
    with pytest.raises(L.CgbnError) as e:
        L.cgbn_forward(**a)
    return e.value.code


def test_forward_argument_errors():
    assert _fwd(x=None) == 1 and _fwd(gamma=None) == 1 and _fwd(y=None) == 1 and _fwd(invstd=None) == 1
    assert _fwd(N=0) == 2 and _fwd(C=-1) == 2 and _fwd(H=0) == 2
    assert _fwd(N=1 << 20, C=1 << 20) == 2
    assert _fwd(K=0) == 3 and _fwd(K=3) == 3 and _fwd(K=8) == 3
    assert _fwd(layout=2) == 4 and _fwd(dtype=-1) == 4
    assert _fwd(eps=0.0) == 5 and _fwd(eps=-1.0) == 5 and _fwd(eps=float("nan")) == 5
    assert _fwd(eps=float("inf")) == 5
    assert _fwd(workspace=None) == 6 and _fwd(workspace_bytes=16) == 6 and _fwd(workspace=P + 64) == 6
    assert _fwd(x=P + 4) == 7 and _fwd(y=P + 8) == 7


def test_backward_argument_errors():
    good = dict(dy=P, x=P, mean=P, invstd=P, gamma=P, dx=P, dgamma=P, dbeta=P, N=4, C=16, H=32, W=32,
                layout="NHWC", K=4, dtype="bf16", mean_lo=None, workspace=P, workspace_bytes=1 << 20,
                stream=0)

    def bwd(**kw):
        with pytest.raises(L.CgbnError) as e:
            L.cgbn_backward(**dict(good, **kw))
        return e.value.code

    assert bwd(dy=None) == 1 and bwd(dgamma=None) == 1 and bwd(mean=None) == 1
    assert bwd(W=0) == 2 and bwd(K=5) == 3 and bwd(layout=-1) == 4 and bwd(dtype=2) == 4
    assert bwd(workspace_bytes=0) == 6 and bwd(dx=P + 2) == 7 and bwd(dy=P + 8) == 7


def test_step_entry_points_validate_too():
    def code(fn, *a, **kw):
        with pytest.raises(L.CgbnError) as e:
            fn(*a, **kw)
        return e.value.code

    assert code(L.cgbn_shard_sum, None, 4, 16, 8, 8, "NCHW", 2, "f32", P, P, 1 << 20, 0) == 1
    assert code(L.cgbn_shard_sum, P, 4, 16, 8, 8, "NCHW", 3, "f32", P, P, 1 << 20, 0) == 3
    assert code(L.cgbn_shard_sum, P, 4, 16, 8, 8, "NCHW", 2, "f32", P, P, 8, 0) == 6
    assert code(L.cgbn_reduce_mean, None, 2, 16, 256, P, None, 0) == 1
    assert code(L.cgbn_reduce_mean, P, 0, 16, 256, P, None, 0) == 3
    assert code(L.cgbn_reduce_mean, P, 2, 16, 0, P, None, 0) == 2
    assert code(L.cgbn_shard_sqdev, P, 4, 16, 8, 8, "NCHW", 2, "f32", None, None, P, P, 1 << 20, 0) == 1
    assert code(L.cgbn_reduce_invstd, P, 2, 16, 256, 0.0, P, 0) == 5
    assert code(L.cgbn_normalize, P, 4, 16, 8, 8, "NCHW", "f32", P, None, P, P, None, P, 0) == 1
    assert code(L.cgbn_normalize, P + 4, 4, 16, 8, 8, "NCHW", "f32", P, None, P, P, P, P, 0) == 7
    assert code(L.cgbn_backward_shard_sums, P, P, 4, 16, 8, 8, "NHWC", 2, "f32", P, None, P, P, None,
                P, 1 << 20, 0) == 1
    assert code(L.cgbn_backward_reduce, P, None, 2, 16, P, P, 0) == 1
    assert code(L.cgbn_backward_dx, P, P, 4, 16, 8, 8, 3, "f32", P, None, P, P, P, P, P, 0) == 4


def test_tuning_knobs():
    assert L.cgbn_get_tuning("no_such_key") == -1
    with pytest.raises(L.CgbnError):
        L.cgbn_set_tuning("no_such_key", 1)
    with pytest.raises(L.CgbnError):
        L.cgbn_set_tuning("reverse", 2)
    with pytest.raises(L.CgbnError):
        L.cgbn_set_tuning("stagger_us", -1)
    with pytest.raises(L.CgbnError):
        L.cgbn_set_tuning("stagger_phases", 1)
    assert L.cgbn_get_tuning("stagger") == 1 and L.cgbn_get_tuning("stagger_us") == 0 and L.cgbn_get_tuning("stagger_phases") == 16
    old = L.cgbn_get_tuning("chunk_bytes")
    before = L.cgbn_workspace_bytes(16, 64, 400, 672, "NCHW", "f32", 8)
    try:
        L.cgbn_set_tuning("chunk_bytes", 2 * old)
        assert L.cgbn_get_tuning("chunk_bytes") == 2 * old
        assert L.cgbn_workspace_bytes(16, 64, 400, 672, "NCHW", "f32", 8) < before
    finally:
        L.cgbn_set_tuning("chunk_bytes", old)


def test_knob_changed_between_sizing_and_call_is_refused_not_overrun():
    """A workspace sized under one set of knobs is too small under another: the call says so before any launch."""
    shape = (16, 64, 400, 672)
    wb = L.cgbn_workspace_bytes(*shape, "NCHW", "f32", 8)
    old = L.cgbn_get_tuning("chunk_bytes")
    try:
        L.cgbn_set_tuning("chunk_bytes", 4096)               # many more row partials per channel
        assert L.cgbn_workspace_bytes(*shape, "NCHW", "f32", 8) > wb
        a = dict(GOOD, N=16, C=64, H=400, W=672, K=8, workspace_bytes=wb)
        with pytest.raises(L.CgbnError) as e:
            L.cgbn_forward(**a)
        assert e.value.code == 6
    finally:
        L.cgbn_set_tuning("chunk_bytes", old)
    assert L.cgbn_workspace_bytes(*shape, "NCHW", "f32", 8) == wb


def test_calls_see_one_consistent_copy_of_the_knobs_under_concurrent_changes():
    """One thread flips a knob that the workspace size depends on while others size workspaces: every answer
    is the size under one setting or under the other, never a mixture, and nothing crashes."""
    import threading
    shape = (8, 48, 300, 500, "NCHW", "f32", 4)
    old = L.cgbn_get_tuning("chunk_bytes")
    sizes = {}
    for v in (8192, 65536):
        L.cgbn_set_tuning("chunk_bytes", v)
        sizes[v] = (L.cgbn_workspace_bytes(*shape), L.cgbn_plan_get(*shape, "rows"))
    assert sizes[8192] != sizes[65536]
    stop, bad = threading.Event(), []

    def flip():
        i = 0
        while not stop.is_set():
            L.cgbn_set_tuning("chunk_bytes", (8192, 65536)[i & 1])
            i += 1

    def size():
        ok_bytes, ok_rows = {s[0] for s in sizes.values()}, {s[1] for s in sizes.values()}
        for _ in range(3000):
            b, r = L.cgbn_workspace_bytes(*shape), L.cgbn_plan_get(*shape, "rows")
            if b not in ok_bytes or r not in ok_rows:
                bad.append((b, r))

    try:
        th = [threading.Thread(target=flip)] + [threading.Thread(target=size) for _ in range(3)]
        for t in th:
            t.start()
        for t in th[1:]:
            t.join()
        stop.set()
        th[0].join()
    finally:
        L.cgbn_set_tuning("chunk_bytes", old)
    assert not bad, bad[:3]


def test_workspace_status_argument_errors_and_fixed_error_offset():
    assert L.cgbn_workspace_error_offset(4, 16, 32, 32, "NCHW", "f32", 2) == 4
    assert L.cgbn_workspace_error_offset(64, 512, 50, 84, "NHWC", "bf16", 32) == 4
    for kw, code in ((dict(workspace=None, gave_up=P), 1), (dict(workspace=P, gave_up=None), 1),
                     (dict(workspace=P + 64, gave_up=P), 6)):
        with pytest.raises(L.CgbnError) as e:
            L.cgbn_workspace_status(stream=0, **kw)
        assert e.value.code == code


def test_forward_static_argument_errors_and_size_limit():
    """The entry point without a workspace: the usual argument errors, and a problem whose scratch would not
    fit the library's static array is refused before anything touches a device."""
    a = {k: v for k, v in GOOD.items() if k not in ("workspace", "workspace_bytes")}

    def code(**kw):
        with pytest.raises(L.CgbnError) as e:
            L.cgbn_forward_static(**dict(a, **kw))
        return e.value.code

    assert code(x=None) == 1 and code(N=0) == 2 and code(K=3) == 3 and code(dtype=9) == 4 and code(eps=0.0) == 5
    assert code(y=P + 4) == 7
    limit = 16 << 20
    big = dict(N=512, C=4096, H=20, W=21, K=256)            # 2 x (C x N floats) + 2 x (K x C doubles) > 16 MiB
    assert L.cgbn_workspace_bytes(big["N"], big["C"], big["H"], big["W"], "NCHW", "f32", big["K"]) > limit
    assert code(**big) == 12
    for shape in [(4, 16, 32, 32, "NCHW", "f32", 2), (16, 64, 400, 672, "NCHW", "f32", 8), (16, 256, 200, 336, "NCHW", "f32", 8),
                  (256, 2048, 25, 42, "NCHW", "f32", 128), (64, 512, 50, 84, "NHWC", "bf16", 32)]:
        assert 0 < L.cgbn_workspace_bytes(*shape) <= limit
