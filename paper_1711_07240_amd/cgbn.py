"""ctypes binding of libcgbn.so: same names and argument order as include/cgbn.h.

Argument marshalling only.  Tensors are passed as anything with a
`data_ptr()` (a torch tensor on the GPU) or as a raw integer device address;
`None` becomes NULL.  Every step of the path runs in the library's kernels.
If the library has not been built this module raises on first use; there is
no fallback of any kind.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcgbn.so")

CGBN_NCHW, CGBN_NHWC = 0, 1
CGBN_F32, CGBN_BF16 = 0, 1
CGBN_OK = 0

LAYOUTS = {"NCHW": CGBN_NCHW, "NHWC": CGBN_NHWC}
DTYPES = {"f32": CGBN_F32, "bf16": CGBN_BF16}

_c_int, _c_ll, _c_f, _c_sz, _c_p = (ctypes.c_int, ctypes.c_longlong, ctypes.c_float,
                                     ctypes.c_size_t, ctypes.c_void_p)

# name -> (restype, argtypes); mirrors include/cgbn.h declaration by declaration
SIGNATURES = {
    "cgbn_workspace_bytes": (_c_sz, [_c_int] * 4 + [_c_int, _c_int, _c_int]),
    "cgbn_workspace_error_offset": (_c_sz, [_c_int] * 4 + [_c_int, _c_int, _c_int]),
    "cgbn_workspace_status": (_c_int, [_c_p, _c_p, _c_p]),
    "cgbn_forward": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int, _c_p, _c_p, _c_f,
                              _c_p, _c_p, _c_p, _c_int, _c_p, _c_p, _c_sz, _c_p]),
    "cgbn_forward_static": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int, _c_p, _c_p, _c_f,
                                     _c_p, _c_p, _c_p, _c_int, _c_p, _c_p]),
    "cgbn_backward": (_c_int, [_c_p] * 8 + [_c_int] * 4 + [_c_int, _c_int, _c_int, _c_p,
                               _c_p, _c_sz, _c_p]),
    "cgbn_forward_relu": (_c_int, [_c_p, _c_p] + [_c_int] * 4 + [_c_int, _c_int, _c_p, _c_p, _c_f,
                                   _c_p, _c_p, _c_p, _c_int, _c_p, _c_p, _c_sz, _c_p]),
    "cgbn_backward_relu": (_c_int, [_c_p] * 10 + [_c_int] * 4 + [_c_int, _c_int, _c_int, _c_p,
                                    _c_p, _c_sz, _c_p]),
    "cgbn_shard_sum": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int, _c_int, _c_p,
                                _c_p, _c_sz, _c_p]),
    "cgbn_reduce_mean": (_c_int, [_c_p, _c_int, _c_int, _c_ll, _c_p, _c_p, _c_p]),
    "cgbn_shard_sqdev": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int, _c_int, _c_p, _c_p, _c_p,
                                  _c_p, _c_sz, _c_p]),
    "cgbn_reduce_invstd": (_c_int, [_c_p, _c_int, _c_int, _c_ll, _c_f, _c_p, _c_p]),
    "cgbn_normalize": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int] + [_c_p] * 7),
    "cgbn_backward_shard_sums": (_c_int, [_c_p, _c_p] + [_c_int] * 4 + [_c_int, _c_int, _c_int]
                                 + [_c_p] * 5 + [_c_p, _c_sz, _c_p]),
    "cgbn_backward_reduce": (_c_int, [_c_p, _c_p, _c_int, _c_int, _c_p, _c_p, _c_p]),
    "cgbn_backward_dx": (_c_int, [_c_p, _c_p] + [_c_int] * 4 + [_c_int, _c_int] + [_c_p] * 8),
    "cgbn_frozen_forward": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int] + [_c_p] * 4 + [_c_f, _c_p, _c_p]),
    "cgbn_frozen_backward": (_c_int, [_c_p] + [_c_int] * 4 + [_c_int, _c_int] + [_c_p] * 2 + [_c_f, _c_p, _c_p]),
    "cgbn_update_running_stats": (_c_int, [_c_p, _c_p, _c_p, _c_f, _c_ll, _c_int, _c_f, _c_int, _c_p, _c_p, _c_p]),
    "cgbn_calibration_copy": (_c_int, [_c_p, _c_p, _c_sz, _c_p]),
    "cgbn_status_string": (ctypes.c_char_p, [_c_int]),
    "cgbn_set_tuning": (_c_int, [ctypes.c_char_p, _c_ll]),
    "cgbn_get_tuning": (_c_ll, [ctypes.c_char_p]),
    "cgbn_plan_get": (_c_ll, [_c_int] * 4 + [_c_int, _c_int, _c_int, ctypes.c_char_p]),
}

_lib = None


class CgbnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


def lib() -> ctypes.CDLL:
    """Load libcgbn.so (once).  Raises if it is missing: build it first."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                "or `python paper_1711_07240_amd/build.py`")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _nbytes(t) -> int:
    return int(t.numel() * t.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _enum(table, v) -> int:
    return table[v] if isinstance(v, str) else int(v)


def _check(code: int, where: str) -> None:
    if code != CGBN_OK:
        raise CgbnError(code, where)


def status_string(code: int) -> str:
    return lib().cgbn_status_string(int(code)).decode()


def cgbn_status_string(code: int) -> str:
    return status_string(code)


def cgbn_workspace_bytes(N, C, H, W, layout, dtype, K) -> int:
    return int(lib().cgbn_workspace_bytes(N, C, H, W, _enum(LAYOUTS, layout), _enum(DTYPES, dtype), K))


def cgbn_workspace_error_offset(N, C, H, W, layout, dtype, K) -> int:
    return int(lib().cgbn_workspace_error_offset(N, C, H, W, _enum(LAYOUTS, layout), _enum(DTYPES, dtype), K))


def cgbn_workspace_status(workspace, gave_up, stream=None) -> None:
    _check(lib().cgbn_workspace_status(_ptr(workspace), _ptr(gave_up), _stream(stream)), "cgbn_workspace_status")


def cgbn_forward(x, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd,
                 dtype="f32", mean_lo=None, workspace=None, workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_forward(_ptr(x), N, C, H, W, _enum(LAYOUTS, layout), K, _ptr(gamma), _ptr(beta),
                              float(eps), _ptr(y), _ptr(mean), _ptr(invstd), _enum(DTYPES, dtype),
                              _ptr(mean_lo), _ptr(workspace), wb, _stream(stream)), "cgbn_forward")


def cgbn_forward_static(x, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd,
                        dtype="f32", mean_lo=None, stream=None) -> None:
    _check(lib().cgbn_forward_static(_ptr(x), N, C, H, W, _enum(LAYOUTS, layout), K, _ptr(gamma), _ptr(beta),
                                     float(eps), _ptr(y), _ptr(mean), _ptr(invstd), _enum(DTYPES, dtype),
                                     _ptr(mean_lo), _stream(stream)), "cgbn_forward_static")


def cgbn_backward(dy, x, mean, invstd, gamma, dx, dgamma, dbeta, N, C, H, W, layout, K,
                  dtype="f32", mean_lo=None, workspace=None, workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_backward(_ptr(dy), _ptr(x), _ptr(mean), _ptr(invstd), _ptr(gamma), _ptr(dx),
                               _ptr(dgamma), _ptr(dbeta), N, C, H, W, _enum(LAYOUTS, layout), K,
                               _enum(DTYPES, dtype), _ptr(mean_lo), _ptr(workspace), wb,
                               _stream(stream)), "cgbn_backward")


def cgbn_forward_relu(x, shortcut, N, C, H, W, layout, K, gamma, beta, eps, y, mean, invstd,
                      dtype="f32", mean_lo=None, workspace=None, workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_forward_relu(_ptr(x), _ptr(shortcut), N, C, H, W, _enum(LAYOUTS, layout), K, _ptr(gamma),
                                   _ptr(beta), float(eps), _ptr(y), _ptr(mean), _ptr(invstd), _enum(DTYPES, dtype),
                                   _ptr(mean_lo), _ptr(workspace), wb, _stream(stream)), "cgbn_forward_relu")


def cgbn_backward_relu(dy, y, x, mean, invstd, gamma, dx, dshortcut, dgamma, dbeta, N, C, H, W, layout, K,
                       dtype="f32", mean_lo=None, workspace=None, workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_backward_relu(_ptr(dy), _ptr(y), _ptr(x), _ptr(mean), _ptr(invstd), _ptr(gamma), _ptr(dx),
                                    _ptr(dshortcut), _ptr(dgamma), _ptr(dbeta), N, C, H, W,
                                    _enum(LAYOUTS, layout), K, _enum(DTYPES, dtype), _ptr(mean_lo),
                                    _ptr(workspace), wb, _stream(stream)), "cgbn_backward_relu")


def cgbn_shard_sum(x, N, C, H, W, layout, K, dtype, s, workspace, workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_shard_sum(_ptr(x), N, C, H, W, _enum(LAYOUTS, layout), K, _enum(DTYPES, dtype),
                                _ptr(s), _ptr(workspace), wb, _stream(stream)), "cgbn_shard_sum")


def cgbn_reduce_mean(s, K, C, M, mean, mean_lo=None, stream=None) -> None:
    _check(lib().cgbn_reduce_mean(_ptr(s), K, C, int(M), _ptr(mean), _ptr(mean_lo), _stream(stream)),
           "cgbn_reduce_mean")


def cgbn_shard_sqdev(x, N, C, H, W, layout, K, dtype, mean, mean_lo, v, workspace,
                     workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_shard_sqdev(_ptr(x), N, C, H, W, _enum(LAYOUTS, layout), K, _enum(DTYPES, dtype),
                                  _ptr(mean), _ptr(mean_lo), _ptr(v), _ptr(workspace), wb,
                                  _stream(stream)), "cgbn_shard_sqdev")


def cgbn_reduce_invstd(v, K, C, M, eps, invstd, stream=None) -> None:
    _check(lib().cgbn_reduce_invstd(_ptr(v), K, C, int(M), float(eps), _ptr(invstd), _stream(stream)),
           "cgbn_reduce_invstd")


def cgbn_normalize(x, N, C, H, W, layout, dtype, mean, mean_lo, invstd, gamma, beta, y, stream=None) -> None:
    _check(lib().cgbn_normalize(_ptr(x), N, C, H, W, _enum(LAYOUTS, layout), _enum(DTYPES, dtype),
                                _ptr(mean), _ptr(mean_lo), _ptr(invstd), _ptr(gamma), _ptr(beta),
                                _ptr(y), _stream(stream)), "cgbn_normalize")


def cgbn_backward_shard_sums(dy, x, N, C, H, W, layout, K, dtype, mean, mean_lo, invstd, a, b,
                             workspace, workspace_bytes=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None and workspace is not None else (workspace_bytes or 0)
    _check(lib().cgbn_backward_shard_sums(_ptr(dy), _ptr(x), N, C, H, W, _enum(LAYOUTS, layout), K,
                                          _enum(DTYPES, dtype), _ptr(mean), _ptr(mean_lo), _ptr(invstd),
                                          _ptr(a), _ptr(b), _ptr(workspace), wb, _stream(stream)),
           "cgbn_backward_shard_sums")


def cgbn_backward_reduce(a, b, K, C, dbeta, dgamma, stream=None) -> None:
    _check(lib().cgbn_backward_reduce(_ptr(a), _ptr(b), K, C, _ptr(dbeta), _ptr(dgamma), _stream(stream)),
           "cgbn_backward_reduce")


def cgbn_backward_dx(dy, x, N, C, H, W, layout, dtype, mean, mean_lo, invstd, gamma, dgamma, dbeta, dx,
                     stream=None) -> None:
    _check(lib().cgbn_backward_dx(_ptr(dy), _ptr(x), N, C, H, W, _enum(LAYOUTS, layout),
                                  _enum(DTYPES, dtype), _ptr(mean), _ptr(mean_lo), _ptr(invstd),
                                  _ptr(gamma), _ptr(dgamma), _ptr(dbeta), _ptr(dx), _stream(stream)),
           "cgbn_backward_dx")


def cgbn_frozen_forward(x, N, C, H, W, layout, dtype, fixed_mean, fixed_var, gamma, beta, eps, y, stream=None) -> None:
    _check(lib().cgbn_frozen_forward(_ptr(x), N, C, H, W, _enum(LAYOUTS, layout), _enum(DTYPES, dtype),
                                     _ptr(fixed_mean), _ptr(fixed_var), _ptr(gamma), _ptr(beta), float(eps),
                                     _ptr(y), _stream(stream)), "cgbn_frozen_forward")


def cgbn_frozen_backward(dy, N, C, H, W, layout, dtype, fixed_var, gamma, eps, dx, stream=None) -> None:
    _check(lib().cgbn_frozen_backward(_ptr(dy), N, C, H, W, _enum(LAYOUTS, layout), _enum(DTYPES, dtype),
                                      _ptr(fixed_var), _ptr(gamma), float(eps), _ptr(dx), _stream(stream)),
           "cgbn_frozen_backward")


def cgbn_update_running_stats(mean, mean_lo, invstd, eps, M, C, momentum, unbiased, running_mean, running_var,
                              stream=None) -> None:
    _check(lib().cgbn_update_running_stats(_ptr(mean), _ptr(mean_lo), _ptr(invstd), float(eps), int(M), int(C),
                                           float(momentum), int(bool(unbiased)), _ptr(running_mean),
                                           _ptr(running_var), _stream(stream)), "cgbn_update_running_stats")


def cgbn_calibration_copy(src, dst, nbytes, stream=None) -> None:
    _check(lib().cgbn_calibration_copy(_ptr(src), _ptr(dst), int(nbytes), _stream(stream)), "cgbn_calibration_copy")


def cgbn_set_tuning(key: str, value: int) -> None:
    _check(lib().cgbn_set_tuning(key.encode(), int(value)), f"cgbn_set_tuning({key!r})")


def cgbn_get_tuning(key: str) -> int:
    return int(lib().cgbn_get_tuning(key.encode()))


def cgbn_plan_get(N, C, H, W, layout, dtype, K, key: str) -> int:
    return int(lib().cgbn_plan_get(N, C, H, W, _enum(LAYOUTS, layout), _enum(DTYPES, dtype), K, key.encode()))
