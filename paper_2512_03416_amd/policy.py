"""ctypes binding of the Token-Velocity policy functions (include/tokenscale_policy.h).

Argument marshalling only: every value is computed by the library.  Same names as the C entry
points without the ts_ prefix.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence, Tuple

import numpy as np

from .binding import Desc, load_library

EXPORTS = ["ts_tv_decode_velocity", "ts_tv_prefillers", "ts_tv_decoders", "ts_tv_regular_decoders",
           "ts_tv_decode_batch", "ts_tv_convertible_prefill_velocity", "ts_tv_reserved_memory",
           "ts_tv_token_bytes", "ts_tv_instances", "ts_tv_largest_chunk", "ts_route_prefill", "ts_route_decode"]

NONE, INVALID = -1, -2
PREFILLER, CONVERTIBLE, QUEUE = 0, 1, 2

_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        d, vp, ci = ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.ts_tv_decode_velocity.argtypes = [vp, ci, d]
        lib.ts_tv_prefillers.argtypes = [d, d, d]
        lib.ts_tv_decoders.argtypes = [vp, vp, ci, vp]
        lib.ts_tv_regular_decoders.argtypes = [d, d]
        lib.ts_tv_decode_batch.argtypes = [d, d]
        lib.ts_tv_convertible_prefill_velocity.argtypes = [d, d, d]
        lib.ts_tv_reserved_memory.argtypes = [d, d, d]
        for n in EXPORTS[:7]:
            getattr(lib, n).restype = d
        lib.ts_tv_token_bytes.argtypes = [ctypes.POINTER(Desc), ci]
        lib.ts_tv_token_bytes.restype = ctypes.c_int64
        lib.ts_tv_instances.argtypes = [d]
        lib.ts_tv_instances.restype = ctypes.c_int64
        lib.ts_tv_largest_chunk.argtypes = [vp, ci, d]
        lib.ts_tv_largest_chunk.restype = ci
        lib.ts_route_prefill.argtypes = [vp, vp, ci, vp, vp, ci, d, ctypes.POINTER(ci)]
        lib.ts_route_prefill.restype = ci
        lib.ts_route_decode.argtypes = [vp, ci, ci, ci, vp, vp, d]
        lib.ts_route_decode.restype = ci
        _ready = True
    return lib


def _arr(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data) if a.size else ctypes.c_void_p(0)


def tv_decode_velocity(request_tokens: Sequence[int], tpot_s: float) -> float:
    t = _arr(request_tokens, np.int64)
    return _lib().ts_tv_decode_velocity(_ptr(t), len(t), tpot_s)


def tv_prefillers(lam: float, v_p: float, v_bw: float) -> float:
    return _lib().ts_tv_prefillers(lam, v_p, v_bw)


def tv_decoders(lambda_b, v_d_b) -> Tuple[float, np.ndarray]:
    lam, v = _arr(lambda_b, np.float64), _arr(v_d_b, np.float64)
    if lam.shape != v.shape:
        raise ValueError("one velocity per bucket")
    per = np.full(lam.shape, np.nan)
    return _lib().ts_tv_decoders(_ptr(lam), _ptr(v), len(lam), _ptr(per)), per


def tv_regular_decoders(i_d: float, i_d_c: float) -> float:
    return _lib().ts_tv_regular_decoders(i_d, i_d_c)


def tv_decode_batch(available_bytes: float, mean_request_bytes: float) -> float:
    return _lib().ts_tv_decode_batch(available_bytes, mean_request_bytes)


def tv_convertible_prefill_velocity(chunk_size: float, batch_size: float, tpot_slo_s: float) -> float:
    return _lib().ts_tv_convertible_prefill_velocity(chunk_size, batch_size, tpot_slo_s)


def tv_reserved_memory(v_d_p: float, mem_t_bytes: float, ttft_slo_s: float) -> float:
    return _lib().ts_tv_reserved_memory(v_d_p, mem_t_bytes, ttft_slo_s)


def tv_token_bytes(desc: Desc, num_layers: int) -> int:
    return _lib().ts_tv_token_bytes(ctypes.byref(desc), num_layers)


def tv_instances(requirement: float) -> int:
    return _lib().ts_tv_instances(requirement)


def tv_largest_chunk(iteration_time_s, tpot_slo_s: float) -> int:
    t = _arr(iteration_time_s, np.float64)
    return _lib().ts_tv_largest_chunk(_ptr(t), len(t), tpot_slo_s)


def route_prefill(prefiller_inflight, prefiller_velocity, conv_inflight, conv_velocity,
                  slo_s: float) -> Tuple[int, int]:
    """(kind, index) with kind one of PREFILLER, CONVERTIBLE, QUEUE; index NONE for the queue."""
    pi, pv = _arr(prefiller_inflight, np.float64), _arr(prefiller_velocity, np.float64)
    di, dv = _arr(conv_inflight, np.float64), _arr(conv_velocity, np.float64)
    if pi.shape != pv.shape or di.shape != dv.shape:
        raise ValueError("one velocity per instance")
    kind = ctypes.c_int(-1)
    idx = _lib().ts_route_prefill(_ptr(pi), _ptr(pv), len(pi), _ptr(di), _ptr(dv), len(di), slo_s,
                                  ctypes.byref(kind))
    return kind.value, idx


def route_decode(inflight_by_type, request_type: int, convertible, mem_util, mem_threshold: float,
                 n_types: Optional[int] = None) -> int:
    inf = _arr(inflight_by_type, np.int32)
    if inf.ndim != 2:
        inf = inf.reshape(0, n_types or 1)
    conv, util = _arr(convertible, np.uint8), _arr(mem_util, np.float64)
    if len(conv) != inf.shape[0] or len(util) != inf.shape[0]:
        raise ValueError("one flag and one utilisation per decoder")
    return _lib().ts_route_decode(_ptr(inf), inf.shape[0], inf.shape[1], request_type, _ptr(conv),
                                  _ptr(util), mem_threshold)
