"""ctypes binding with the same names as include/tokenscale.h (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtokenscale.so")

DTYPES = {"f32": 0, "bf16": 1, "fp8": 2}
TS_OK, TS_ERR_INVALID_ARG, TS_ERR_UNSUPPORTED, TS_ERR_HIP, TS_ERR_NOMEM = 0, -1, -2, -3, -4
TS_VELOCITY_RESET, TS_VELOCITY_SYNC = 1, 2

EXPORTS = ["ts_check_desc", "ts_cache_bytes", "ts_create", "ts_destroy", "ts_reserve", "ts_kv_append",
           "ts_mixed_paged_attention", "ts_mixed_paged_attention_noalloc", "ts_token_velocity", "ts_last_error", "ts_set_option",
           "ts_get_option", "ts_plan_describe", "ts_plan_export", "ts_kernel_times"]
CALIB_EXPORTS = ["ts_calib_copy", "ts_calib_read", "ts_calib_mfma"]     # include/tokenscale_calib.h

KERNEL_NAMES = ["append", "decode", "combine", "prefill", "rows", "mixed"]


class TokenScaleError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"tokenscale error {code}: {msg}")
        self.code = code


class Desc(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("q_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
                ("num_pages", ctypes.c_int64), ("max_pages_per_seq", ctypes.c_int32)]

    @classmethod
    def make(cls, Hq, Hkv, D, q_dtype, kv_dtype, num_pages, max_pages_per_seq, page_size=16):
        qd = DTYPES[q_dtype] if isinstance(q_dtype, str) else int(q_dtype)
        kd = DTYPES[kv_dtype] if isinstance(kv_dtype, str) else int(kv_dtype)
        return cls(Hq, Hkv, D, page_size, qd, kd, num_pages, max_pages_per_seq)


class Velocity(ctypes.Structure):
    _fields_ = [("prefill_tok_per_s", ctypes.c_double), ("decode_tok_per_s", ctypes.c_double),
                ("prefill_tokens", ctypes.c_uint64), ("decode_tokens", ctypes.c_uint64),
                ("passes", ctypes.c_uint64), ("window_s", ctypes.c_double)]


class KernelStats(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_uint64 * 6), ("mean_ms", ctypes.c_double * 6)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("total_tokens", ctypes.c_int64), ("decode_tokens", ctypes.c_int64),
                ("prefill_tokens", ctypes.c_int64), ("n_decode_items", ctypes.c_int32),
                ("n_combine_rows", ctypes.c_int32), ("n_prefill_tiles", ctypes.c_int32),
                ("n_generic_rows", ctypes.c_int32), ("split_pages", ctypes.c_int32),
                ("tile_tokens", ctypes.c_int32), ("partial_slots", ctypes.c_int64),
                ("ctx_pages", ctypes.c_int64), ("mixed_mode", ctypes.c_int32), ("prefill_workgroups", ctypes.c_int32),
                ("widened_pages", ctypes.c_int64), ("prefill_parts", ctypes.c_int64)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2512_03416_amd.build` "
                          "or __graft_entry__.build(); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32p = ctypes.c_void_p, ctypes.c_void_p
    lib.ts_check_desc.argtypes = [ctypes.POINTER(Desc)]
    lib.ts_check_desc.restype = ctypes.c_int
    lib.ts_cache_bytes.argtypes = [ctypes.POINTER(Desc)]
    lib.ts_cache_bytes.restype = ctypes.c_int64
    lib.ts_create.argtypes = [ctypes.POINTER(Desc), ctypes.c_int, ctypes.POINTER(vp)]
    lib.ts_create.restype = ctypes.c_int
    lib.ts_destroy.argtypes = [vp]
    lib.ts_destroy.restype = ctypes.c_int
    lib.ts_reserve.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    lib.ts_reserve.restype = ctypes.c_int
    lib.ts_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32p, i32p, ctypes.c_int]
    lib.ts_kv_append.restype = ctypes.c_int
    lib.ts_mixed_paged_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32p, i32p,
                                             ctypes.c_int, ctypes.c_float, vp]
    lib.ts_mixed_paged_attention.restype = ctypes.c_int
    lib.ts_mixed_paged_attention_noalloc.argtypes = lib.ts_mixed_paged_attention.argtypes
    lib.ts_mixed_paged_attention_noalloc.restype = ctypes.c_int
    lib.ts_token_velocity.argtypes = [vp, ctypes.POINTER(Velocity), ctypes.c_int]
    lib.ts_token_velocity.restype = ctypes.c_int
    lib.ts_last_error.argtypes = [vp]
    lib.ts_last_error.restype = ctypes.c_char_p
    lib.ts_set_option.argtypes = [vp, ctypes.c_char_p, ctypes.c_int64]
    lib.ts_set_option.restype = ctypes.c_int
    lib.ts_get_option.argtypes = [vp, ctypes.c_char_p, ctypes.POINTER(ctypes.c_int64)]
    lib.ts_get_option.restype = ctypes.c_int
    lib.ts_plan_describe.argtypes = [ctypes.POINTER(Desc), i32p, i32p, ctypes.c_int, ctypes.c_int32,
                                     ctypes.POINTER(PlanInfo)]
    lib.ts_plan_describe.restype = ctypes.c_int
    lib.ts_plan_export.argtypes = [ctypes.POINTER(Desc), i32p, i32p, ctypes.c_int, ctypes.c_int32,
                                   ctypes.c_int32, ctypes.c_int32, ctypes.c_int, i32p, ctypes.c_int64]
    lib.ts_plan_export.restype = ctypes.c_int64
    lib.ts_kernel_times.argtypes = [vp, ctypes.POINTER(KernelStats), ctypes.c_int]
    lib.ts_kernel_times.restype = ctypes.c_int
    lib.ts_calib_copy.argtypes = [vp, vp, vp, ctypes.c_int64]
    lib.ts_calib_copy.restype = ctypes.c_int
    lib.ts_calib_read.argtypes = [vp, vp, vp, ctypes.c_int64]
    lib.ts_calib_read.restype = ctypes.c_int
    lib.ts_calib_mfma.argtypes = [vp, vp, vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
    lib.ts_calib_mfma.restype = ctypes.c_int
    _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _np_ptr(a: Optional[np.ndarray]):
    return ctypes.c_void_p(a.ctypes.data if a is not None and a.size else 0) if a is not None else ctypes.c_void_p(0)


def _dev_ptr(t) -> ctypes.c_void_p:
    """Device pointer of a torch tensor (or None / int)."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_cuda:
        raise ValueError("expected a GPU tensor")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def check_desc(desc: Desc) -> int:
    return int(load_library().ts_check_desc(ctypes.byref(desc)))


def cache_bytes(desc: Desc) -> int:
    return int(load_library().ts_cache_bytes(ctypes.byref(desc)))


def plan_describe(desc: Desc, q_lens, ctx_lens, split_pages: int = 0) -> PlanInfo:
    ql, cl = _i32(q_lens), _i32(ctx_lens)
    info = PlanInfo()
    rc = load_library().ts_plan_describe(ctypes.byref(desc), _np_ptr(ql), _np_ptr(cl), len(ql),
                                         split_pages, ctypes.byref(info))
    if rc != TS_OK:
        raise TokenScaleError(rc, "ts_plan_describe")
    return info


PLAN_LISTS = {"decode": (0, 8), "combine": (1, 4), "prefill": (2, 12), "pfmap": (3, 2), "rows": (4, 4),
              "queue": (5, 4), "qoff": (6, 1), "append": (7, 8),
              "append_rows": (8, 4), "widen": (9, 2), "pfcombine": (10, 4)}


def plan_export(desc: Desc, q_lens, ctx_lens, which: str, split_pages: int = 0, wg_slots: int = 0,
                mixed_mode: int = -1) -> np.ndarray:
    """One of the planner's work lists as an int32 array [records, words] (see tokenscale.h)."""
    ql, cl = _i32(q_lens), _i32(ctx_lens)
    lib = load_library()
    code, words = PLAN_LISTS[which]
    n = lib.ts_plan_export(ctypes.byref(desc), _np_ptr(ql), _np_ptr(cl), len(ql), split_pages, wg_slots, mixed_mode,
                           code, ctypes.c_void_p(0), 0)
    if n < 0:
        raise TokenScaleError(int(n), "ts_plan_export")
    out = np.zeros((int(n), words), dtype=np.int32)
    if n:
        lib.ts_plan_export(ctypes.byref(desc), _np_ptr(ql), _np_ptr(cl), len(ql), split_pages, wg_slots, mixed_mode,
                           code, _np_ptr(out), int(n) * words)
    return out


def plan_decode_items(desc: Desc, q_lens, ctx_lens, split_pages: int = 0) -> np.ndarray:
    return plan_export(desc, q_lens, ctx_lens, "decode", split_pages)[:, :5]


class Context:
    """Owns a ts_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, desc: Desc, device: int = 0):
        self._lib = load_library()
        self.desc = desc
        self._h = ctypes.c_void_p(0)
        rc = self._lib.ts_create(ctypes.byref(desc), device, ctypes.byref(self._h))
        if rc != TS_OK:
            msg = self._lib.ts_last_error(ctypes.c_void_p(0)).decode()
            self._h = ctypes.c_void_p(0)
            raise TokenScaleError(rc, msg)

    def close(self):
        if self._h:
            self._lib.ts_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self._lib.ts_last_error(self._h).decode()

    def _check(self, rc: int):
        if rc != TS_OK:
            raise TokenScaleError(rc, self.last_error())

    @staticmethod
    def _stream(stream) -> ctypes.c_void_p:
        if stream is None:
            import torch
            return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if isinstance(stream, int):
            return ctypes.c_void_p(stream)
        return ctypes.c_void_p(stream.cuda_stream)

    def reserve(self, max_tokens: int, max_seqs: int, max_ctx_pages: int):
        self._check(self._lib.ts_reserve(self._h, max_tokens, max_seqs, max_ctx_pages))

    def set_option(self, name: str, value: int):
        self._check(self._lib.ts_set_option(self._h, name.encode(), int(value)))

    def get_option(self, name: str) -> int:
        v = ctypes.c_int64(0)
        rc = self._lib.ts_get_option(self._h, name.encode(), ctypes.byref(v))
        if rc != TS_OK:
            raise TokenScaleError(rc, f"ts_get_option({name})")
        return int(v.value)

    def kv_append(self, k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table, q_lens,
                  ctx_lens, stream=None):
        ql, cl = _i32(q_lens), _i32(ctx_lens)
        self._check(self._lib.ts_kv_append(self._h, self._stream(stream), _dev_ptr(k_new), _dev_ptr(v_new),
                                           _dev_ptr(k_cache), _dev_ptr(v_cache), _dev_ptr(k_scale),
                                           _dev_ptr(v_scale), _dev_ptr(block_table), _np_ptr(ql),
                                           _np_ptr(cl), len(ql)))

    def mixed_paged_attention(self, q, k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table,
                              q_lens, ctx_lens, sm_scale: float, out, stream=None, noalloc: bool = False):
        """noalloc=True calls ts_mixed_paged_attention_noalloc (same arguments)."""
        ql, cl = _i32(q_lens), _i32(ctx_lens)
        fn = self._lib.ts_mixed_paged_attention_noalloc if noalloc else self._lib.ts_mixed_paged_attention
        self._check(fn(
            self._h, self._stream(stream), _dev_ptr(q), _dev_ptr(k_new), _dev_ptr(v_new),
            _dev_ptr(k_cache), _dev_ptr(v_cache), _dev_ptr(k_scale), _dev_ptr(v_scale),
            _dev_ptr(block_table), _np_ptr(ql), _np_ptr(cl), len(ql), ctypes.c_float(sm_scale),
            _dev_ptr(out)))

    def kernel_times(self, reset: bool = False) -> dict:
        """{kernel name: (launches, mean ms)} of the launches timed since the last reset."""
        st = KernelStats()
        self._check(self._lib.ts_kernel_times(self._h, ctypes.byref(st), 1 if reset else 0))
        return {n: (int(st.launches[i]), float(st.mean_ms[i])) for i, n in enumerate(KERNEL_NAMES)}

    def token_velocity(self, reset: bool = False, sync: bool = False) -> Velocity:
        v = Velocity()
        flags = (TS_VELOCITY_RESET if reset else 0) | (TS_VELOCITY_SYNC if sync else 0)
        self._check(self._lib.ts_token_velocity(self._h, ctypes.byref(v), flags))
        return v


def calib_copy(src, dst, nbytes: int, stream=None):
    rc = load_library().ts_calib_copy(Context._stream(stream), _dev_ptr(src), _dev_ptr(dst), nbytes)
    if rc != TS_OK:
        raise TokenScaleError(rc, "ts_calib_copy")


def calib_read(src, result4, nbytes: int, stream=None):
    rc = load_library().ts_calib_read(Context._stream(stream), _dev_ptr(src), _dev_ptr(result4), nbytes)
    if rc != TS_OK:
        raise TokenScaleError(rc, "ts_calib_read")


def calib_mfma(operands, result4, iters: int, softmax: bool, stream=None) -> int:
    """Launches the MFMA calibration stream; returns the floating-point operations of the launch."""
    flops = ctypes.c_int64(0)
    rc = load_library().ts_calib_mfma(Context._stream(stream), _dev_ptr(operands), _dev_ptr(result4), int(iters),
                                      int(bool(softmax)), ctypes.byref(flops))
    if rc != 0:
        raise TokenScaleError(rc, "ts_calib_mfma")
    return int(flops.value)
