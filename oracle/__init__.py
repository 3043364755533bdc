"""TEST INFRASTRUCTURE: Python face of the fp64 CPU oracle (oracle/ts_oracle.c).

Only tests/, the smoke check and bench.py's cpu_baseline leg may import this package.  It is
independent of the GPU library: nothing here imports it, and nothing in it imports this.

Arrays cross as raw bytes: bf16 tensors are passed as uint16 numpy arrays, fp8 caches as uint8.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ts_oracle.c")
_LIB = os.path.join(_HERE, "libts_oracle.so")

DTYPE_CODE = {"f32": 0, "bf16": 1, "fp8": 2}
ELEM_SIZE = {"f32": 4, "bf16": 2, "fp8": 1}
NP_RAW = {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}
PAGE = 16


class _Desc(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("q_dtype", ctypes.c_int32),
                ("kv_dtype", ctypes.c_int32), ("num_pages", ctypes.c_int64),
                ("max_pages_per_seq", ctypes.c_int32)]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over rows).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.or_e4m3_to_double.restype = ctypes.c_double
        _lib.or_e4m3_to_double.argtypes = [ctypes.c_uint8]
        _lib.or_e4m3_encode.restype = ctypes.c_uint8
        _lib.or_e4m3_encode.argtypes = [ctypes.c_float, ctypes.c_float]
        _lib.or_num_threads.restype = ctypes.c_int
    return _lib


def _ptr(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _desc(Hq, Hkv, D, q_dtype, kv_dtype, num_pages, max_pages):
    return _Desc(Hq, Hkv, D, DTYPE_CODE[q_dtype], DTYPE_CODE[kv_dtype], num_pages, max_pages)


def cache_elems(num_pages: int, Hkv: int, D: int) -> int:
    return num_pages * Hkv * PAGE * D


def new_cache(num_pages: int, Hkv: int, D: int, kv_dtype: str) -> np.ndarray:
    """Flat raw cache buffer with every byte 0xFF (a NaN in all three element types)."""
    a = np.empty(cache_elems(num_pages, Hkv, D), dtype=NP_RAW[kv_dtype])
    a.view(np.uint8)[:] = 0xFF
    return a


def raw(t) -> np.ndarray:
    """torch tensor (cpu) -> contiguous raw numpy array (bf16 as uint16)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype in (getattr(torch, "float8_e4m3fn", None),):
        return t.view(torch.uint8).numpy()
    return t.numpy()


def e4m3_to_double(b: int) -> float:
    return float(lib().or_e4m3_to_double(int(b) & 0xFF))


def e4m3_encode(x: float, scale: float) -> int:
    return int(lib().or_e4m3_encode(ctypes.c_float(x), ctypes.c_float(scale)))


def kv_append(Hq, Hkv, D, q_dtype, kv_dtype, k_new, v_new, k_cache, v_cache, k_scale, v_scale,
              block_table, q_lens, ctx_lens, num_pages) -> None:
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    ql = np.ascontiguousarray(q_lens, dtype=np.int32)
    cl = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    d = _desc(Hq, Hkv, D, q_dtype, kv_dtype, num_pages, bt.shape[1])
    rc = lib().or_kv_append(ctypes.byref(d), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                            _ptr(k_scale), _ptr(v_scale), _ptr(bt), _ptr(ql), _ptr(cl),
                            ctypes.c_int(len(ql)))
    if rc:
        raise RuntimeError(f"or_kv_append failed: {rc}")


def attention_row(Hq, Hkv, D, q_dtype, kv_dtype, q, k_cache, v_cache, k_scale, v_scale, bt_row,
                  n_keys, q_row, h, sm_scale, num_pages):
    """Returns (weights[n_keys], out[D]) in float64 for one (query row, head)."""
    btr = np.ascontiguousarray(bt_row, dtype=np.int32)
    d = _desc(Hq, Hkv, D, q_dtype, kv_dtype, num_pages, len(btr))
    w = np.zeros(max(n_keys, 1), dtype=np.float64)
    out = np.zeros(D, dtype=np.float64)
    rc = lib().or_attention_row(ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                _ptr(k_scale), _ptr(v_scale), _ptr(btr), ctypes.c_int(n_keys),
                                ctypes.c_int64(q_row), ctypes.c_int(h), ctypes.c_double(sm_scale),
                                _ptr(w), _ptr(out))
    if rc:
        raise RuntimeError(f"or_attention_row failed: {rc}")
    return w[:n_keys], out


def mixed_paged_attention(Hq, Hkv, D, q_dtype, kv_dtype, q, k_cache, v_cache, k_scale, v_scale,
                          block_table, q_lens, ctx_lens, sm_scale, num_pages, row_stride: int = 1,
                          row_offset: int = 0) -> np.ndarray:
    """Attention for every query token from the cache as it stands.  Returns float64 [T,Hq,D]
    (rows not selected by row_stride/row_offset stay NaN)."""
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    ql = np.ascontiguousarray(q_lens, dtype=np.int32)
    cl = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    d = _desc(Hq, Hkv, D, q_dtype, kv_dtype, num_pages, bt.shape[1])
    T = int(ql.sum())
    out = np.full((T, Hq, D), np.nan, dtype=np.float64)
    rc = lib().or_mixed_paged_attention(ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                        _ptr(k_scale), _ptr(v_scale), _ptr(bt), _ptr(ql), _ptr(cl),
                                        ctypes.c_int(len(ql)), ctypes.c_double(sm_scale), _ptr(out),
                                        ctypes.c_int64(row_stride), ctypes.c_int64(row_offset))
    if rc:
        raise RuntimeError(f"or_mixed_paged_attention failed: {rc}")
    return out


def num_threads() -> int:
    return int(lib().or_num_threads())


def run_batch(batch, with_append: bool = True):
    """Convenience for tests: fill a fresh cache with the batch's prefix, append the new
    tokens, attend.  Returns (out float64 [T,Hq,D], k_cache raw, v_cache raw)."""
    sh = batch.shape
    Hq, Hkv, D = sh.num_q_heads, sh.num_kv_heads, sh.head_dim
    kc = new_cache(batch.num_pages, Hkv, D, sh.kv_dtype)
    vc = new_cache(batch.num_pages, Hkv, D, sh.kv_dtype)
    ks = None if batch.k_scale is None else raw(batch.k_scale)
    vs = None if batch.v_scale is None else raw(batch.v_scale)
    pre = batch.prefix_lens
    if int(pre.sum()) > 0:
        kv_append(Hq, Hkv, D, sh.q_dtype, sh.kv_dtype, raw(batch.k_prefix), raw(batch.v_prefix),
                  kc, vc, ks, vs, batch.block_table, pre, pre, batch.num_pages)
    if with_append and batch.total_q > 0:
        kv_append(Hq, Hkv, D, sh.q_dtype, sh.kv_dtype, raw(batch.k_new), raw(batch.v_new), kc, vc,
                  ks, vs, batch.block_table, batch.q_lens, batch.ctx_lens, batch.num_pages)
    out = mixed_paged_attention(Hq, Hkv, D, sh.q_dtype, sh.kv_dtype, raw(batch.q), kc, vc, ks, vs,
                                batch.block_table, batch.q_lens, batch.ctx_lens, batch.sm_scale,
                                batch.num_pages)
    return out, kc, vc
