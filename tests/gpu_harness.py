"""Runs a workloads.Batch through the GPU library (C ABI via the ctypes binding)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_03416_amd as ts

RAW_TORCH = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8": torch.uint8}


def to_dev(batch, device="cuda"):
    for name in ("q", "k_new", "v_new", "k_prefix", "v_prefix", "k_scale", "v_scale"):
        t = getattr(batch, name)
        if t is not None:
            setattr(batch, name, t.to(device).contiguous())
    return batch


def new_caches(batch, device="cuda"):
    sh = batch.shape
    desc = make_desc(batch)
    nbytes = ts.cache_bytes(desc)
    kc = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=device)
    vc = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=device)
    return kc, vc


def make_desc(batch):
    sh = batch.shape
    return ts.Desc.make(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype, sh.kv_dtype,
                        batch.num_pages, batch.max_pages_per_seq)


def cache_raw(t, kv_dtype) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view({"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}[kv_dtype])


def run_batch(batch, ctx=None, with_append=True, fused_append=True, options=None):
    """Fill a fresh cache with the prefix, then one pass.  Returns (out float64 numpy [T,Hq,D],
    k_cache raw numpy, v_cache raw numpy)."""
    batch = to_dev(batch)
    sh = batch.shape
    own = ctx is None
    if own:
        ctx = ts.Context(make_desc(batch))
    for k, v in (options or {}).items():
        ctx.set_option(k, v)
    kc, vc = new_caches(batch)
    bt = torch.from_numpy(batch.block_table).to("cuda").contiguous()
    pre = batch.prefix_lens
    if int(pre.sum()) > 0:
        ctx.kv_append(batch.k_prefix, batch.v_prefix, kc, vc, batch.k_scale, batch.v_scale, bt, pre, pre)
    out = torch.full((batch.total_q, sh.num_q_heads, sh.head_dim), float("nan"), dtype=batch.q.dtype,
                     device="cuda")
    if with_append and not fused_append:
        ctx.kv_append(batch.k_new, batch.v_new, kc, vc, batch.k_scale, batch.v_scale, bt, batch.q_lens,
                      batch.ctx_lens)
    fused = with_append and fused_append
    ctx.mixed_paged_attention(batch.q, batch.k_new if fused else None, batch.v_new if fused else None,
                              kc, vc, batch.k_scale, batch.v_scale, bt, batch.q_lens, batch.ctx_lens,
                              batch.sm_scale, out)
    torch.cuda.synchronize()
    res = out.double().cpu().numpy(), cache_raw(kc, sh.kv_dtype), cache_raw(vc, sh.kv_dtype)
    if own:
        ctx.close()
    return res
