"""Seeded synthetic inputs for the mixed paged-attention pass.

This module only draws lengths, page tables and tensor values.  It holds none of the
method's arithmetic and knows nothing about how the paged cache is laid out in memory:
the cached prefix of every sequence is handed out as *logical* rows ``[tokens, Hkv, D]``
and each consumer (the CPU oracle, the GPU library) fills its own cache from them through
its own append routine.

The batch structure follows the serving iteration of a Convertible Decoder: a decode batch
(one query token per sequence) next to absorbed prefill chunks (many query tokens that
attend causally to their cached prefix and to themselves) -- paper Sec. 3.4 and Sec. 4.4.
Head geometry and length ranges stand in for the Llama-3.1-8B / Qwen-2.5 deployments and
the <= 8192-token inputs of the paper's evaluation (Sec. 5); values are i.i.d. normal.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np
import torch

PAGE = 16  # tokens per KV page

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclass
class AttnShape:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    q_dtype: str   # "f32" | "bf16"      (queries, new K/V rows, outputs)
    kv_dtype: str  # "f32" | "bf16" | "fp8"   (cache elements)

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


@dataclass
class Batch:
    """One iteration's worth of inputs.  Tensors live on ``device``."""
    shape: AttnShape
    q_lens: np.ndarray            # int32 [S] new (query) tokens of each sequence
    ctx_lens: np.ndarray          # int32 [S] keys visible to the LAST query token (includes q_len)
    block_table: np.ndarray       # int32 [S, max_pages_per_seq], -1 = unused
    num_pages: int                # size of the physical page pool
    q: torch.Tensor               # [T, Hq, D]   q_dtype
    k_new: torch.Tensor           # [T, Hkv, D]  q_dtype
    v_new: torch.Tensor           # [T, Hkv, D]  q_dtype
    k_prefix: torch.Tensor        # [sum(prefix), Hkv, D] q_dtype, packed by sequence
    v_prefix: torch.Tensor        # [sum(prefix), Hkv, D] q_dtype
    k_scale: Optional[torch.Tensor]  # fp32 [Hkv] (fp8 cache only)
    v_scale: Optional[torch.Tensor]
    sm_scale: float
    name: str = ""
    notes: dict = field(default_factory=dict)

    @property
    def num_seqs(self) -> int:
        return int(self.q_lens.shape[0])

    @property
    def prefix_lens(self) -> np.ndarray:
        return (self.ctx_lens - self.q_lens).astype(np.int32)

    @property
    def total_q(self) -> int:
        return int(self.q_lens.sum())

    @property
    def max_pages_per_seq(self) -> int:
        return int(self.block_table.shape[1])


def pages_for(n_tokens) -> int:
    return (int(n_tokens) + PAGE - 1) // PAGE


def deal_block_table(ctx_lens: Sequence[int], num_pages: int, rng: np.random.Generator,
                     min_row: int = 1) -> np.ndarray:
    """Random permutation of the pool, dealt out sequence after sequence."""
    need = [pages_for(c) for c in ctx_lens]
    total = int(sum(need))
    if total > num_pages:
        raise ValueError(f"pool of {num_pages} pages cannot hold {total} pages")
    perm = rng.permutation(num_pages)[:total].astype(np.int32)
    width = max(min_row, max(need) if need else 1)
    bt = np.full((len(need), width), -1, dtype=np.int32)
    o = 0
    for s, n in enumerate(need):
        bt[s, :n] = perm[o:o + n]
        o += n
    return bt


def _randn(n_rows: int, heads: int, dim: int, gen: torch.Generator, device, dtype, mult: float,
           chunk_rows: int = 1 << 16) -> torch.Tensor:
    """N(0,1)*mult drawn in fp32 and rounded (nearest-even cast of the library) to dtype."""
    out = torch.empty((n_rows, heads, dim), dtype=dtype, device=device)
    for r0 in range(0, n_rows, chunk_rows):
        r1 = min(n_rows, r0 + chunk_rows)
        x = torch.randn((r1 - r0, heads, dim), generator=gen, device=device, dtype=torch.float32)
        out[r0:r1] = (x * mult).to(dtype)
    return out


def make_batch(shape: AttnShape, q_lens: Sequence[int], ctx_lens: Sequence[int], *, seed: int,
               num_pages: Optional[int] = None, pool_rule: float = 1.0, value_mult: float = 1.0,
               device: str = "cpu", sm_scale: Optional[float] = None, name: str = "custom",
               q_zero: bool = False) -> Batch:
    """General seeded batch: any mix of (q_len, ctx_len) per sequence."""
    q_lens = np.asarray(q_lens, dtype=np.int32)
    ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
    assert q_lens.shape == ctx_lens.shape and np.all(ctx_lens >= q_lens) and np.all(q_lens >= 0)
    rng = np.random.default_rng(seed)
    need = int(sum(pages_for(c) for c in ctx_lens))
    if num_pages is None:
        num_pages = max(1, int(math.ceil(pool_rule * need)))
    num_pages = max(num_pages, need)
    bt = deal_block_table(ctx_lens, num_pages, rng)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    dt = _TORCH_DTYPE[shape.q_dtype]
    T = int(q_lens.sum())
    Pn = int((ctx_lens - q_lens).sum())
    q = _randn(T, shape.num_q_heads, shape.head_dim, gen, dev, dt, value_mult)
    if q_zero:
        q.zero_()
    k_new = _randn(T, shape.num_kv_heads, shape.head_dim, gen, dev, dt, value_mult)
    v_new = _randn(T, shape.num_kv_heads, shape.head_dim, gen, dev, dt, value_mult)
    k_prefix = _randn(Pn, shape.num_kv_heads, shape.head_dim, gen, dev, dt, value_mult)
    v_prefix = _randn(Pn, shape.num_kv_heads, shape.head_dim, gen, dev, dt, value_mult)
    k_scale = v_scale = None
    if shape.kv_dtype == "fp8":
        # one scale per KV head = absmax over everything that head will ever hold / 448
        # (448 = largest finite e4m3 value), so parity inputs never saturate.
        def head_absmax(a, b):
            m = torch.zeros(shape.num_kv_heads, dtype=torch.float32, device=dev)
            for t in (a, b):
                if t.shape[0]:
                    m = torch.maximum(m, t.float().abs().amax(dim=(0, 2)))
            return torch.clamp(m, min=1e-6)
        k_scale = (head_absmax(k_new, k_prefix) / 448.0).contiguous()
        v_scale = (head_absmax(v_new, v_prefix) / 448.0).contiguous()
    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(shape.head_dim)
    return Batch(shape, q_lens, ctx_lens, bt, int(num_pages), q, k_new, v_new, k_prefix, v_prefix,
                 k_scale, v_scale, float(sm_scale), name)


# ----------------------------------------------------------------------------------------------
# The five named configurations.
# ----------------------------------------------------------------------------------------------

LLAMA8B = dict(num_q_heads=32, num_kv_heads=8, head_dim=128)


def _lognormal_int(rng, median, sigma, lo, hi, n):
    z = rng.standard_normal(n)
    v = np.rint(np.exp(math.log(median) + sigma * z))
    return np.clip(v, lo, hi).astype(np.int32)


def config1(seed: int = 0, device: str = "cpu") -> Batch:
    """Tiny fp32 mixed batch: 6 decode rows, chunks (q=37,prefix 0) and (q=64,prefix 48)."""
    shape = AttnShape(4, 1, 64, "f32", "f32")
    rng = np.random.default_rng(seed)
    dec_ctx = rng.integers(1, 201, size=6)
    q_lens = [1] * 6 + [37, 64]
    ctx_lens = list(dec_ctx) + [37, 48 + 64]
    need = sum(pages_for(c) for c in ctx_lens)
    b = make_batch(shape, q_lens, ctx_lens, seed=seed, num_pages=max(64, need), value_mult=1.0,
                   device=device, name="cfg1_tiny_fp32_mixed")
    b.notes["pool_pages"] = b.num_pages
    return b


def config2_lengths(seed: int = 1, n_seqs: int = 256):
    rng = np.random.default_rng(seed)
    ctx = rng.integers(512, 4097, size=n_seqs).astype(np.int32)
    return np.ones(n_seqs, dtype=np.int32), ctx


def config2(seed: int = 1, device: str = "cpu", n_seqs: int = 256) -> Batch:
    """Decode-only, 32/8/128 bf16, 256 sequences, context U[512,4096]."""
    shape = AttnShape(q_dtype="bf16", kv_dtype="bf16", **LLAMA8B)
    q_lens, ctx = config2_lengths(seed, n_seqs)
    need = sum(pages_for(c) for c in ctx)
    pool = max(20000, int(math.ceil(1.25 * need))) if n_seqs == 256 else int(math.ceil(1.25 * need))
    return make_batch(shape, q_lens, ctx, seed=seed, num_pages=pool, value_mult=0.5, device=device,
                      name="cfg2_decode_bf16")


def config3_prompts(seed: int = 2, n_prompts: int = 8):
    rng = np.random.default_rng(seed)
    return _lognormal_int(rng, 1024, 0.8, 128, 8192, n_prompts)


def config3_step(step: int, seed: int = 2, device: str = "cpu", n_prompts: int = 8,
                 chunk: int = 512) -> Optional[Batch]:
    """Step ``step`` of chunked prefill: every prompt with tokens left contributes its next
    ``min(chunk, remaining)`` tokens over a cached prefix of ``chunk*step`` tokens."""
    shape = AttnShape(q_dtype="bf16", kv_dtype="bf16", **LLAMA8B)
    L = config3_prompts(seed, n_prompts)
    q_lens, ctx = [], []
    for l in L:
        done = chunk * step
        if done < l:
            q = min(chunk, int(l) - done)
            q_lens.append(q)
            ctx.append(done + q)
    if not q_lens:
        return None
    return make_batch(shape, q_lens, ctx, seed=seed * 1000 + step, pool_rule=1.25, value_mult=0.5,
                      device=device, name=f"cfg3_prefill_bf16_step{step}")


def config4(seed: int = 3, device: str = "cpu", n_decode: int = 128, n_chunks: int = 4,
            chunk: int = 2048) -> Batch:
    """Convertible-decoder burst: decode rows with context U[1024,8192] plus prefill chunks of
    2048 tokens over cached prefixes U[0,4096], one launch with KV append."""
    shape = AttnShape(q_dtype="bf16", kv_dtype="bf16", **LLAMA8B)
    rng = np.random.default_rng(seed)
    dec = rng.integers(1024, 8193, size=n_decode)
    pre = rng.integers(0, 4097, size=n_chunks)
    q_lens = [1] * n_decode + [chunk] * n_chunks
    ctx = list(dec) + [int(p) + chunk for p in pre]
    return make_batch(shape, q_lens, ctx, seed=seed, pool_rule=1.25, value_mult=0.5, device=device,
                      name="cfg4_burst_bf16")


def config5(seed: int = 4, device: str = "cpu", n_decode: int = 512, n_chunks: int = 16,
            chunk: int = 4096, sigma: float = 0.8) -> Batch:
    """70B-like layer, fp8 e4m3 cache with per-KV-head scales, bf16 queries."""
    shape = AttnShape(64, 8, 128, "bf16", "fp8")
    rng = np.random.default_rng(seed)
    dec = _lognormal_int(rng, 4096, sigma, 256, 32768, n_decode)
    q_lens = [1] * n_decode + [chunk] * n_chunks
    ctx = list(dec) + [chunk] * n_chunks
    return make_batch(shape, q_lens, ctx, seed=seed, pool_rule=1.25, value_mult=1.0, device=device,
                      name="cfg5_70b_fp8kv")


def select_sequences(batch: Batch, idx: Sequence[int], seed: int = 0) -> Batch:
    """The sub-batch made of the given sequences (same logical tensors, a fresh page table of its
    own).  Pure data plumbing: lets a bounded sample of a large batch be handed to another consumer."""
    idx = [int(i) for i in idx]
    pre = batch.prefix_lens
    q_off = np.concatenate([[0], np.cumsum(batch.q_lens)])
    p_off = np.concatenate([[0], np.cumsum(pre)])

    def take(t, off):
        parts = [t[int(off[i]):int(off[i + 1])] for i in idx]
        return torch.cat(parts).contiguous() if parts else t[:0]

    q_lens = batch.q_lens[idx]
    ctx = batch.ctx_lens[idx]
    need = int(sum(pages_for(c) for c in ctx))
    rng = np.random.default_rng(seed)
    bt = deal_block_table(ctx, max(need, 1), rng)
    return Batch(batch.shape, q_lens.astype(np.int32), ctx.astype(np.int32), bt, max(need, 1),
                 take(batch.q, q_off), take(batch.k_new, q_off), take(batch.v_new, q_off),
                 take(batch.k_prefix, p_off), take(batch.v_prefix, p_off), batch.k_scale, batch.v_scale,
                 batch.sm_scale, batch.name + "_sample")


def to_cpu(batch: Batch) -> Batch:
    for name in ("q", "k_new", "v_new", "k_prefix", "v_prefix", "k_scale", "v_scale"):
        t = getattr(batch, name)
        if t is not None:
            setattr(batch, name, t.cpu())
    return batch
