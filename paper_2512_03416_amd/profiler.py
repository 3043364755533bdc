"""Chunk-size profiling of a Convertible Decoder on this GPU (paper Sec. 4.4), attention part.

The paper profiles, per model and hardware, the iteration time of a decoder that runs one restricted
prefill chunk next to its decode batch, raises the chunk size until the TPOT SLO is violated and
keeps the largest size that met it.  This module does that sweep for the attention pass of this
library: a fixed decode batch, one prefill task of growing size, the pass timed on the GPU, the
per-iteration attention time taken as pass time x layers and compared with the share of the TPOT
SLO that attention may use.  The choice, the Convertible Decoder's prefill velocity V_D^{P'} and its
memory reservation come from the library's policy functions (include/tokenscale_policy.h).

    python -m paper_2512_03416_amd.profiler --decode-batch 128 --chunks 128,512,1024,2048,4096,8192

Inputs are seeded and synthetic (workloads.make_batch); every number printed is measured here.
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import asdict, dataclass
from typing import List, Sequence

import numpy as np


@dataclass
class SweepPoint:
    chunk_size: int            # prefill tokens + decode batch size (the paper's definition)
    prefill_tokens: int
    pass_ms: float             # one attention pass (one layer)
    iteration_attention_ms: float   # pass_ms x layers
    decode_only_ratio: float   # pass time relative to the decode-only pass


def time_pass(shape, q_lens, ctx_lens, seed: int, steps: int, warmup: int, options=None) -> float:
    """Milliseconds per ts_mixed_paged_attention call (KV append included) on a seeded batch; options: names and
    values for ts_set_option."""
    import torch
    import paper_2512_03416_amd as ts
    from workloads import make_batch
    batch = make_batch(shape, q_lens, ctx_lens, seed=seed, pool_rule=1.1, value_mult=0.5, device="cuda")
    desc = ts.Desc.make(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, shape.q_dtype, shape.kv_dtype,
                        batch.num_pages, batch.max_pages_per_seq)
    ctx = ts.Context(desc)
    for name, value in (options or {}).items():
        ctx.set_option(name, value)
    nbytes = ts.cache_bytes(desc)
    kc = torch.zeros((nbytes,), dtype=torch.uint8, device="cuda")
    vc = torch.zeros((nbytes,), dtype=torch.uint8, device="cuda")
    bt = torch.from_numpy(batch.block_table).cuda()
    pre = batch.prefix_lens
    if int(pre.sum()):
        ctx.kv_append(batch.k_prefix, batch.v_prefix, kc, vc, batch.k_scale, batch.v_scale, bt, pre, pre)
    out = torch.zeros((batch.total_q, shape.num_q_heads, shape.head_dim), dtype=batch.q.dtype, device="cuda")

    def step():
        ctx.mixed_paged_attention(batch.q, batch.k_new, batch.v_new, kc, vc, batch.k_scale, batch.v_scale, bt,
                                  batch.q_lens, batch.ctx_lens, batch.sm_scale, out)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ctx.close()
    return ms


def sweep(shape, decode_ctx: Sequence[int], chunk_sizes: Sequence[int], prefill_prefix: int, layers: int,
          seed: int = 7, steps: int = 30, warmup: int = 5, options=None) -> List[SweepPoint]:
    """Times the pass for the decode batch alone and with one prefill task per chunk size (ascending)."""
    batch_size = len(decode_ctx)
    base = time_pass(shape, [1] * batch_size, list(decode_ctx), seed, steps, warmup, options)
    points = []
    for c in sorted(chunk_sizes):
        n_pf = c - batch_size
        if n_pf <= 0:
            raise ValueError(f"chunk size {c} leaves no room for prefill next to {batch_size} decode rows")
        q_lens = [1] * batch_size + [n_pf]
        ctx_lens = list(decode_ctx) + [prefill_prefix + n_pf]
        ms = time_pass(shape, q_lens, ctx_lens, seed, steps, warmup, options)
        points.append(SweepPoint(c, n_pf, ms, ms * layers, ms / base))
        print(f"[profiler] chunk {c:6d} ({n_pf:6d} prefill tokens): {ms:8.3f} ms per pass, "
              f"{ms * layers:8.2f} ms per iteration, {ms / base:5.2f} x decode-only", file=sys.stderr, flush=True)
    return points


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--heads", default="32,8", help="query heads, kv heads")
    ap.add_argument("--kv", default="bf16", choices=["bf16", "fp8"])
    ap.add_argument("--decode-batch", type=int, default=128)
    ap.add_argument("--ctx-min", type=int, default=1024)
    ap.add_argument("--ctx-max", type=int, default=8192)
    ap.add_argument("--prefill-prefix", type=int, default=0, help="tokens of the prefill task already cached")
    ap.add_argument("--chunks", default="256,512,1024,2048,4096,8192")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--tpot-slo-ms", type=float, default=100.0, help="TPOT SLO (paper Sec. 5: 100 ms)")
    ap.add_argument("--ttft-slo-ms", type=float, default=400.0, help="TTFT SLO used for the memory reservation")
    ap.add_argument("--attention-share", type=float, default=0.3,
                    help="fraction of the TPOT SLO the attention passes of an iteration may use")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--seed", type=int, default=7)
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="library option for every pass (ts_set_option), e.g. mixed_mode=1; may be repeated")
    args = ap.parse_args(argv)
    options = {k: int(v) for k, v in (o.split("=", 1) for o in args.option)}

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("the profiler measures on a GPU")
    import paper_2512_03416_amd as ts
    from paper_2512_03416_amd import policy
    from workloads import AttnShape
    hq, hkv = (int(x) for x in args.heads.split(","))
    shape = AttnShape(hq, hkv, 128, "bf16", args.kv)
    rng = np.random.default_rng(args.seed)
    decode_ctx = rng.integers(args.ctx_min, args.ctx_max + 1, args.decode_batch).tolist()
    chunks = [int(x) for x in args.chunks.split(",")]
    pts = sweep(shape, decode_ctx, chunks, args.prefill_prefix, args.layers, args.seed, args.steps, options=options)

    budget_s = args.tpot_slo_ms * 1e-3 * args.attention_share
    idx = policy.tv_largest_chunk([p.iteration_attention_ms * 1e-3 for p in pts], budget_s)
    desc = ts.Desc.make(hq, hkv, 128, "bf16", args.kv, 1, 1)
    mem_t = policy.tv_token_bytes(desc, args.layers)
    result = dict(shape=f"{hq}q/{hkv}kv/d128 kv={args.kv}", decode_batch=args.decode_batch,
                  decode_ctx=[args.ctx_min, args.ctx_max], layers=args.layers, tpot_slo_ms=args.tpot_slo_ms,
                  attention_budget_ms=budget_s * 1e3, options=options, sweep=[asdict(p) for p in pts], chosen_index=idx)
    if idx >= 0:
        c = pts[idx].chunk_size
        v = policy.tv_convertible_prefill_velocity(c, args.decode_batch, args.tpot_slo_ms * 1e-3)
        result.update(chunk_size=c, prefill_velocity_tok_per_s=v, token_bytes=mem_t,
                      reserved_bytes=policy.tv_reserved_memory(v, mem_t, args.ttft_slo_ms * 1e-3))
    print(json.dumps(result))
    return result


if __name__ == "__main__":
    main()
