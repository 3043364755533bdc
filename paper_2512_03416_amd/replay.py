"""Synthetic burst replay through one Convertible Decoder's attention pass.

The paper's adaptation experiment (Sec. 6.2) serves stable traffic of 1 request/s and steps to 10
requests/s at t = 10 s.  This module replays that arrival pattern, with seeded lognormal input and
output lengths, against ONE decoder that absorbs every prefill as restricted chunks next to its
decode batch (Sec. 3.4, 4.4: at most one prefill task at a time, chunk size = prefill tokens +
decode batch size), and drives the library with the mixed batch of every iteration.  Simulated time
advances by the measured pass time x layers plus a fixed per-iteration allowance for the rest of
the model.  It reports, per second of simulated time: arrivals, prefill and decode token rates,
queue length, TTFT of the requests whose first token came out in that second.

    python -m paper_2512_03416_amd.replay --seconds 20 --step-at 10 --rps 1,10

No traces, weights or datasets: K/V/Q contents are random, only the batch structure is replayed.

Scheduling rules (readings where the paper is silent): a request becomes the prefill task when a table row
and pages for its input + output are free, in arrival order, the head of the queue is never overtaken; the
iteration that finishes a prefill releases the request's first token, and the request joins the decode batch
from the next iteration on; a request is done after out_len tokens (the first one counts).  `replay` can be
given the time of a pass as a function of the batch (instead of measuring it), which makes the schedule a
function of the arrival list alone, and a callback that sees every pass.
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

PAGE = 16


@dataclass
class Request:
    rid: int
    arrival: float
    in_len: int
    out_len: int
    row: int = -1                  # row of the block table while resident
    cached: int = 0                # tokens in the cache
    generated: int = 0
    first_token_at: Optional[float] = None
    done_at: Optional[float] = None
    pages: List[int] = field(default_factory=list)


def make_arrivals(rng, seconds: float, step_at: float, rps_before: float, rps_after: float,
                  in_median: int, out_median: int, in_max: int, out_max: int) -> List[Request]:
    reqs, t, rid = [], 0.0, 0
    while True:
        rate = rps_before if t < step_at else rps_after
        t += rng.exponential(1.0 / rate)
        if t >= seconds:
            return reqs
        in_len = int(np.clip(rng.lognormal(np.log(in_median), 1.0), 16, in_max))
        out_len = int(np.clip(rng.lognormal(np.log(out_median), 0.7), 4, out_max))
        reqs.append(Request(rid, t, in_len, out_len))
        rid += 1


class Decoder:
    """Cache bookkeeping (pages, block table rows) and the per-iteration call into the library."""

    def __init__(self, hq, hkv, kv, max_resident, max_ctx, chunk_size, seed):
        import torch
        import paper_2512_03416_amd as ts
        self.torch, self.ts = torch, ts
        self.hq, self.hkv, self.chunk_size = hq, hkv, chunk_size
        self.max_pages = (max_ctx + PAGE - 1) // PAGE
        self.num_pages = max_resident * self.max_pages // 2 + self.max_pages
        self.desc = ts.Desc.make(hq, hkv, 128, "bf16", kv, self.num_pages, self.max_pages)
        self.ctx = ts.Context(self.desc)
        nbytes = ts.cache_bytes(self.desc)
        self.kc = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
        self.vc = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        # a pass carries the decode batch (at most max_resident rows) plus a chunk that fills what the chunk size
        # leaves: never more than max(chunk_size, max_resident) rows
        T = max(chunk_size, max_resident)
        self.rows = T
        self.q = (torch.randn(T, hq, 128, generator=gen, device="cuda") * 0.5).to(torch.bfloat16)
        self.k = (torch.randn(T, hkv, 128, generator=gen, device="cuda") * 0.5).to(torch.bfloat16)
        self.v = (torch.randn(T, hkv, 128, generator=gen, device="cuda") * 0.5).to(torch.bfloat16)
        self.out = torch.zeros(T, hq, 128, dtype=torch.bfloat16, device="cuda")
        self.scale = torch.full((hkv,), 4.0 / 448.0, dtype=torch.float32, device="cuda") if kv == "fp8" else None
        self.free_pages = list(range(self.num_pages - 1, -1, -1))
        self.free_rows = list(range(max_resident - 1, -1, -1))
        self.table = np.zeros((max_resident, self.max_pages), dtype=np.int32)
        self.ctx.reserve(T, max_resident, self.num_pages)

    def admit(self, r: Request) -> bool:
        need = (r.in_len + r.out_len + PAGE - 1) // PAGE
        if not self.free_rows or len(self.free_pages) < need or need > self.max_pages:
            return False
        r.row = self.free_rows.pop()
        r.pages = [self.free_pages.pop() for _ in range(need)]
        self.table[r.row, :need] = r.pages
        return True

    def release(self, r: Request):
        self.free_pages.extend(r.pages)
        self.free_rows.append(r.row)
        r.pages, r.row = [], -1

    def run(self, seqs: List[Request], q_lens: List[int]) -> float:
        """One attention pass over the given sequences; returns its wall time in seconds."""
        torch = self.torch
        T = int(sum(q_lens))
        if T > self.rows:
            raise ValueError(f"a pass of {T} rows exceeds the {self.rows} rows of the buffers")
        ctx_lens = [r.cached + n for r, n in zip(seqs, q_lens)]
        bt = torch.from_numpy(self.table[[r.row for r in seqs]]).cuda()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.ctx.mixed_paged_attention(self.q[:T], self.k[:T], self.v[:T], self.kc, self.vc, self.scale, self.scale,
                                       bt, np.asarray(q_lens, np.int32), np.asarray(ctx_lens, np.int32), 0.0,
                                       self.out[:T])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        self.last = dict(bt=bt, q_lens=np.asarray(q_lens, np.int32), ctx_lens=np.asarray(ctx_lens, np.int32), T=T)
        for r, n in zip(seqs, q_lens):
            r.cached += n
        return dt


def replay(args, time_fn=None, on_pass=None, record=False) -> dict:
    """time_fn(q_lens, ctx_lens) -> seconds: the time charged for a pass instead of the measured one.
    on_pass(iteration, decoder): called after every pass (decoder.last describes it).
    record: the result also lists every iteration's (request ids, q_lens, ctx_lens) and the first-token and
    completion times by request id."""
    rng = np.random.default_rng(args.seed)
    rps_before, rps_after = (float(x) for x in args.rps.split(","))
    hq, hkv = (int(x) for x in args.heads.split(","))
    reqs = make_arrivals(rng, args.seconds, args.step_at, rps_before, rps_after, args.in_median, args.out_median,
                         args.in_max, args.out_max)
    dec = Decoder(hq, hkv, args.kv, args.max_resident, args.in_max + args.out_max, args.chunk_size, args.seed)
    now, nxt = 0.0, 0
    queue: List[Request] = []
    decoding: List[Request] = []
    task: Optional[Request] = None
    n_windows = int(np.ceil(args.seconds + args.drain)) + 1
    win = [dict(t=i, arrivals=0, prefill_tokens=0, decode_tokens=0, first_tokens=0, ttft_sum=0.0, queue=0,
                iterations=0, pass_ms_sum=0.0) for i in range(n_windows)]
    iterations = pf_rows = dec_rows = 0
    log = []
    while now < args.seconds + args.drain:
        while nxt < len(reqs) and reqs[nxt].arrival <= now:
            queue.append(reqs[nxt])
            win[min(int(reqs[nxt].arrival), n_windows - 1)]["arrivals"] += 1
            nxt += 1
        if task is None and queue and dec.admit(queue[0]):
            task = queue.pop(0)
        seqs, q_lens = list(decoding), [1] * len(decoding)
        n_pf = 0
        if task is not None:
            n_pf = max(0, min(task.in_len - task.cached, args.chunk_size - len(decoding)))   # decode rows come first
            if n_pf > 0:
                seqs.append(task)
                q_lens.append(n_pf)
        if not seqs:
            nxt_t = reqs[nxt].arrival if nxt < len(reqs) else args.seconds + args.drain
            now = max(now + 1e-3, nxt_t)                   # idle until the next arrival
            continue
        dt = dec.run(seqs, q_lens)
        if time_fn is not None:
            dt = float(time_fn(list(q_lens), [int(x) for x in dec.last["ctx_lens"]]))
        if record:
            log.append((tuple(r.rid for r in seqs), tuple(q_lens), tuple(int(x) for x in dec.last["ctx_lens"])))
        if on_pass is not None:
            on_pass(iterations, dec)
        iterations += 1
        pf_rows += n_pf if n_pf > 1 else 0                 # the library counts a one-token chunk as a decode row
        dec_rows += len(decoding) + (1 if n_pf == 1 else 0)
        now += dt * args.layers + args.other_ms * 1e-3
        w = win[min(int(now), n_windows - 1)]
        w["prefill_tokens"] += n_pf
        w["decode_tokens"] += len(decoding)
        w["iterations"] += 1
        w["pass_ms_sum"] += dt * 1e3
        w["queue"] = len(queue)
        still = []
        for r in decoding:
            r.generated += 1
            if r.generated >= r.out_len:
                r.done_at = now
                dec.release(r)
            else:
                still.append(r)
        decoding = still
        if task is not None and task.cached >= task.in_len:   # prefill complete: first token out
            task.first_token_at = now
            task.generated = 1
            w["first_tokens"] += 1
            w["ttft_sum"] += now - task.arrival
            if task.generated >= task.out_len:
                task.done_at = now
                dec.release(task)
            else:
                decoding.append(task)
            task = None
    vel = dec.ctx.token_velocity(sync=True)
    series = []
    for w in win:
        if w["iterations"] == 0 and w["arrivals"] == 0:
            continue
        series.append(dict(t=w["t"], arrivals=w["arrivals"], prefill_tok_per_s=w["prefill_tokens"],
                           decode_tok_per_s=w["decode_tokens"], queue=w["queue"],
                           mean_ttft_s=(w["ttft_sum"] / w["first_tokens"]) if w["first_tokens"] else None,
                           mean_pass_ms=(w["pass_ms_sum"] / w["iterations"]) if w["iterations"] else None))
    started = [r for r in reqs if r.first_token_at is not None]
    result = dict(requests=len(reqs), first_tokens=len(started), completed=sum(r.done_at is not None for r in reqs),
                  iterations=iterations, passes_counted=int(vel.passes),
                  prefill_tokens_counted=int(vel.prefill_tokens), decode_tokens_counted=int(vel.decode_tokens),
                  prefill_tokens_submitted=pf_rows, decode_tokens_submitted=dec_rows,
                  kernel_prefill_tok_per_s=vel.prefill_tok_per_s, kernel_decode_tok_per_s=vel.decode_tok_per_s,
                  series=series)
    if record:
        result["iteration_log"] = log
        result["first_token_at"] = {r.rid: r.first_token_at for r in reqs if r.first_token_at is not None}
        result["done_at"] = {r.rid: r.done_at for r in reqs if r.done_at is not None}
        result["arrivals"] = [(r.arrival, r.in_len, r.out_len) for r in reqs]
        result["num_pages"], result["max_pages_per_seq"] = dec.num_pages, dec.max_pages
    dec.ctx.close()
    return result


def main(argv=None, **replay_kwargs):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--heads", default="32,8")
    ap.add_argument("--kv", default="bf16", choices=["bf16", "fp8"])
    ap.add_argument("--seconds", type=float, default=20.0)
    ap.add_argument("--step-at", type=float, default=10.0)
    ap.add_argument("--rps", default="1,10", help="request rate before and after the step (paper Sec. 6.2: 1 -> 10)")
    ap.add_argument("--drain", type=float, default=5.0, help="seconds simulated after the last arrival")
    ap.add_argument("--in-median", type=int, default=1024)
    ap.add_argument("--out-median", type=int, default=200)
    ap.add_argument("--in-max", type=int, default=8192)
    ap.add_argument("--out-max", type=int, default=610)
    ap.add_argument("--chunk-size", type=int, default=2048)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--other-ms", type=float, default=8.0, help="per-iteration time of everything but attention")
    ap.add_argument("--max-resident", type=int, default=256)
    ap.add_argument("--seed", type=int, default=3)
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("the replay measures on a GPU")
    res = replay(args, **replay_kwargs)
    for s in res["series"]:
        ttft = f"{s['mean_ttft_s'] * 1e3:7.0f} ms" if s["mean_ttft_s"] is not None else "      -   "
        print(f"[replay] t={s['t']:3d}s arrivals {s['arrivals']:3d}  prefill {s['prefill_tok_per_s']:7d} tok/s  decode "
              f"{s['decode_tok_per_s']:6d} tok/s  queue {s['queue']:3d}  TTFT {ttft}  pass "
              f"{(s['mean_pass_ms'] or 0):6.3f} ms", file=sys.stderr)
    print(json.dumps({k: v for k, v in res.items() if k not in ("iteration_log", "first_token_at", "done_at", "arrivals")}))
    return res


if __name__ == "__main__":
    main()
