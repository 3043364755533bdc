"""TEST INFRASTRUCTURE: the iteration scheduler of one Convertible Decoder, written out plainly.

Only tests/ may import this module; the product's replay (paper_2512_03416_amd/replay.py) shares nothing
with it.  It forms, iteration by iteration, the batch a Convertible Decoder runs (TokenScale paper, Sec. 3.4
and Sec. 4.4): the decode batch comes first -- every request that is generating contributes one row -- and
at most one prefill task at a time is absorbed as a restricted chunk whose length is bounded by what the
profiled chunk size leaves next to the decode batch ("chunk size" counts prefill tokens plus the decode batch
size, Sec. 4.4).  The time of a pass is GIVEN (a function of the batch's lengths), so the schedule and the
first-token times follow from the arrival list alone.

Readings where the paper is silent (the product's replay takes the same ones, stated in its docstring):
  * a request is admitted as the prefill task when a table row and pages for input + output are free;
    requests wait in arrival order and the head of the queue is never overtaken;
  * simulated time advances per iteration by pass_time * layers + other_s;
  * a request's first token is released by the iteration that finishes its prefill, and it joins the decode
    batch from the next iteration on; a decode row's context includes the token it appends;
  * a request is done when it has generated out_len tokens (the first token counts).

Pinned by tests/test_replay_pins.py on a hand-worked trace of three requests.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Sequence, Tuple

PAGE = 16


def schedule(requests: Sequence[Tuple[float, int, int]], *, chunk_size: int, max_resident: int, num_pages: int,
             max_pages_per_seq: int, pass_time: Callable[[List[int], List[int]], float], layers: int,
             other_s: float, horizon_s: float):
    """requests: (arrival time, input length, output length), in arrival order; request i has id i.
    Returns (iterations, first_token_at, done_at): iterations is a list of (request ids, q_lens, ctx_lens) in
    batch order (decode rows first, then the chunk); the two dicts map request id -> simulated time."""
    now = 0.0
    nxt = 0
    queue: List[int] = []
    decoding: List[int] = []
    task = -1
    cached: Dict[int, int] = {}
    generated: Dict[int, int] = {}
    pages_held: Dict[int, int] = {}
    free_rows, free_pages = max_resident, num_pages
    iterations = []
    first_token_at: Dict[int, float] = {}
    done_at: Dict[int, float] = {}

    def release(r):
        nonlocal free_rows, free_pages
        free_rows += 1
        free_pages += pages_held.pop(r)

    while now < horizon_s:
        while nxt < len(requests) and requests[nxt][0] <= now:
            queue.append(nxt)
            nxt += 1
        if task < 0 and queue:
            r = queue[0]
            need = (requests[r][1] + requests[r][2] + PAGE - 1) // PAGE
            if free_rows > 0 and need <= free_pages and need <= max_pages_per_seq:
                queue.pop(0)
                free_rows -= 1
                free_pages -= need
                pages_held[r] = need
                cached[r] = 0
                generated[r] = 0
                task = r
        ids = list(decoding)
        q_lens = [1] * len(decoding)
        n_pf = 0
        if task >= 0:
            n_pf = min(requests[task][1] - cached[task], chunk_size - len(decoding))
            if n_pf > 0:
                ids.append(task)
                q_lens.append(n_pf)
        if not ids:
            nxt_t = requests[nxt][0] if nxt < len(requests) else horizon_s
            now = max(now + 1e-3, nxt_t)
            continue
        ctx_lens = [cached[r] + n for r, n in zip(ids, q_lens)]
        iterations.append((tuple(ids), tuple(q_lens), tuple(ctx_lens)))
        now += pass_time(q_lens, ctx_lens) * layers + other_s
        for r, n in zip(ids, q_lens):
            cached[r] += n
        still = []
        for r in decoding:
            generated[r] += 1
            if generated[r] >= requests[r][2]:
                done_at[r] = now
                release(r)
            else:
                still.append(r)
        decoding = still
        if task >= 0 and cached[task] >= requests[task][1]:
            first_token_at[task] = now
            generated[task] = 1
            if generated[task] >= requests[task][2]:
                done_at[task] = now
                release(task)
            else:
                decoding.append(task)
            task = -1
    return iterations, first_token_at, done_at
