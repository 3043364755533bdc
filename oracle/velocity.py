"""TEST INFRASTRUCTURE: the Token-Velocity policy formulas, written out plainly in Python floats (fp64).

Only tests/ may import this module; the product is the C library, which shares nothing with it.
Each function follows one passage of the TokenScale paper, in its notation.  Where the paper leaves
a choice open the reading taken is stated in the docstring.

Pinned by tests/test_velocity_pins.py: the two-burst example of the scaling-policy figure (Sec. 3.2),
a step-by-step simulation of a Convertible Decoder's iterations, hand-worked routing cases, and the
invariants the formulas imply.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple


def decode_velocity(completed_request_tokens: Sequence[int], tpot_s: float) -> float:
    """Decode velocity V_D (Sec. 3.2, first equation): the tokens held by the requests in R,
    summed, divided by the measured TPOT.  Reading: R is the set of requests that complete during
    one decode iteration, whose duration is the TPOT, so the quotient is tokens released per second."""
    if not tpot_s > 0:
        return math.nan
    total = 0
    for L_r in completed_request_tokens:
        if L_r < 0:
            return math.nan
        total += L_r
    return total / tpot_s


def prefillers_required(lam: float, V_P: float, V_BW: float) -> float:
    """I^P (Sec. 4.3, prefiller autoscaler): input token arrival rate over the smaller of the
    prefill and the network velocity."""
    if not (lam >= 0 and V_P > 0 and V_BW > 0):
        return math.nan
    return lam / min(V_P, V_BW)


def decoders_required(lam_b: Sequence[float], V_D_b: Sequence[float]) -> Tuple[float, list]:
    """I^D (Sec. 4.3, decoder autoscaler): per bucket b the arrival rate of input plus predicted
    output tokens over that bucket's profiled velocity; the total is their sum.  Returns
    (I^D, [I^(b)])."""
    if len(lam_b) != len(V_D_b):
        return math.nan, []
    per = []
    for lam, v in zip(lam_b, V_D_b):
        if not (lam >= 0 and v > 0):
            return math.nan, []
        per.append(lam / v)
    total = 0.0
    for x in per:          # summed in bucket order
        total += x
    return total, per


def regular_decoders_required(I_D: float, I_D_c: float) -> float:
    """I^D_r (Sec. 4.3): what is left of I^D after the fixed pool of Convertible Decoders, never
    below zero."""
    if not (I_D >= 0 and I_D_c >= 0):
        return math.nan
    return max(I_D - I_D_c, 0.0)


def decode_batch_estimate(available_bytes: float, mean_request_bytes: float) -> float:
    """Average decode batch size (Sec. 4.4): available GPU memory over the average memory one
    request of the trace occupies."""
    if not (available_bytes >= 0 and mean_request_bytes > 0):
        return math.nan
    return available_bytes / mean_request_bytes


def convertible_prefill_velocity(chunk_size: float, batch_size: float, tpot_slo_s: float) -> float:
    """V_D^{P'} (Sec. 4.4): an iteration has room for chunk_size - batch_size prefill tokens and may
    last one TPOT SLO.  Reading: a decode batch that already fills the chunk leaves velocity 0
    (the paper defines chunk size as the maximum of the sum, so the difference is not negative)."""
    if not (chunk_size >= 0 and batch_size >= 0 and tpot_slo_s > 0):
        return math.nan
    return max(chunk_size - batch_size, 0.0) / tpot_slo_s


def reserved_memory(V_D_P: float, Mem_T: float, ttft_slo_s: float) -> float:
    """Mem_Reserved (Sec. 4.4): the tokens a Convertible Decoder can prefill within one TTFT SLO,
    times the memory footprint of a token."""
    if not (V_D_P >= 0 and Mem_T >= 0 and ttft_slo_s >= 0):
        return math.nan
    return V_D_P * Mem_T * ttft_slo_s


def instances_to_provision(requirement: float) -> int:
    """Sec. 4.3 allocates the minimum number of instances that gives enough velocity: the smallest
    integer not below the requirement.  -1 for a requirement that is not a finite number >= 0."""
    if not (requirement >= 0 and math.isfinite(requirement)):
        return -1
    return int(math.ceil(requirement))


def largest_admissible_chunk(iteration_time_s: Sequence[float], tpot_slo_s: float) -> int:
    """Chunk-size profiling of a Convertible Decoder (Sec. 4.4): the chunk size is raised step by
    step and the iteration time measured until the TPOT SLO is violated; the largest size that
    still met it is chosen.  iteration_time_s[i] is the time measured at the i-th (ascending) chunk
    size.  Returns the index chosen, -1 when even the first size violates the SLO.  Reading: the
    sweep stops at the first violation, so a larger size that happens to pass again is not looked
    at."""
    chosen = -1
    for i, t in enumerate(iteration_time_s):
        if not t <= tpot_slo_s:
            break
        chosen = i
    return chosen


PREFILLER, CONVERTIBLE, QUEUE = 0, 1, 2


def route_prefill(prefiller_inflight: Sequence[float], prefiller_velocity: Sequence[float],
                  conv_inflight: Sequence[float], conv_velocity: Sequence[float],
                  slo_s: float) -> Tuple[int, int]:
    """Prefill routing (Sec. 4.5, Alg. 1).  First round: prefillers in order, waiting time =
    in-flight tokens over the prefiller's velocity; the first one within the request's TTFT SLO
    takes it.  Second round: the same over the Convertible Decoders with their prefill velocity
    V_D^{P'}.  Otherwise the request is queued.  Returns (kind, index); index is -1 for QUEUE.
    Reading: the comparison is inclusive as printed; an instance with velocity 0 can take a request
    only if it has nothing in flight (waiting time 0), else its waiting time is unbounded."""
    def waiting(tokens, v):
        if tokens == 0:
            return 0.0
        return tokens / v if v > 0 else math.inf

    for p in range(len(prefiller_inflight)):
        if waiting(prefiller_inflight[p], prefiller_velocity[p]) <= slo_s:
            return PREFILLER, p
    for d in range(len(conv_inflight)):
        if waiting(conv_inflight[d], conv_velocity[d]) <= slo_s:
            return CONVERTIBLE, d
    return QUEUE, -1


def route_decode(inflight_by_type: Sequence[Sequence[int]], request_type: int,
                 convertible: Sequence[bool], mem_util: Sequence[float],
                 mem_threshold: float) -> int:
    """Decode routing (Sec. 4.5, decode load balancing): among all decoders, the one with the fewest
    in-flight requests of the request's type; Convertible Decoders whose memory utilisation exceeds
    the threshold are left out.  Reading: ties go to the lowest index; -1 when no decoder is
    eligible."""
    best: Optional[int] = None
    for d in range(len(inflight_by_type)):
        if convertible[d] and mem_util[d] > mem_threshold:
            continue
        if best is None or inflight_by_type[d][request_type] < inflight_by_type[best][request_type]:
            best = d
    return -1 if best is None else best
