"""Pins of the Token-Velocity oracle (oracle/velocity.py) to what the paper and arithmetic fix:
the worked two-burst example, a bucket table with a hand-checked sum, iteration-by-iteration
simulations, hand-worked routing cases and invariants.  None of them re-types a formula."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import velocity as ov

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def test_two_burst_example_of_the_scaling_policy_figure():
    """Sec. 3.2: both bursts need a second instance under the velocity policy; a request-count
    policy sees only the first."""
    for name, n_req, tok, vel, thr, tokens, needs, req_reacts, vel_reacts in rows("scaling_policy_two_bursts.txt"):
        n_req, tok, vel, thr, tokens = int(n_req), int(tok), float(vel), float(thr), int(tokens)
        assert n_req * tok == tokens
        need = ov.prefillers_required(float(tokens), vel, math.inf)      # arrival within one second
        assert (need > 1.0) == bool(int(needs)) == bool(int(vel_reacts))
        assert ov.instances_to_provision(need) == 2
        assert (n_req > thr) == bool(int(req_reacts))


def test_bucket_sum_on_the_paper_table_matches_hand_computation():
    """Sec. 5 table + Sec. 6.2: one request per second of each of the nine types.  The per-bucket terms
    were worked by hand to five decimals; exact rational arithmetic confirms the sum; the paper
    reports 3.2 decoders for its uniform mix at a rate it does not state."""
    t = rows("decoder_bucket_velocity.txt")
    hand = [0.01513, 0.07439, 0.16855, 0.03395, 0.14029, 0.28339, 0.20965, 0.75526, 1.35520]
    lam = [float(int(r[1]) + int(r[2])) for r in t]
    vel = [float(r[3]) for r in t]
    total, per = ov.decoders_required(lam, vel)
    assert np.allclose(per, hand, atol=6e-6)
    exact = sum(Fraction(int(r[1]) + int(r[2]), int(r[3])) for r in t)
    assert abs(total - float(exact)) < 1e-12
    assert abs(total - 3.0358) < 1e-4
    assert ov.instances_to_provision(total) == 4
    # twice the traffic needs twice the decoders; a bucket alone needs its own term
    assert abs(ov.decoders_required([2 * x for x in lam], vel)[0] - 2 * total) < 1e-12
    assert ov.decoders_required(lam[3:4], vel[3:4])[0] == per[3]


def test_prefiller_count_follows_the_slower_stage():
    assert ov.prefillers_required(12000.0, 6000.0, 1e9) == 2.0
    assert ov.prefillers_required(12000.0, 1e9, 4000.0) == 3.0
    assert ov.prefillers_required(12000.0, 6000.0, 4000.0) == ov.prefillers_required(12000.0, 4000.0, 6000.0) == 3.0
    assert ov.prefillers_required(0.0, 6000.0, 4000.0) == 0.0
    assert math.isnan(ov.prefillers_required(1.0, 0.0, 1.0))
    assert ov.instances_to_provision(2.0) == 2 and ov.instances_to_provision(2.0001) == 3
    assert ov.instances_to_provision(0.0) == 0 and ov.instances_to_provision(math.nan) == -1


def test_regular_decoders_never_negative():
    assert ov.regular_decoders_required(5.5, 2.0) == 3.5
    assert ov.regular_decoders_required(1.5, 2.0) == 0.0
    assert ov.regular_decoders_required(2.0, 2.0) == 0.0


def test_convertible_velocity_and_reserved_memory_against_iteration_simulation():
    """Sec. 4.4 by brute force: run iterations of one TPOT SLO each, every iteration admitting
    chunk_size - batch_size prefill tokens, for one TTFT SLO; the tokens admitted per second and
    the memory they occupy are what the two formulas must give."""
    chunk, batch, tpot, ttft, mem_t = 2048, 96, 0.1, 2.0, 131072
    iters = round(ttft / tpot)
    admitted = 0
    for _ in range(iters):
        admitted += chunk - batch
    v = ov.convertible_prefill_velocity(chunk, batch, tpot)
    assert abs(v - admitted / ttft) < 1e-9
    assert abs(ov.reserved_memory(v, mem_t, ttft) - admitted * mem_t) < 1e-3
    assert ov.convertible_prefill_velocity(512, 512, tpot) == 0.0
    assert ov.convertible_prefill_velocity(512, 600, tpot) == 0.0
    assert ov.decode_batch_estimate(40e9, 0.5e9) == 80.0


def test_decode_velocity_counts_released_tokens_per_iteration():
    # three requests finish in one 50 ms iteration holding 100, 350 and 610 tokens
    assert abs(ov.decode_velocity([100, 350, 610], 0.05) - 21200.0) < 1e-9
    assert ov.decode_velocity([], 0.05) == 0.0
    assert math.isnan(ov.decode_velocity([1], 0.0))


def test_prefill_routing_hand_cases():
    """Alg. 1 on cases small enough to read: velocities 1000 tok/s, SLO 0.25 s -> 250 tokens is the
    largest backlog a prefiller may hold."""
    V = [1000.0, 1000.0, 1000.0]
    assert ov.route_prefill([300, 250, 0], V, [0], [500.0], 0.25) == (ov.PREFILLER, 1)     # first that fits, inclusive
    assert ov.route_prefill([300, 251, 0], V, [0], [500.0], 0.25) == (ov.PREFILLER, 2)
    assert ov.route_prefill([300, 251, 400], V, [200, 100], [500.0, 500.0], 0.25) == (ov.CONVERTIBLE, 1)
    assert ov.route_prefill([300, 251, 400], V, [200, 126], [500.0, 500.0], 0.25) == (ov.QUEUE, -1)
    assert ov.route_prefill([], [], [], [], 0.25) == (ov.QUEUE, -1)
    # a convertible decoder whose decode batch fills the chunk has no prefill velocity
    assert ov.route_prefill([300], V[:1], [10], [0.0], 0.25) == (ov.QUEUE, -1)
    assert ov.route_prefill([300], V[:1], [0], [0.0], 0.25) == (ov.CONVERTIBLE, 0)


def test_prefill_routing_properties_random():
    rng = np.random.default_rng(3)
    for _ in range(300):
        n_p, n_d = rng.integers(0, 5), rng.integers(0, 4)
        pin, pv = rng.integers(0, 4000, n_p).astype(float), rng.uniform(500, 4000, n_p)
        din, dv = rng.integers(0, 4000, n_d).astype(float), rng.uniform(100, 2000, n_d)
        slo = float(rng.choice([0.25, 0.4, 2.0]))
        kind, idx = ov.route_prefill(pin, pv, din, dv, slo)
        p_ok = [i for i in range(n_p) if pin[i] <= slo * pv[i] * (1 + 1e-12)]
        d_ok = [i for i in range(n_d) if din[i] <= slo * dv[i] * (1 + 1e-12)]
        if p_ok:
            assert (kind, idx) == (ov.PREFILLER, p_ok[0])
        elif d_ok:
            assert (kind, idx) == (ov.CONVERTIBLE, d_ok[0])
        else:
            assert (kind, idx) == (ov.QUEUE, -1)


def test_decode_routing_hand_cases():
    inflight = [[3, 1], [2, 5], [2, 0], [0, 0]]
    conv = [False, False, False, True]
    util = [0.5, 0.5, 0.5, 0.95]
    assert ov.route_decode(inflight, 0, conv, util, 0.9) == 1        # decoder 3 is left out, tie 1/2 -> lowest
    assert ov.route_decode(inflight, 1, conv, util, 0.9) == 2
    assert ov.route_decode(inflight, 0, conv, [0.5, 0.5, 0.5, 0.9], 0.9) == 3   # at the threshold: still eligible
    assert ov.route_decode(inflight, 0, [False, False, False, False], util, 0.9) == 3  # regular decoders are never left out
    assert ov.route_decode([[1]], 0, [True], [0.99], 0.9) == -1
    assert ov.route_decode([], 0, [], [], 0.9) == -1


def test_chunk_profiling_stops_at_the_first_violation():
    """Sec. 4.4 on hand-made sweeps (TPOT SLO 100 ms, Sec. 5)."""
    slo = 0.100
    assert ov.largest_admissible_chunk([0.020, 0.040, 0.080, 0.100, 0.130, 0.300], slo) == 3   # meeting it exactly counts
    assert ov.largest_admissible_chunk([0.020, 0.040, 0.101, 0.090, 0.095], slo) == 1           # later passes are not looked at
    assert ov.largest_admissible_chunk([0.150, 0.050], slo) == -1
    assert ov.largest_admissible_chunk([], slo) == -1
    assert ov.largest_admissible_chunk([0.01, 0.02, 0.03], slo) == 2
    assert ov.largest_admissible_chunk([0.01, math.nan, 0.02], slo) == 0
    # growing the sweep never makes the choice smaller; tightening the SLO never makes it larger
    rng = np.random.default_rng(9)
    for _ in range(200):
        t = np.cumsum(rng.uniform(0.001, 0.02, 12))
        full = ov.largest_admissible_chunk(list(t), slo)
        assert ov.largest_admissible_chunk(list(t[:6]), slo) <= full
        assert ov.largest_admissible_chunk(list(t), slo * 0.5) <= full
        assert full == int(np.searchsorted(t, slo, side="right")) - 1      # monotone sweep: a plain count
