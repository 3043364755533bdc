"""Token-Velocity policy functions of the library (C ABI, host only) against the oracle
(oracle/velocity.py): element by element on seeded inputs, plus the domain errors."""
import math

import numpy as np
import pytest

from oracle import velocity as ov
from paper_2512_03416_amd import Desc, policy

TTFT = [0.25, 0.4, 2.0]          # Sec. 5: TTFT SLOs by input length; TPOT SLO 0.1 s


def same(a, b):
    return (math.isnan(a) and math.isnan(b)) or a == b


def test_scalar_formulas_bit_exact_on_random_inputs():
    rng = np.random.default_rng(11)
    for _ in range(500):
        lam, vp, vbw = rng.uniform(0, 5e5), rng.uniform(1, 5e4), rng.uniform(1, 5e6)
        assert same(policy.tv_prefillers(lam, vp, vbw), ov.prefillers_required(lam, vp, vbw))
        i_d, i_c = rng.uniform(0, 40), rng.uniform(0, 10)
        assert same(policy.tv_regular_decoders(i_d, i_c), ov.regular_decoders_required(i_d, i_c))
        chunk, batch = float(rng.integers(0, 8192)), float(rng.integers(0, 600))
        v = policy.tv_convertible_prefill_velocity(chunk, batch, 0.1)
        assert same(v, ov.convertible_prefill_velocity(chunk, batch, 0.1))
        mem_t, ttft = float(rng.integers(1, 1 << 20)), float(rng.choice(TTFT))
        assert same(policy.tv_reserved_memory(v, mem_t, ttft), ov.reserved_memory(v, mem_t, ttft))
        a, m = rng.uniform(0, 2.88e11), rng.uniform(1e6, 1e10)
        assert same(policy.tv_decode_batch(a, m), ov.decode_batch_estimate(a, m))
        req = rng.uniform(0, 50)
        assert policy.tv_instances(req) == ov.instances_to_provision(req)
        toks = rng.integers(0, 9000, rng.integers(0, 12))
        tpot = rng.uniform(0.01, 0.2)
        assert same(policy.tv_decode_velocity(toks, tpot), ov.decode_velocity([int(t) for t in toks], tpot))


def test_decoder_sum_bit_exact_and_per_bucket_terms():
    rng = np.random.default_rng(12)
    for n in (0, 1, 2, 9, 64):
        lam, v = rng.uniform(0, 1e5, n), rng.uniform(1e3, 4e4, n)
        total, per = policy.tv_decoders(lam, v)
        want, want_per = ov.decoders_required(list(lam), list(v))
        assert total == want and list(per) == want_per


def test_domain_errors_agree():
    nan, inf = math.nan, math.inf
    for args in ((-1.0, 1.0, 1.0), (1.0, 0.0, 1.0), (1.0, 1.0, 0.0), (nan, 1.0, 1.0), (1.0, nan, 1.0)):
        assert math.isnan(policy.tv_prefillers(*args)) and math.isnan(ov.prefillers_required(*args))
    assert policy.tv_prefillers(10.0, 5.0, inf) == 2.0
    total, per = policy.tv_decoders([1.0, 2.0], [3.0, 0.0])
    assert math.isnan(total) and np.isnan(per).all()               # nothing written on error
    assert math.isnan(ov.decoders_required([1.0, 2.0], [3.0, 0.0])[0])
    assert math.isnan(policy.tv_convertible_prefill_velocity(1.0, 1.0, 0.0))
    assert math.isnan(policy.tv_regular_decoders(-1.0, 0.0))
    assert math.isnan(policy.tv_reserved_memory(-1.0, 1.0, 1.0))
    assert math.isnan(policy.tv_decode_batch(1.0, 0.0))
    assert math.isnan(policy.tv_decode_velocity([1, -1], 0.1)) and math.isnan(policy.tv_decode_velocity([1], 0.0))
    for bad in (nan, inf, -0.5):
        assert policy.tv_instances(bad) == policy.INVALID and ov.instances_to_provision(bad) == -1


def test_token_bytes():
    # Llama-3.1-8B geometry (Sec. 5): 8 KV heads of 128 dims, 32 layers, bf16 -> 128 KiB per token
    d = Desc.make(32, 8, 128, "bf16", "bf16", 1000, 64)
    assert policy.tv_token_bytes(d, 32) == 2 * 8 * 128 * 2 * 32 == 131072
    assert policy.tv_token_bytes(Desc.make(64, 8, 128, "bf16", "fp8", 1000, 64), 80) == 2 * 8 * 128 * 80
    assert policy.tv_token_bytes(d, 0) == 0
    assert policy.tv_token_bytes(Desc.make(32, 8, 100, "bf16", "bf16", 1000, 64), 1) == 0


def test_prefill_routing_matches_oracle():
    rng = np.random.default_rng(13)
    kinds = {ov.PREFILLER: policy.PREFILLER, ov.CONVERTIBLE: policy.CONVERTIBLE, ov.QUEUE: policy.QUEUE}
    seen = set()
    for _ in range(2000):
        n_p, n_d = int(rng.integers(0, 6)), int(rng.integers(0, 5))
        pin = rng.integers(0, 6000, n_p).astype(float) * rng.integers(0, 2, n_p)
        pv = rng.uniform(0, 8000, n_p) * rng.integers(0, 2, n_p)     # some stalled instances (velocity 0)
        din = rng.integers(0, 3000, n_d).astype(float) * rng.integers(0, 2, n_d)
        dv = np.array([ov.convertible_prefill_velocity(2048, b, 0.1) for b in rng.integers(0, 2300, n_d)])
        slo = float(rng.choice(TTFT))
        kind, idx = policy.route_prefill(pin, pv, din, dv, slo)
        okind, oidx = ov.route_prefill(list(pin), list(pv), list(din), list(dv), slo)
        assert (kind, idx) == (kinds[okind], oidx)
        seen.add(kind)
    assert seen == {policy.PREFILLER, policy.CONVERTIBLE, policy.QUEUE}


def test_decode_routing_matches_oracle():
    rng = np.random.default_rng(14)
    none = 0
    for _ in range(2000):
        n_d, n_t = int(rng.integers(0, 8)), 9                        # nine request types (Sec. 5 table)
        inflight = rng.integers(0, 6, (n_d, n_t)).astype(np.int32)
        conv = rng.integers(0, 2, n_d).astype(bool)
        util = rng.choice([0.3, 0.8, 0.9, 0.95], n_d)
        typ = int(rng.integers(0, n_t))
        got = policy.route_decode(inflight, typ, conv, util, 0.9, n_types=n_t)
        want = ov.route_decode(inflight.tolist(), typ, list(conv), list(util), 0.9)
        assert got == want
        none += got == policy.NONE
    assert none > 0
    assert policy.route_decode(np.zeros((2, 3), np.int32), 3, [0, 0], [0.1, 0.1], 0.9) == policy.INVALID


def test_chunk_sweep_choice_matches_oracle():
    rng = np.random.default_rng(15)
    for _ in range(1000):
        n = int(rng.integers(0, 14))
        t = np.cumsum(rng.uniform(0.0, 0.03, n)) * rng.choice([1.0, 1.0, 1.0, -1.0]) ** 0
        if n and rng.random() < 0.3:
            t[rng.integers(0, n)] *= rng.choice([0.2, 3.0])           # a non-monotone sample
        if n and rng.random() < 0.1:
            t[rng.integers(0, n)] = math.nan
        slo = float(rng.choice([0.05, 0.1, 0.2]))
        assert policy.tv_largest_chunk(t, slo) == ov.largest_admissible_chunk(list(t), slo)
    assert policy.tv_largest_chunk([], 0.1) == policy.NONE
