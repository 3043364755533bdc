"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the whole
batch runs on the GPU, a seeded sample of its rows is recomputed by the oracle one by one."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def _sampled_check(batch, seq_sample, row_stride, tol):
    import gpu_harness as g
    print(f"[case] {batch.name} full size S={batch.num_seqs} T={batch.total_q} sample={list(seq_sample)}",
          flush=True)
    out, _, _ = g.run_batch(batch)
    assert np.all(np.isfinite(out))
    q_off = np.concatenate([[0], np.cumsum(batch.q_lens)])
    sub = W.to_cpu(W.select_sequences(batch, seq_sample))
    sh = sub.shape
    ref_out, _, _ = None, None, None
    kc = oracle.new_cache(sub.num_pages, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
    vc = oracle.new_cache(sub.num_pages, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
    ks = None if sub.k_scale is None else oracle.raw(sub.k_scale)
    vs = None if sub.v_scale is None else oracle.raw(sub.v_scale)
    pre = sub.prefix_lens
    args = (sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype, sh.kv_dtype)
    if pre.sum():
        oracle.kv_append(*args, oracle.raw(sub.k_prefix), oracle.raw(sub.v_prefix), kc, vc, ks, vs,
                         sub.block_table, pre, pre, sub.num_pages)
    oracle.kv_append(*args, oracle.raw(sub.k_new), oracle.raw(sub.v_new), kc, vc, ks, vs, sub.block_table,
                     sub.q_lens, sub.ctx_lens, sub.num_pages)
    ref = oracle.mixed_paged_attention(*args, oracle.raw(sub.q), kc, vc, ks, vs, sub.block_table, sub.q_lens,
                                       sub.ctx_lens, sub.sm_scale, sub.num_pages, row_stride=row_stride)
    worst, n_rows, o = 0.0, 0, 0
    for s in seq_sample:
        ql = int(batch.q_lens[s])
        got = out[q_off[s]:q_off[s] + ql]
        want = ref[o:o + ql]
        sel = ~np.isnan(want[:, 0, 0])
        if sel.any():
            worst = max(worst, float(np.max(np.abs(got[sel] - want[sel]))))
        n_rows += int(sel.sum())
        o += ql
    print(f"       {n_rows} sampled rows, max abs err {worst:.3e} (bar {tol})", flush=True)
    assert n_rows > 0 and worst <= tol


def test_config2_decode_full_size_sampled():
    b = W.config2(device="cuda")
    assert b.num_seqs == 256 and b.shape.num_q_heads == 32
    sample = np.random.default_rng(7).choice(256, size=12, replace=False)
    longest, shortest = int(np.argmax(b.ctx_lens)), int(np.argmin(b.ctx_lens))
    _sampled_check(b, sorted(set(sample.tolist() + [longest, shortest])), 1, 2e-2)


def test_config4_burst_full_size_sampled():
    b = W.config4(device="cuda")
    dec = np.random.default_rng(8).choice(128, size=6, replace=False).tolist()
    _sampled_check(b, sorted(dec) + [128, 131], 7, 2e-2)      # every 7th row of the sample, two chunks included


def test_config5_fp8_full_size_sampled():
    b = W.config5(device="cuda")
    assert b.shape.kv_dtype == "fp8" and b.num_seqs == 528
    dec = np.random.default_rng(9).choice(512, size=5, replace=False).tolist()
    longest = int(np.argmax(b.ctx_lens[:512]))
    _sampled_check(b, sorted(set(dec + [longest])) + [512, 527], 61, 6e-2)   # two chunks, every 61st row of the sample


@pytest.mark.parametrize("step", [0, 3])
def test_config3_chunked_prefill_full_size_sampled(step):
    b = W.config3_step(step, device="cuda")
    _sampled_check(b, list(range(b.num_seqs)), 11, 2e-2)                     # every sequence, every 11th row


def test_many_short_sequences():
    """4096 decode rows with contexts of 1..64 tokens (first tokens, half-filled pages, page-opening
    tokens): work lists far longer than the number of resident workgroups."""
    rng = np.random.default_rng(21)
    ctx = rng.integers(1, 65, 4096).tolist()
    b = W.make_batch(W.AttnShape(32, 8, 128, "bf16", "bf16"), [1] * 4096, ctx, seed=21, pool_rule=1.1,
                     value_mult=0.5, device="cuda")
    _sampled_check(b, sorted(rng.choice(4096, size=64, replace=False).tolist()), 1, 2e-2)


@pytest.mark.parametrize("kv", ["bf16", "fp8"])
def test_one_very_long_row_and_one_long_chunk(kv):
    """A decode row over 131072 cached tokens (cut into many items whose partial results are merged)
    next to a prefill chunk of 4096 tokens over a prefix of 12288, at the page-table limit of both."""
    shape = W.AttnShape(32, 8, 128, "bf16", kv)
    b = W.make_batch(shape, [1, 4096], [131072, 16384], seed=22, num_pages=8192 + 1024 + 8, value_mult=0.5,
                     device="cuda")
    assert b.max_pages_per_seq == 8192
    _sampled_check(b, [0, 1], 257, 2e-2 if kv == "bf16" else 6e-2)
