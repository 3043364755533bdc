"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the whole
batch runs on the GPU, a seeded sample of its rows is recomputed by the oracle one by one, and the
cache pages of the sampled sequences are compared byte for byte with the oracle's."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

_ES = {"f32": 4, "bf16": 2, "fp8": 1}


def _oracle_caches(sub):
    """Fresh oracle caches holding the sub-batch's prefix and new tokens."""
    sh = sub.shape
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
    return args, kc, vc, ks, vs


def _run_gpu_keep_caches(batch):
    """One pass through the C ABI exactly as gpu_harness.run_batch does, but the caches stay on the
    GPU (they are gigabytes at these sizes); returns (out float64 numpy, k cache, v cache, page bytes)."""
    import gpu_harness as g
    import paper_2512_03416_amd as ts
    batch = g.to_dev(batch)
    sh = batch.shape
    ctx = ts.Context(g.make_desc(batch))
    kc, vc = g.new_caches(batch)
    bt = torch.from_numpy(batch.block_table).to("cuda").contiguous()
    pre = batch.prefix_lens
    if int(pre.sum()) > 0:
        ctx.kv_append(batch.k_prefix, batch.v_prefix, kc, vc, batch.k_scale, batch.v_scale, bt, pre, pre)
    out = torch.full((batch.total_q, sh.num_q_heads, sh.head_dim), float("nan"), dtype=batch.q.dtype,
                     device="cuda")
    ctx.mixed_paged_attention(batch.q, batch.k_new, batch.v_new, kc, vc, batch.k_scale, batch.v_scale, bt,
                              batch.q_lens, batch.ctx_lens, batch.sm_scale, out)
    torch.cuda.synchronize()
    ctx.close()
    page_bytes = sh.num_kv_heads * 16 * sh.head_dim * _ES[sh.kv_dtype]
    return out.double().cpu().numpy(), kc.view(-1, page_bytes), vc.view(-1, page_bytes), page_bytes


def _check_cache_pages(batch, sub, seq_sample, gk, gv, ok, ov, page_bytes):
    """Every page of every sampled sequence: the GPU's bytes at its page id against the oracle's at the
    sub-batch's page id, whole pages (all KV heads, all 16 slots, untouched slots included).  Pure
    indexing through the two page tables; nothing here knows the order of elements inside a page."""
    ok = ok.view(np.uint8).reshape(-1, page_bytes)
    ov = ov.view(np.uint8).reshape(-1, page_bytes)
    n_pages = 0
    for i, s in enumerate(seq_sample):
        used = (int(batch.ctx_lens[s]) + 15) // 16
        gpu_ids = torch.from_numpy(batch.block_table[s, :used].astype(np.int64)).cuda()
        ref_ids = sub.block_table[i, :used].astype(np.int64)
        assert np.array_equal(gk[gpu_ids].cpu().numpy(), ok[ref_ids]), f"K cache pages of sequence {s} differ"
        assert np.array_equal(gv[gpu_ids].cpu().numpy(), ov[ref_ids]), f"V cache pages of sequence {s} differ"
        n_pages += used
    return n_pages


def _sampled_check(batch, seq_sample, row_stride, tol, tile_rows=()):
    """tile_rows: (sequence, first chunk token, count) runs of consecutive chunk rows that the oracle
    recomputes in full, on top of the strided sample."""
    print(f"[case] {batch.name} full size S={batch.num_seqs} T={batch.total_q} sample={list(seq_sample)}",
          flush=True)
    out, gk, gv, page_bytes = _run_gpu_keep_caches(batch)
    assert np.all(np.isfinite(out))
    # pages the batch does not use must still hold the fill pattern (a stray store would show here)
    used_ids = np.unique(batch.block_table[batch.block_table >= 0])
    unused = np.setdiff1d(np.arange(batch.num_pages), used_ids)
    if unused.size:
        pick = torch.from_numpy(unused[:: max(1, unused.size // 4096)].astype(np.int64)).cuda()
        assert bool((gk[pick] == 0xFF).all()) and bool((gv[pick] == 0xFF).all()), "an unused page was written"
    q_off = np.concatenate([[0], np.cumsum(batch.q_lens)])
    sub = W.to_cpu(W.select_sequences(batch, seq_sample))
    args, kc, vc, ks, vs = _oracle_caches(sub)
    n_pages = _check_cache_pages(batch, sub, seq_sample, gk, gv, kc, vc, page_bytes)
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
    # whole runs of consecutive chunk rows (complete query tiles of the prefill kernel): the oracle
    # sees the chunk tokens in front of the run as cached prefix, which is the same attention problem
    sub_q_off = np.concatenate([[0], np.cumsum(sub.q_lens)])
    sub_p_off = np.concatenate([[0], np.cumsum(sub.prefix_lens)])
    for s, t0, cnt in tile_rows:
        i = list(seq_sample).index(s)
        ql, pre = int(sub.q_lens[i]), int(sub.prefix_lens[i])
        assert 0 <= t0 and t0 + cnt <= ql
        a, b = int(sub_q_off[i]), int(sub_p_off[i])
        run = W.make_batch(sub.shape, [cnt], [pre + t0 + cnt], seed=5, sm_scale=sub.sm_scale)
        run.q = sub.q[a + t0:a + t0 + cnt].clone()
        run.k_new, run.v_new = sub.k_new[a + t0:a + t0 + cnt].clone(), sub.v_new[a + t0:a + t0 + cnt].clone()
        run.k_prefix = torch.cat([sub.k_prefix[b:b + pre], sub.k_new[a:a + t0]]).contiguous()
        run.v_prefix = torch.cat([sub.v_prefix[b:b + pre], sub.v_new[a:a + t0]]).contiguous()
        run.k_scale, run.v_scale = sub.k_scale, sub.v_scale
        want, _, _ = oracle.run_batch(run)
        got = out[q_off[s] + t0:q_off[s] + t0 + cnt]
        worst = max(worst, float(np.max(np.abs(got - want))))
        n_rows += cnt
    print(f"       {n_rows} sampled rows, max abs err {worst:.3e} (bar {tol}); {n_pages} cache pages byte-equal",
          flush=True)
    assert n_rows > 0 and worst <= tol


def test_config2_decode_full_size_sampled():
    b = W.config2(device="cuda")
    assert b.num_seqs == 256 and b.shape.num_q_heads == 32
    sample = np.random.default_rng(7).choice(256, size=12, replace=False)
    longest, shortest = int(np.argmax(b.ctx_lens)), int(np.argmin(b.ctx_lens))
    _sampled_check(b, sorted(set(sample.tolist() + [longest, shortest])), 1, 2e-2)


def test_config4_burst_full_size_sampled():
    import gpu_harness as g
    import paper_2512_03416_amd as ts
    b = W.config4(device="cuda")
    assert ts.plan_describe(g.make_desc(b), b.q_lens, b.ctx_lens).mixed_mode == 2      # co-resident launch
    dec = np.random.default_rng(8).choice(128, size=6, replace=False).tolist()
    # every 7th row of the sample, two chunks included, plus whole query tiles (64 tokens x 4 heads) of one
    # chunk: one in the middle with its neighbours' edges, and the chunk's last
    _sampled_check(b, sorted(dec) + [128, 131], 7, 2e-2, tile_rows=[(131, 1000, 100), (131, 2048 - 64, 64)])


def test_config5_fp8_full_size_sampled():
    b = W.config5(device="cuda")
    assert b.shape.kv_dtype == "fp8" and b.num_seqs == 528
    import gpu_harness as g
    import paper_2512_03416_amd as ts
    assert ts.plan_describe(g.make_desc(b), b.q_lens, b.ctx_lens).mixed_mode == 2      # co-resident launch
    dec = np.random.default_rng(9).choice(512, size=5, replace=False).tolist()
    longest = int(np.argmax(b.ctx_lens[:512]))
    # two chunks, every 61st row of the sample, plus two whole query tiles (32 tokens x 8 heads) and the edges around them
    _sampled_check(b, sorted(set(dec + [longest])) + [512, 527], 61, 6e-2, tile_rows=[(527, 2040, 80)])


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
