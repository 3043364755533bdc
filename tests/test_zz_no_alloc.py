"""The allocation-free entry point against the ordinary one (GPU, through the C ABI).

Collected last on purpose: it runs after every other GPU test of the directory."""
import numpy as np
import pytest
import torch

import workloads as W
from workloads import AttnShape, make_batch

pytestmark = pytest.mark.gpu


def _pass(ctx, b, noalloc):
    """Fresh caches, prefix append, one pass with append; returns (out, k cache, v cache) as byte arrays."""
    import gpu_harness as g
    kc, vc = g.new_caches(b)
    bt = torch.from_numpy(b.block_table).cuda()
    pre = b.prefix_lens
    if int(pre.sum()):
        ctx.kv_append(b.k_prefix, b.v_prefix, kc, vc, b.k_scale, b.v_scale, bt, pre, pre)
    out = torch.full((b.total_q, b.shape.num_q_heads, b.shape.head_dim), float("nan"), dtype=b.q.dtype, device="cuda")
    ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, b.k_scale, b.v_scale, bt, b.q_lens, b.ctx_lens,
                              b.sm_scale, out, noalloc=noalloc)
    torch.cuda.synchronize()
    raw = lambda t: t.view(torch.uint8).cpu().numpy()
    return raw(out), raw(kc), raw(vc)


@pytest.mark.parametrize("kv,persistent", [("bf16", 2), ("bf16", 1), ("fp8", 1), ("bf16", 0)])
def test_noalloc_entry_point_matches_the_ordinary_one(kv, persistent):
    """Two calls in a row through ts_mixed_paged_attention_noalloc, the second with a smaller batch: outputs
    and caches byte-equal to ts_mixed_paged_attention's (same kernels, other scratch), which in turn is
    checked against the oracle; the context allocates nothing meanwhile; an oversized batch is refused
    before anything is launched."""
    import gpu_harness as g
    import oracle
    import paper_2512_03416_amd as ts
    from paper_2512_03416_amd import binding
    shape = AttnShape(32, 8, 128, "bf16", kv)
    big = dict(q=[1, 1, 1, 300, 1, 130, 1, 700], c=[3000, 555, 40, 420, 64, 135, 1, 900])
    small = dict(q=[1, 70], c=[900, 70])
    tol = 2e-2 if kv == "bf16" else 6e-2
    b0 = g.to_dev(make_batch(shape, big["q"], big["c"], seed=91, value_mult=0.5))
    ctx = ts.Context(g.make_desc(b0))
    ctx.set_option("decode_split_pages", 8)                   # split rows: partial results and their merge are in play
    ctx.set_option("mixed_mode", persistent)
    for i, spec in enumerate((big, small)):
        print(f"[case] noalloc kv={kv} persistent={persistent} call {i}: q_lens={spec['q']}", flush=True)
        b = g.to_dev(make_batch(shape, spec["q"], spec["c"], seed=91 + i, value_mult=0.5, num_pages=b0.num_pages))
        b.block_table = np.ascontiguousarray(np.pad(b.block_table, ((0, 0), (0, b0.max_pages_per_seq - b.max_pages_per_seq)),
                                                    constant_values=-1))
        want = _pass(ctx, b, noalloc=False)
        n0 = ctx.get_option("scratch_allocations")
        got = _pass(ctx, b, noalloc=True)
        assert ctx.get_option("scratch_allocations") == n0
        for x, y, what in zip(got, want, ("out", "k cache", "v cache")):
            assert x.shape == y.shape and x.tobytes() == y.tobytes(), what
        ref, _, _ = oracle.run_batch(W.to_cpu(make_batch(shape, spec["q"], spec["c"], seed=91 + i, value_mult=0.5,
                                                         num_pages=b0.num_pages)))
        out = torch.from_numpy(got[0].copy()).view(torch.bfloat16).double().numpy().reshape(ref.shape)
        assert float(np.max(np.abs(out - ref))) <= tol
    # a second context shares the GPU's static scratch: same answer again
    ctx2 = ts.Context(g.make_desc(b0))
    ctx2.set_option("decode_split_pages", 8)
    ctx2.set_option("mixed_mode", persistent)
    again = _pass(ctx2, b, noalloc=True)
    assert again[0].tobytes() == got[0].tobytes()
    ctx2.close()
    # too large for the static scratch: refused, nothing written
    n = 40000
    ql, cl = np.ones(n, np.int32), np.ones(n, np.int32)
    bt = torch.zeros((n, b0.max_pages_per_seq), dtype=torch.int32, device="cuda")
    q = torch.zeros((n, 32, 128), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((n, 8, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.full((n, 32, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    kc, vc = g.new_caches(b0)
    with pytest.raises(ts.TokenScaleError) as e:
        ctx.mixed_paged_attention(q, kn, kn, kc, vc, b0.k_scale, b0.v_scale, bt, ql, cl, 0.0, out, noalloc=True)
    assert e.value.code == binding.TS_ERR_UNSUPPORTED and "allocation-free" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()) and bool((kc == 0xFF).all()) and bool((vc == 0xFF).all())
    ctx.set_option("validate_block_table", 1)
    with pytest.raises(ts.TokenScaleError) as e:
        _pass(ctx, b, noalloc=True)
    assert e.value.code == binding.TS_ERR_UNSUPPORTED
    ctx.close()
