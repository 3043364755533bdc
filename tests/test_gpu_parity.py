"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs.

Bars: KV append bit-exact; attention max-abs-error <= 1e-5 (fp32), 2e-2 (bf16), 6e-2 (fp8 cache,
the oracle reading the same quantised bytes).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from workloads import AttnShape, make_batch

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2, "fp8": 6e-2}


def gpu():
    import gpu_harness
    return gpu_harness


def same_bytes(a, b):
    """Bit-exact comparison (the 0xFF poison is a NaN in every element type)."""
    return np.array_equal(np.ascontiguousarray(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8))


def check(batch, options=None, fused_append=True, tol=None, what=""):
    print(f"[case] {batch.name} {what} shape={batch.shape} S={batch.num_seqs} T={batch.total_q} "
          f"opts={options}", flush=True)
    ref, rk, rv = oracle.run_batch(W.to_cpu(batch))
    out, gk, gv = gpu().run_batch(batch, options=options, fused_append=fused_append)
    assert same_bytes(gk, rk), "K cache differs from the oracle's"
    assert same_bytes(gv, rv), "V cache differs from the oracle's"
    assert out.shape == ref.shape
    assert np.all(np.isfinite(out)), "non-finite output"
    err = float(np.max(np.abs(out - ref))) if out.size else 0.0
    bar = tol if tol is not None else TOL[batch.shape.kv_dtype]
    print(f"       max abs err {err:.3e} (bar {bar})", flush=True)
    assert err <= bar
    return err


# ---------------------------------------------------------------------------------------------
# configuration 1 and its relatives (generic row kernel)
# ---------------------------------------------------------------------------------------------

def test_config1_tiny_fp32_mixed():
    check(W.config1())


@pytest.mark.parametrize("shape", [
    AttnShape(4, 1, 64, "f32", "f32"), AttnShape(8, 2, 128, "f32", "f32"),
    AttnShape(8, 2, 64, "bf16", "bf16"), AttnShape(8, 2, 64, "bf16", "fp8"),
], ids=["f32-64", "f32-128", "bf16-64", "fp8-64"])
def test_generic_rows_shapes(shape):
    b = make_batch(shape, [1, 1, 1, 37, 64, 0, 1, 130], [1, 16, 333, 37, 112, 40, 17, 130], seed=21,
                   pool_rule=1.4, value_mult=0.7)
    check(b)


# ---------------------------------------------------------------------------------------------
# MFMA decode path (bf16 / fp8 cache, head_dim 128 and 64)
# ---------------------------------------------------------------------------------------------

DEC_CTX = [1, 2, 15, 16, 17, 31, 33, 64, 100, 255, 256, 257, 600, 1000, 2049, 3000]


@pytest.mark.parametrize("head_dim", [128, 64])
@pytest.mark.parametrize("kv", ["bf16", "fp8"])
@pytest.mark.parametrize("heads", [(8, 2), (4, 4), (16, 2), (32, 2), (6, 2), (10, 2), (7, 1)], ids=lambda h: f"{h[0]}q{h[1]}kv")
def test_decode_rows(kv, heads, head_dim):
    import paper_2512_03416_amd as ts
    shape = AttnShape(heads[0], heads[1], head_dim, "bf16", kv)
    b = make_batch(shape, [1] * len(DEC_CTX), DEC_CTX, seed=31, pool_rule=1.3, value_mult=0.5)
    info = ts.plan_describe(gpu().make_desc(b), b.q_lens, b.ctx_lens)
    assert info.n_decode_items >= len(DEC_CTX) and info.n_generic_rows == 0       # the matrix-core decode items
    check(b)


@pytest.mark.parametrize("head_dim", [128, 64])
@pytest.mark.parametrize("kv", ["bf16", "fp8"])
@pytest.mark.parametrize("heads", [(8, 2), (4, 4), (32, 4)], ids=lambda h: f"{h[0]}q{h[1]}kv")
def test_decode_items_append_their_rows_tokens_or_the_append_kernel_does(kv, heads, head_dim):
    """A decode-only pass with the append fused into the decode items (the wave that reads a row's last page
    patches in the new token and writes its cache entry) and with the append launch in front: same cache bytes
    as the oracle, outputs within the bar and bit-identical between the two forms, whole and split rows; new
    tokens in the first slot of a fresh page, in the last slot of a page, and anywhere in between."""
    shape = AttnShape(heads[0], heads[1], head_dim, "bf16", kv)
    ctxs = DEC_CTX + [32, 48, 49, 4096, 4097]
    mk = lambda: make_batch(shape, [1] * len(ctxs), ctxs, seed=33, pool_rule=1.3, value_mult=0.5 if kv == "bf16" else 1.0)
    ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
    g = gpu()
    for split in (0, 9):
        outs = []
        for fused in (1, 0):
            print(f"[case] decode rows kv={kv} heads={heads} D={head_dim} fused append={fused} split={split}", flush=True)
            out, gk, gv = g.run_batch(mk(), options={"decode_fused_append": fused, "decode_split_pages": split})
            assert same_bytes(gk, rk) and same_bytes(gv, rv)
            assert np.all(np.isfinite(out))
            assert float(np.max(np.abs(out - ref))) <= TOL[kv]
            outs.append(out)
        assert np.array_equal(outs[0], outs[1])


def test_fused_append_converts_every_bf16_pattern_like_the_append_kernel():
    """All 65 536 bf16 bit patterns as the new K and V of 128 decode rows (4 kv heads = 4 scales) through the fused
    form: the e4m3 cache bytes equal the oracle's (NaNs, infinities, values beyond the range, -0, denormals)."""
    import paper_2512_03416_amd as ts
    shape = AttnShape(4, 4, 128, "bf16", "fp8")
    n = 65536 // (4 * 128)
    rng = np.random.default_rng(34)
    ctxs = [int(x) for x in rng.integers(1, 70, size=n)]
    b = make_batch(shape, [1] * n, ctxs, seed=52)
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    allv = bits.view(torch.bfloat16).view(n, 4, 128)
    g = gpu()
    for rot in range(2):
        b.k_new = torch.roll(allv, rot, dims=1).contiguous()
        b.v_new = torch.roll(allv, rot + 1, dims=1).contiguous()
        b.k_scale = torch.tensor([1.0, 0.0078125, 0.0123, 3.7])
        b.v_scale = torch.tensor([1.0 / 448.0, 2.5, 0.3, 1e-3])
        print(f"[case] fused append, every bf16 pattern, rotation {rot}", flush=True)
        _, rk, rv = oracle.run_batch(W.to_cpu(b))
        _, gk, gv = g.run_batch(b, options={"decode_fused_append": 1})
        assert same_bytes(gk, rk) and same_bytes(gv, rv)
        W.to_cpu(b)


@pytest.mark.parametrize("head_dim", [128, 64])
@pytest.mark.parametrize("split", [8, 9, 64, 128])
@pytest.mark.parametrize("nbuf", [2, 3, 4])
def test_decode_split_and_prefetch_variants(split, nbuf, head_dim):
    shape = AttnShape(8, 2, head_dim, "bf16", "bf16" if (split + nbuf) % 2 else "fp8")
    b = make_batch(shape, [1] * len(DEC_CTX), DEC_CTX, seed=32, pool_rule=1.3, value_mult=0.5)
    check(b, options={"decode_split_pages": split, "decode_prefetch_tiles": nbuf})


def test_head_dim_64_mixed_batch_and_every_fp8_code():
    """Head dim 64 with a bf16 or e4m3 cache: decode rows through the matrix-core items, chunks through the
    matrix-core tiles (e4m3: widened pages; the generic kernel when widening is off), in one pass; every
    finite e4m3 code through K and V of single-key decode rows."""
    for kv in ("bf16", "fp8"):
        shape = AttnShape(16, 4, 64, "bf16", kv)
        q = [1, 1, 90, 1, 0, 33, 1, 1]
        c = [40, 1500, 150, 16, 9, 33, 4097, 1]
        check(make_batch(shape, q, c, seed=46, pool_rule=1.25, value_mult=0.5))
        check(make_batch(shape, q, c, seed=46, pool_rule=1.25, value_mult=0.5), options={"prefill_widen_pages": 0})
    shape = AttnShape(2, 2, 64, "bf16", "fp8")
    codes = [cd for cd in range(256) if (cd & 0x7F) != 0x7F]
    vals = torch.tensor([oracle.e4m3_to_double(cd) for cd in codes] + [0.0, 1.0], dtype=torch.float32)   # 256 values
    b = make_batch(shape, [1, 1], [1, 1], seed=53, value_mult=0.05)
    b.k_scale, b.v_scale = torch.tensor([1.0, 0.5]), torch.tensor([1.0, 0.25])
    for s_ in range(2):
        b.v_new[s_, 0] = vals[128 * s_:128 * s_ + 64].to(torch.bfloat16)
        b.v_new[s_, 1] = (vals[128 * s_ + 64:128 * s_ + 128] * 0.25).to(torch.bfloat16)
        b.k_new[s_, 0] = vals[128 * s_ + 64:128 * s_ + 128].to(torch.bfloat16)
        b.k_new[s_, 1] = (vals[128 * s_:128 * s_ + 64] * 0.5).to(torch.bfloat16)
    ref, rk, rv = oracle.run_batch(W.to_cpu(b))
    out, gk, gv = gpu().run_batch(b)
    assert same_bytes(gk, rk) and same_bytes(gv, rv)
    assert np.array_equal(out, ref)                          # weight 1 on one key: exact


@pytest.mark.parametrize("kv", ["bf16", "fp8"])
def test_split_rows_merged_by_their_last_item_or_by_a_launch(kv):
    """Rows cut into 2 ... 60 items: merged by the merge launch (default) and inside the decode kernel by the last
    item to arrive; both within the bar, each bit-identical over 20 repetitions on one context (the order of the
    sums is fixed, whichever item comes last), next to a prefill chunk in all three launch modes."""
    import paper_2512_03416_amd as ts
    g = gpu()
    shape = AttnShape(32, 8, 128, "bf16", kv)
    ctxs = [9000, 130, 1, 4000, 257, 33, 2100, 16, 7777, 640]
    for q, c, modes in (([1] * len(ctxs), ctxs, [0]), ([1] * len(ctxs) + [300], ctxs + [300 + 1000], [2, 1, 0])):
        mk = lambda: make_batch(shape, q, c, seed=34, pool_rule=1.2, value_mult=0.5 if kv == "bf16" else 1.0)
        ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
        for mode in modes:
            for in_kernel in (1, 0):
                b = g.to_dev(mk())
                ctx = ts.Context(g.make_desc(b))
                for k_, v_ in (("decode_split_pages", 9), ("mixed_mode", mode), ("decode_merge_in_kernel", in_kernel)):
                    ctx.set_option(k_, v_)
                print(f"[case] split rows kv={kv} rows={len(q)} mode={mode} in_kernel={in_kernel}", flush=True)
                first = None
                for rep in range(20):
                    out, gk, gv = g.run_batch(b, ctx=ctx)
                    if first is None:
                        first = out
                        assert same_bytes(gk, rk) and same_bytes(gv, rv)
                        assert float(np.max(np.abs(out - ref))) <= TOL[kv]
                    else:
                        assert np.array_equal(out, first), f"repetition {rep} differs"
                ctx.close()


def test_decode_large_scores_and_shifting_maximum():
    # keys grow along the sequence so the running maximum keeps rising across pages and splits
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    b = make_batch(shape, [1, 1], [700, 90], seed=33, value_mult=1.0, sm_scale=1.0)
    ramp = torch.linspace(0.05, 1.5, 699).view(-1, 1, 1)
    b.k_prefix[:699] = (b.k_prefix[:699].float() * ramp).to(torch.bfloat16)
    check(b, options={"decode_split_pages": 8, "decode_prefetch_tiles": 3})


# ---------------------------------------------------------------------------------------------
# MFMA prefill path
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("head_dim", [128, 64])
@pytest.mark.parametrize("kv", ["bf16", "fp8"])
@pytest.mark.parametrize("heads", [(8, 2), (4, 4), (16, 2), (32, 2), (6, 2), (10, 2), (7, 1)], ids=lambda h: f"{h[0]}q{h[1]}kv")
def test_prefill_chunks(kv, heads, head_dim):
    import paper_2512_03416_amd as ts
    shape = AttnShape(heads[0], heads[1], head_dim, "bf16", kv)
    q = [37, 64, 2, 130, 300, 17]
    pre = [0, 48, 0, 5, 200, 63]
    b = make_batch(shape, q, [a + c for a, c in zip(q, pre)], seed=41, pool_rule=1.3, value_mult=0.5)
    info = ts.plan_describe(gpu().make_desc(b), b.q_lens, b.ctx_lens)
    assert info.n_prefill_tiles >= len(q) and info.n_generic_rows == 0          # the matrix-core tiles
    check(b)


@pytest.mark.parametrize("head_dim", [128, 64])
@pytest.mark.parametrize("kv", ["bf16", "fp8"])
@pytest.mark.parametrize("heads", [(8, 2), (16, 2)], ids=lambda h: f"{h[0]}q{h[1]}kv")
def test_prefill_pipeline_boundaries(kv, heads, head_dim):
    """Chunks whose first and last tiles start at every kind of position relative to the 32-token
    half-stages, the 64-token stages and the tile size: tiles with one, two, three ... half-stages,
    with and without an unmasked steady state, prefixes that end inside a stage (cache tail beyond
    ctx_len holds the poison pattern)."""
    shape = AttnShape(heads[0], heads[1], head_dim, "bf16", kv)
    pre = [0, 1, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 159, 160, 191, 192, 193, 255, 257]
    q = [2 + (7 * i) % 70 for i in range(len(pre))]
    b = make_batch(shape, q, [a + c for a, c in zip(q, pre)], seed=43, pool_rule=1.2, value_mult=0.5)
    check(b, options={"mixed_mode": 0})


@pytest.mark.parametrize("head_dim", [128, 64])
def test_prefill_maximum_rises_late(head_dim):
    """Scores that keep growing along the context: the running maximum has to be raised again and
    again after the weights were formed (large jumps included), in the steady state and in the
    drain."""
    shape = AttnShape(8, 2, head_dim, "bf16", "bf16")
    b = make_batch(shape, [300, 70], [1500, 400], seed=44, pool_rule=1.2, value_mult=0.5)
    # scale the keys with their position: later keys score higher by construction for positive q . k
    pos_pre = torch.cat([torch.arange(1200), torch.arange(330)]).float()
    pos_new = torch.cat([1200 + torch.arange(300), 330 + torch.arange(70)]).float()
    b.k_prefix = (b.k_prefix.float() * (1.0 + pos_pre / 60.0)[:, None, None]).to(b.k_prefix.dtype)
    b.k_new = (b.k_new.float() * (1.0 + pos_new / 60.0)[:, None, None]).to(b.k_new.dtype)
    check(b, options={"mixed_mode": 0})


@pytest.mark.parametrize("kv", ["bf16", "fp8"])
def test_mixed_batch_one_pass(kv):
    shape = AttnShape(32, 8, 128, "bf16", kv)
    q = [1, 1, 200, 1, 0, 77, 1, 1, 512, 1]
    c = [40, 1500, 260, 16, 9, 77, 4097, 333, 700, 1]
    b = make_batch(shape, q, c, seed=42, pool_rule=1.25, value_mult=0.5)
    e1 = check(b)
    # appended beforehand (k_new = NULL) gives the same result as the fused pass
    b2 = make_batch(shape, q, c, seed=42, pool_rule=1.25, value_mult=0.5)
    e2 = check(b2, fused_append=False, what="pre-appended")
    assert e1 == e2


@pytest.mark.parametrize("kv", ["bf16", "fp8"])
@pytest.mark.parametrize("persistent", [2, 1, 0])
def test_mixed_batch_persistent_and_separate_launches(persistent, kv):
    """The three ways of launching a mixed batch: co-resident (resident prefill workgroups, decode grid on
    the side stream), one persistent kernel, one launch per class."""
    import paper_2512_03416_amd as ts
    shape = AttnShape(32, 8, 128, "bf16", kv)
    q = [1] * 40 + [300, 129, 1400] + [1] * 17
    rng = np.random.default_rng(5)
    c = list(rng.integers(1, 4000, size=40)) + [300 + 77, 129, 1400 + 640] + list(rng.integers(1, 600, size=17))
    b = make_batch(shape, q, c, seed=44, pool_rule=1.25, value_mult=0.5)
    g = gpu()
    assert ts.plan_describe(g.make_desc(b), b.q_lens, b.ctx_lens).mixed_mode == 2      # large enough for the default
    check(b, options={"mixed_mode": persistent})
    # a second pass on the same context must find the queue counters reset
    b = g.to_dev(make_batch(shape, q, c, seed=44, pool_rule=1.25, value_mult=0.5))
    ctx = ts.Context(g.make_desc(b))
    ctx.set_option("mixed_mode", persistent)
    outs = []
    for _ in range(3):
        o, _, _ = g.run_batch(b, ctx=ctx)
        outs.append(o)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    ctx.close()


@pytest.mark.parametrize("kv", ["bf16", "fp8"])
def test_co_resident_launch_with_any_number_of_resident_prefill_workgroups(kv):
    """The co-resident launch with a stated number of resident prefill workgroups (fewer than the dies, fewer than
    the tiles, more than the CUs) and with the planner's own choice: oracle parity each time, and the chunk rows
    bit-identical across all of them (the tiles do not depend on who runs them)."""
    import paper_2512_03416_amd as ts
    shape = AttnShape(32, 8, 128, "bf16", kv)
    rng = np.random.default_rng(8)
    q = [1] * 48 + [700, 333] + [1] * 10
    c = list(rng.integers(1, 3500, size=48)) + [700 + 1300, 333] + list(rng.integers(1, 700, size=10))
    mk = lambda: make_batch(shape, q, c, seed=47, pool_rule=1.25, value_mult=0.5 if kv == "bf16" else 1.0)
    g = gpu()
    ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
    q_off = np.concatenate([[0], np.cumsum(q)])
    rows = np.concatenate([np.arange(q_off[i], q_off[i + 1]) for i in range(len(q)) if q[i] > 1])
    outs = []
    for r in (0, 3, 8, 40, 256, 5000):
        print(f"[case] co-resident kv={kv} resident prefill workgroups={r}", flush=True)
        out, gk, gv = g.run_batch(mk(), options={"mixed_mode": 2, "prefill_resident_workgroups": r})
        assert same_bytes(gk, rk) and same_bytes(gv, rv)
        assert np.all(np.isfinite(out))
        assert float(np.max(np.abs(out - ref))) <= TOL[kv]
        outs.append(out)
    for o in outs[1:]:
        assert np.array_equal(o[rows], outs[0][rows])
    # a stated number keeps the co-resident form even for a batch the planner would launch class by class
    tiny = make_batch(shape, [1] * 40 + [20], list(rng.integers(1, 900, size=40)) + [20], seed=48, value_mult=0.5)
    assert ts.plan_describe(g.make_desc(tiny), tiny.q_lens, tiny.ctx_lens).mixed_mode == 0
    check(tiny, options={"prefill_resident_workgroups": 16})


@pytest.mark.parametrize("mode", [2, 1, 0])
def test_fp8_prefill_widened_pages_and_in_tile_widening_agree(mode):
    """fp8 cache: the prefill tiles read bf16 copies of the chunk sequences' pages made once per pass (default)
    or widen the cache themselves (option 0, or more pages than the option allows); both must match the oracle
    and each other bit for bit (the conversion is exact), in every launch mode, with ragged page tails."""
    import paper_2512_03416_amd as ts
    shape = AttnShape(32, 8, 128, "bf16", "fp8")
    q = [1] * 60 + [333, 1800, 64, 2] + [1] * 9
    rng = np.random.default_rng(6)
    c = list(rng.integers(1, 4000, size=60)) + [333 + 1111, 1800, 64 + 15, 2 + 640] + list(rng.integers(1, 900, size=9))
    mk = lambda: make_batch(shape, q, c, seed=45, pool_rule=1.25, value_mult=1.0)
    g = gpu()
    b = mk()
    info = ts.plan_describe(g.make_desc(b), b.q_lens, b.ctx_lens)
    chunk_pages = sum(-(-cl // 16) for ql, cl in zip(q, c) if ql > 1)
    assert info.widened_pages == chunk_pages and info.mixed_mode == 2
    wide = binding_export(g.make_desc(b), b, "widen")
    assert len(wide) == chunk_pages and sorted(set(wide[:, 0].tolist())) == [60, 61, 62, 63]
    ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
    outs = []
    for pages in (16384, 0, chunk_pages - 1):
        out, gk, gv = g.run_batch(mk(), options={"mixed_mode": mode, "prefill_widen_pages": pages})
        assert same_bytes(gk, rk) and same_bytes(gv, rv)
        assert float(np.max(np.abs(out - ref))) <= TOL["fp8"]
        outs.append(out)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[1], outs[2])


@pytest.mark.parametrize("kv,heads,head_dim", [("bf16", (32, 8), 128), ("fp8", (64, 8), 128), ("bf16", (8, 8), 128),
                                               ("fp8", (16, 1), 128), ("bf16", (32, 8), 64), ("fp8", (16, 2), 64)])
def test_prefill_tiles_cut_along_the_keys(kv, heads, head_dim):
    """A short chunk over a long prefix cannot give every CU a tile: the tiles are cut along the keys and the
    parts merged.  Chunks whose prefix ends inside a page, a stage and a part; parts of 64 keys (the finest cut)
    and the default; next to decode rows (one persistent kernel) and alone; same results with cutting off."""
    import paper_2512_03416_amd as ts
    shape = AttnShape(heads[0], heads[1], head_dim, "bf16", kv)
    g = gpu()
    for q, c in [([200], [200 + 4099]), ([64, 37], [64 + 2048, 37 + 1000]), ([1, 130, 1, 1], [700, 130 + 3001, 64, 2500])]:
        mk = lambda: make_batch(shape, q, c, seed=61, pool_rule=1.2, value_mult=0.5 if kv == "bf16" else 1.0)
        b = mk()
        assert ts.plan_describe(g.make_desc(b), b.q_lens, b.ctx_lens).prefill_parts > 1
        ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
        outs = []
        last = {"prefill_split_min_keys": 64, "mixed_mode": 0}
        if head_dim == 128:
            last["prefill_widen_pages"] = 0                  # (head dim 64 reads an e4m3 cache through widened pages only)
        for opts in ({}, {"prefill_split_min_keys": 64}, {"prefill_split_min_keys": 0}, last):
            print(f"[case] cut tiles kv={kv} heads={heads} q={q} ctx={c} opts={opts}", flush=True)
            out, gk, gv = g.run_batch(mk(), options=opts)
            assert same_bytes(gk, rk) and same_bytes(gv, rv)
            assert np.all(np.isfinite(out))
            err = float(np.max(np.abs(out - ref)))
            print(f"       max abs err {err:.3e}", flush=True)
            assert err <= TOL[kv]
            outs.append(out)
        # same cuts, other launch mode / widening: the chunk rows come out bit-identical (decode rows may be
        # cut into other page ranges in another launch mode)
        q_off = np.concatenate([[0], np.cumsum(q)])
        rows = np.concatenate([np.arange(q_off[i], q_off[i + 1]) for i in range(len(q)) if q[i] > 1])
        assert np.array_equal(outs[1][rows], outs[3][rows])


def binding_export(desc, b, which):
    from paper_2512_03416_amd import binding
    return binding.plan_export(desc, b.q_lens, b.ctx_lens, which)


def test_prefill_generic_path_agrees():
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    b = make_batch(shape, [150, 1], [190, 50], seed=43, value_mult=0.5)
    check(b, options={"prefill_path": 1})


# ---------------------------------------------------------------------------------------------
# append and fp8 codec
# ---------------------------------------------------------------------------------------------

def test_fp8_append_exhaustive_bf16_inputs():
    """All 65536 bf16 bit patterns through ts_kv_append (4 kv heads = 4 scales), bit-exact."""
    shape = AttnShape(4, 4, 128, "bf16", "fp8")
    n = 65536 // (4 * 128)                                       # tokens so that K holds every pattern once
    b = make_batch(shape, [n], [n], seed=51)
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    allv = bits.view(torch.bfloat16).view(n, 4, 128)
    # every head sees every pattern: rotate the assignment over 4 passes
    for rot in range(4):
        b.k_new = torch.roll(allv, rot, dims=1).contiguous()
        b.v_new = torch.roll(allv, rot + 1, dims=1).contiguous()
        b.k_scale = torch.tensor([1.0, 0.0078125, 0.0123, 3.7])
        b.v_scale = torch.tensor([1.0 / 448.0, 2.5, 0.3, 1e-3])
        b.name = f"fp8_exhaustive_rot{rot}"
        print(f"[case] {b.name}", flush=True)
        kc = oracle.new_cache(b.num_pages, 4, 128, "fp8")
        vc = oracle.new_cache(b.num_pages, 4, 128, "fp8")
        oracle.kv_append(4, 4, 128, "bf16", "fp8", oracle.raw(b.k_new), oracle.raw(b.v_new), kc, vc,
                         oracle.raw(b.k_scale), oracle.raw(b.v_scale), b.block_table, b.q_lens, b.ctx_lens,
                         b.num_pages)
        import paper_2512_03416_amd as ts
        g = gpu()
        b = g.to_dev(b)
        ctx = ts.Context(g.make_desc(b))
        gk, gv = g.new_caches(b)
        bt = torch.from_numpy(b.block_table).cuda()
        ctx.kv_append(b.k_new, b.v_new, gk, gv, b.k_scale, b.v_scale, bt, b.q_lens, b.ctx_lens)
        torch.cuda.synchronize()
        assert same_bytes(g.cache_raw(gk, "fp8"), kc)
        assert same_bytes(g.cache_raw(gv, "fp8"), vc)
        ctx.close()
        W.to_cpu(b)


@pytest.mark.parametrize("q_len", [1, 3])
def test_fp8_every_code_dequantises_exactly(q_len):
    """A row that sees one key returns that key's value: run every finite e4m3 code through K and V,
    through the decode kernel (q_len 1) and the prefill kernel (first row of a chunk)."""
    shape = AttnShape(2, 2, 128, "bf16", "fp8")
    codes = [c for c in range(256) if (c & 0x7F) != 0x7F]
    vals = torch.tensor([oracle.e4m3_to_double(c) for c in codes], dtype=torch.float32)   # exact in bf16
    vals = torch.cat([vals, vals[:2]])                                                   # 256 values
    S = 2
    b = make_batch(shape, [q_len] * S, [q_len] * S, seed=52, value_mult=0.05)
    b.k_scale = torch.tensor([1.0, 0.5])
    b.v_scale = torch.tensor([1.0, 0.25])
    for s in range(S):
        row = s * q_len                                      # first row of each sequence sees one key
        b.v_new[row, 0] = vals[:128].to(torch.bfloat16)
        b.v_new[row, 1] = (vals[128:] * 0.25).to(torch.bfloat16)
        b.k_new[row, 0] = vals[128:].to(torch.bfloat16)      # K goes through every code as well
        b.k_new[row, 1] = (vals[:128] * 0.5).to(torch.bfloat16)
    print(f"[case] fp8 single-key rows q_len={q_len}", flush=True)
    ref, rk, rv = oracle.run_batch(W.to_cpu(b))
    out, gk, gv = gpu().run_batch(b)
    assert same_bytes(gk, rk) and same_bytes(gv, rv)
    first = [s * q_len for s in range(S)]
    assert np.array_equal(out[first], ref[first])            # weight 1 on one key: exact
    rel = np.abs(out - ref) / np.maximum(1.0, np.abs(ref))
    assert float(rel.max()) <= 6e-2


def test_append_only_entry_point_bit_exact():
    import paper_2512_03416_amd as ts
    g = gpu()
    for shape in (AttnShape(4, 1, 64, "f32", "f32"), AttnShape(8, 2, 128, "bf16", "bf16"),
                  AttnShape(8, 2, 128, "bf16", "fp8")):
        b = make_batch(shape, [1, 37, 64, 3, 0, 500], [70, 37, 112, 16, 5, 777], seed=53, pool_rule=1.7)
        print(f"[case] append_only {shape}", flush=True)
        _, rk, rv = oracle.run_batch(b)
        b = g.to_dev(b)
        ctx = ts.Context(g.make_desc(b))
        gk, gv = g.new_caches(b)
        bt = torch.from_numpy(b.block_table).cuda()
        pre = b.prefix_lens
        ctx.kv_append(b.k_prefix, b.v_prefix, gk, gv, b.k_scale, b.v_scale, bt, pre, pre)
        ctx.kv_append(b.k_new, b.v_new, gk, gv, b.k_scale, b.v_scale, bt, b.q_lens, b.ctx_lens)
        torch.cuda.synchronize()
        assert same_bytes(g.cache_raw(gk, shape.kv_dtype), rk)
        assert same_bytes(g.cache_raw(gv, shape.kv_dtype), rv)
        ctx.close()


@pytest.mark.parametrize("kv", ["bf16", "fp8"])
def test_append_page_alignments_bit_exact(kv):
    """Chunks that start and end anywhere inside a page, next to short sequences that take the
    per-token kernel: every byte of both caches equals the oracle's, untouched bytes included."""
    g = gpu()
    q_lens = [7, 8, 9, 16, 17, 33, 100, 1, 8, 15, 16, 48, 2]
    prefix = [3, 0, 15, 16, 5, 31, 77, 40, 9, 1, 8, 32, 14]
    shape = AttnShape(8, 4, 128, "bf16", kv)
    b = make_batch(shape, q_lens, [q + p for q, p in zip(q_lens, prefix)], seed=59, pool_rule=1.3)
    print(f"[case] append_alignments {shape}", flush=True)
    _, rk, rv = oracle.run_batch(b)
    _, gk, gv = g.run_batch(b)
    assert same_bytes(gk, rk)
    assert same_bytes(gv, rv)


# ---------------------------------------------------------------------------------------------
# boundary behaviour on the GPU
# ---------------------------------------------------------------------------------------------

def test_errors_have_no_side_effects_and_empty_batches_are_fine():
    import paper_2512_03416_amd as ts
    from paper_2512_03416_amd import binding
    g = gpu()
    b = g.to_dev(make_batch(AttnShape(8, 2, 128, "bf16", "bf16"), [1, 5], [20, 30], seed=61))
    ctx = ts.Context(g.make_desc(b))
    kc, vc = g.new_caches(b)
    bt = torch.from_numpy(b.block_table).cuda()
    out = torch.zeros_like(b.q)
    before = kc.clone()
    for ql, cl in (([1, 31], [20, 30]), ([-1, 5], [20, 30]), ([1, 5], [20, 16 * b.max_pages_per_seq + 1])):
        with pytest.raises(ts.TokenScaleError) as e:
            ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, None, None, bt, ql, cl, 0.0, out)
        assert e.value.code == binding.TS_ERR_INVALID_ARG and ctx.last_error()
    with pytest.raises(ts.TokenScaleError):
        ctx.mixed_paged_attention(b.q, b.k_new, None, kc, vc, None, None, bt, b.q_lens, b.ctx_lens, 0.0, out)
    with pytest.raises(ts.TokenScaleError):
        ctx.set_option("no_such_option", 1)
    torch.cuda.synchronize()
    assert torch.equal(kc, before) and float(out.float().abs().sum()) == 0.0
    # empty batches
    ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, None, None, bt, [], [], 0.0, out)
    ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, None, None, bt, [0, 0], [3, 0], 0.0, out)
    ctx.kv_append(b.k_new, b.v_new, kc, vc, None, None, bt, [0, 0], [3, 0])
    torch.cuda.synchronize()
    assert torch.equal(kc, before)
    ctx.close()


def test_block_table_validation_option_catches_bad_page_ids():
    """Debug option: a page id outside the pool in a page the batch uses fails the call before any
    kernel has touched the caches; ids in unused entries of the table are never looked at."""
    import paper_2512_03416_amd as ts
    from paper_2512_03416_amd import binding
    g = gpu()
    b = g.to_dev(make_batch(AttnShape(8, 2, 128, "bf16", "bf16"), [1, 40, 3], [70, 90, 3], seed=63))
    ctx = ts.Context(g.make_desc(b))
    ctx.set_option("validate_block_table", 1)
    kc, vc = g.new_caches(b)
    out = torch.zeros_like(b.q)
    before_k, before_v = kc.clone(), vc.clone()
    table = b.block_table.copy()
    used = [(int(c) + 15) // 16 for c in b.ctx_lens]
    for s in range(len(used)):
        table[s, used[s]:] = -1                                  # unused entries: anything goes
    good = torch.from_numpy(table).cuda()
    for s, p, bad_id in ((1, used[1] - 1, b.num_pages), (0, 0, -1), (2, 0, 2 ** 31 - 1)):
        bad = table.copy()
        bad[s, p] = bad_id
        bt = torch.from_numpy(bad).cuda()
        for call in ("attention", "append"):
            with pytest.raises(ts.TokenScaleError) as e:
                if call == "attention":
                    ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, None, None, bt, b.q_lens, b.ctx_lens, 0.0, out)
                else:
                    ctx.kv_append(b.k_new, b.v_new, kc, vc, None, None, bt, b.q_lens, b.ctx_lens)
            assert e.value.code == binding.TS_ERR_INVALID_ARG
            assert f"sequence {s}, page {p}" in ctx.last_error()
    torch.cuda.synchronize()
    assert torch.equal(kc, before_k) and torch.equal(vc, before_v) and float(out.float().abs().sum()) == 0.0
    # the same table without the planted ids passes, and the pass still matches the oracle
    ctx.set_option("validate_block_table", 1)
    b.block_table = table
    ref, rk, rv = oracle.run_batch(W.to_cpu(make_batch(AttnShape(8, 2, 128, "bf16", "bf16"), [1, 40, 3], [70, 90, 3], seed=63)))
    o, gk, gv = g.run_batch(b, ctx=ctx)
    assert same_bytes(gk, rk) and same_bytes(gv, rv)
    assert float(np.max(np.abs(o - ref))) <= TOL["bf16"]
    ctx.close()


def test_run_to_run_identical_and_default_scale():
    g = gpu()
    shape = AttnShape(32, 8, 128, "bf16", "bf16")
    mk = lambda: make_batch(shape, [1, 1, 300, 1], [3000, 555, 420, 64], seed=62, value_mult=0.5)
    o1, k1, _ = g.run_batch(mk(), options={"decode_split_pages": 8})
    o2, k2, _ = g.run_batch(mk(), options={"decode_split_pages": 8})
    assert np.array_equal(o1, o2) and np.array_equal(k1, k2)
    b = mk()
    b.sm_scale = 0.0                       # <= 0 selects 1/sqrt(D)
    o3, _, _ = g.run_batch(b, options={"decode_split_pages": 8})
    assert np.array_equal(o1, o3)


def test_context_follows_stream_switch():
    """Calls of one context may move to another stream without a host synchronisation in between:
    the library orders the new stream behind its previous call (its work lists share one buffer)."""
    import paper_2512_03416_amd as ts
    g = gpu()
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    b = make_batch(shape, [1, 300, 1, 64], [900, 700, 33, 64], seed=64, value_mult=0.5)
    print("[case] stream switch", flush=True)
    ref, rk, rv = oracle.run_batch(b)
    b = g.to_dev(b)
    ctx = ts.Context(g.make_desc(b))
    kc, vc = g.new_caches(b)
    bt = torch.from_numpy(b.block_table).cuda()
    out = torch.zeros_like(b.q)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    pre = b.prefix_lens
    ctx.kv_append(b.k_prefix, b.v_prefix, kc, vc, None, None, bt, pre, pre, stream=s1)
    ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, None, None, bt, b.q_lens, b.ctx_lens, b.sm_scale, out,
                              stream=s2)
    torch.cuda.synchronize()
    assert same_bytes(g.cache_raw(kc, "bf16"), rk) and same_bytes(g.cache_raw(vc, "bf16"), rv)
    assert float(np.max(np.abs(out.double().cpu().numpy() - ref))) <= 2e-2
    ctx.close()


def test_token_velocity_counters():
    import time
    import paper_2512_03416_amd as ts
    g = gpu()
    b = g.to_dev(make_batch(AttnShape(8, 2, 128, "bf16", "bf16"), [1, 1, 40, 1, 7], [20, 30, 40, 5, 9], seed=63))
    ctx = ts.Context(g.make_desc(b))
    kc, vc = g.new_caches(b)
    bt = torch.from_numpy(b.block_table).cuda()
    out = torch.zeros_like(b.q)
    v0 = ctx.token_velocity()
    assert v0.passes == 0 and v0.window_s == 0.0 and v0.decode_tok_per_s == 0.0
    for _ in range(3):
        ctx.mixed_paged_attention(b.q, b.k_new, b.v_new, kc, vc, None, None, bt, b.q_lens, b.ctx_lens, 0.0, out)
    time.sleep(0.05)
    v = ctx.token_velocity(reset=True, sync=True)
    assert (v.passes, v.decode_tokens, v.prefill_tokens) == (3, 9, 141)
    assert v.window_s >= 0.05
    assert abs(v.decode_tok_per_s - 9 / v.window_s) < 1e-6 * v.decode_tok_per_s + 1e-9
    assert abs(v.prefill_tok_per_s - 141 / v.window_s) < 1e-6 * v.prefill_tok_per_s + 1e-9
    assert ctx.token_velocity().passes == 0
    ctx.close()


def test_chunk_size_profiler_sweep():
    """Sec. 4.4 sweep on a small decoder: times grow with the chunk, the choice is the oracle's choice
    on the measured times, velocity and reservation follow from it."""
    from oracle import velocity as ov
    from paper_2512_03416_amd import profiler
    res = profiler.main(["--heads", "8,2", "--decode-batch", "16", "--ctx-min", "200", "--ctx-max", "600",
                         "--chunks", "64,256,1024", "--layers", "4", "--tpot-slo-ms", "100", "--steps", "5"])
    times = [p["iteration_attention_ms"] * 1e-3 for p in res["sweep"]]
    assert all(t > 0 for t in times) and times[-1] > times[0]
    assert res["chosen_index"] == ov.largest_admissible_chunk(times, res["attention_budget_ms"] * 1e-3)
    if res["chosen_index"] >= 0:
        c = res["sweep"][res["chosen_index"]]["chunk_size"]
        v = ov.convertible_prefill_velocity(c, 16, 0.1)
        assert res["prefill_velocity_tok_per_s"] == v
        assert res["reserved_bytes"] == ov.reserved_memory(v, 2 * 2 * 128 * 2 * 4, 0.4)


def test_burst_replay_accounts_for_every_token():
    """A short 2 -> 12 requests/s step through one small Convertible Decoder: batches change shape
    every iteration (new prefill task, rows finishing), the library's velocity counters see exactly
    the rows that were submitted, every admitted request gets its first token."""
    from paper_2512_03416_amd import replay
    res = replay.main(["--heads", "8,2", "--seconds", "3", "--step-at", "1", "--rps", "2,12", "--drain", "2",
                       "--in-median", "120", "--in-max", "600", "--out-median", "12", "--out-max", "40",
                       "--chunk-size", "256", "--layers", "2", "--other-ms", "4", "--max-resident", "64"])
    assert res["iterations"] > 50 and res["passes_counted"] == res["iterations"]
    assert res["prefill_tokens_counted"] == res["prefill_tokens_submitted"]
    assert res["decode_tokens_counted"] == res["decode_tokens_submitted"]
    assert res["requests"] > 10 and res["first_tokens"] >= res["requests"] - 2
    assert res["completed"] >= res["first_tokens"] - 40 and res["completed"] > 0


REPLAY_ARGS = ["--heads", "8,2", "--seconds", "3", "--step-at", "1", "--rps", "2,12", "--drain", "2",
               "--in-median", "120", "--in-max", "600", "--out-median", "12", "--out-max", "40",
               "--layers", "2", "--other-ms", "4"]


@pytest.mark.parametrize("chunk,resident", [(256, 64), (24, 48)])
def test_burst_replay_against_the_scheduler_oracle_and_the_attention_oracle(chunk, resident):
    """The replay with a given pass time (1 us per query token + 20 us) forms exactly the batches of the
    scheduler oracle, iteration by iteration, with the same first-token and completion times; a CPU mirror of
    the cache follows every pass through the oracle's append, and every 9th pass is recomputed by the attention
    oracle: outputs within the bf16 bar, the cache pages of every sequence of the pass byte-equal.
    (24, 48): the chunk size is below the number of resident requests, so the decode batch alone can exceed it.)"""
    from oracle import replay as orp
    from paper_2512_03416_amd import replay
    time_fn = lambda q, c: 1e-6 * sum(q) + 20e-6
    Hq, Hkv, D = 8, 2, 128
    state = dict(kc=None, vc=None, checked=0, worst=0.0)

    def on_pass(i, dec):
        if state["kc"] is None:
            state["kc"] = oracle.new_cache(dec.num_pages, Hkv, D, "bf16")
            state["vc"] = oracle.new_cache(dec.num_pages, Hkv, D, "bf16")
        last = dec.last
        T, bt = last["T"], last["bt"].cpu().numpy()
        args = (Hq, Hkv, D, "bf16", "bf16")
        oracle.kv_append(*args, oracle.raw(dec.k[:T]), oracle.raw(dec.v[:T]), state["kc"], state["vc"], None, None, bt,
                         last["q_lens"], last["ctx_lens"], dec.num_pages)
        if i % 9:
            return
        ref = oracle.mixed_paged_attention(*args, oracle.raw(dec.q[:T]), state["kc"], state["vc"], None, None, bt,
                                           last["q_lens"], last["ctx_lens"], 1.0 / np.sqrt(D), dec.num_pages)
        out = dec.out[:T].double().cpu().numpy()
        state["worst"] = max(state["worst"], float(np.max(np.abs(out - ref))))
        page_elems = Hkv * 16 * D
        ids = np.unique(np.concatenate([bt[s, :-(-int(c) // 16)] for s, c in enumerate(last["ctx_lens"])]))
        gk = dec.kc.view(torch.int16).view(-1, page_elems)[torch.from_numpy(ids.astype(np.int64)).cuda()].cpu().numpy()
        gv = dec.vc.view(torch.int16).view(-1, page_elems)[torch.from_numpy(ids.astype(np.int64)).cuda()].cpu().numpy()
        assert np.array_equal(gk.view(np.uint16), state["kc"].reshape(-1, page_elems)[ids]), f"K pages differ at pass {i}"
        assert np.array_equal(gv.view(np.uint16), state["vc"].reshape(-1, page_elems)[ids]), f"V pages differ at pass {i}"
        state["checked"] += 1

    res = replay.main(REPLAY_ARGS + ["--chunk-size", str(chunk), "--max-resident", str(resident)],
                      time_fn=time_fn, on_pass=on_pass, record=True)
    its, first, done = orp.schedule(res["arrivals"], chunk_size=chunk, max_resident=resident,
                                    num_pages=res["num_pages"], max_pages_per_seq=res["max_pages_per_seq"],
                                    pass_time=time_fn, layers=2, other_s=4e-3, horizon_s=5.0)
    assert len(its) > 50 and res["iteration_log"] == its
    assert res["first_token_at"] == first and res["done_at"] == done
    assert state["checked"] >= 6 and state["worst"] <= TOL["bf16"]
    print(f"       {len(its)} iterations equal to the scheduler oracle, {state['checked']} passes recomputed, "
          f"max abs err {state['worst']:.3e}", flush=True)


def test_mfma_calibration_stream_runs_and_counts_its_work():
    """The calibration launch returns, leaves the result word alone and reports
    CUs x 8 waves x iters x 16 MFMAs x 32768 flop."""
    import paper_2512_03416_amd as ts
    ops = torch.randn(65536, device="cuda").to(torch.bfloat16)
    res = torch.zeros(1, dtype=torch.float32, device="cuda")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    for softmax in (False, True):
        flops = ts.calib_mfma(ops, res, 50, softmax)
        torch.cuda.synchronize()
        assert flops == n_cu * 8 * 50 * 16 * 32768
        assert float(res.item()) == 0.0


@pytest.mark.parametrize("seed", range(8))
def test_seeded_random_batches(seed):
    """Batches drawn from a seeded generator: random head geometry, cache type, number of sequences,
    a length mix of empty sequences, decode rows and chunks of any size over prefixes of any length
    (page-aligned or not), persistent or separate launches, forced or automatic decode splits."""
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 2, 3, 4, 8]))
    kv = str(rng.choice(["bf16", "fp8"]))
    shape = AttnShape(hkv * group, hkv, 128, "bf16", kv)
    n = int(rng.integers(1, 14))
    q, c = [], []
    for _ in range(n):
        kind = rng.choice(["empty", "decode", "decode", "decode", "chunk", "chunk"])
        if kind == "empty":
            ql, pre = 0, int(rng.integers(0, 200))
        elif kind == "decode":
            ql, pre = 1, int(rng.choice([0, int(rng.integers(0, 64)), int(rng.integers(0, 3000))]))
        else:
            ql = int(rng.choice([2, int(rng.integers(2, 40)), int(rng.integers(40, 700))]))
            pre = int(rng.choice([0, 16 * int(rng.integers(0, 20)), int(rng.integers(0, 1500))]))
        q.append(ql)
        c.append(ql + pre)
    if sum(q) == 0:
        q[0], c[0] = 1, c[0] + 1
    opts = {"mixed_mode": int(rng.integers(0, 3))}
    if rng.integers(0, 2):
        opts["decode_split_pages"] = int(rng.choice([8, 13, 40]))
    b = make_batch(shape, q, c, seed=2000 + seed, pool_rule=1.3, value_mult=0.5)
    print(f"[case] random batch {seed}: q={q} ctx={c}", flush=True)
    check(b, options=opts)


def test_one_context_many_different_batches_in_a_row():
    """Twelve batches of different shape through one context, back to back: the staging ring for the work
    lists (four slots) is refilled several times, and every pass must be planned from its own lists."""
    import paper_2512_03416_amd as ts
    g = gpu()
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    rng = np.random.default_rng(77)
    batches = []
    for i in range(12):
        n = int(rng.integers(1, 9))
        q = [int(rng.choice([0, 1, 1, 1, int(rng.integers(2, 300))])) for _ in range(n)]
        if sum(q) == 0:
            q[0] = 1
        c = [ql + int(rng.integers(0, 900)) for ql in q]
        batches.append(make_batch(shape, q, c, seed=300 + i, pool_rule=1.3, value_mult=0.5))
    num_pages = max(b.num_pages for b in batches)
    stride = max(b.max_pages_per_seq for b in batches)
    refs = [oracle.run_batch(W.to_cpu(b)) for b in batches]
    ctx = ts.Context(ts.Desc.make(8, 2, 128, "bf16", "bf16", num_pages, stride))
    for i, b in enumerate(batches):
        table = np.full((b.num_seqs, stride), -1, dtype=np.int32)
        table[:, :b.block_table.shape[1]] = b.block_table
        b.block_table = table
        b.num_pages = num_pages
        print(f"[case] batch {i} on the shared context: q={list(b.q_lens)} ctx={list(b.ctx_lens)}", flush=True)
        out, gk, gv = g.run_batch(b, ctx=ctx)
        ref, rk, rv = refs[i]
        n_el = rk.size                                          # the oracle's pool is the batch's own, smaller one
        assert same_bytes(gk[:n_el], rk) and same_bytes(gv[:n_el], rv)
        assert float(np.max(np.abs(out - ref))) <= TOL["bf16"]
    ctx.close()


def test_two_contexts_keep_their_own_options():
    """Options are per context: one context with four tiles in flight per decode wave and forced splits,
    one with the defaults, called in turns on one GPU; each reports its own settings and both match the
    oracle."""
    import paper_2512_03416_amd as ts
    g = gpu()
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    mk = lambda: make_batch(shape, [1, 1, 90, 1], [2500, 300, 150, 17], seed=72, value_mult=0.5)
    b = g.to_dev(mk())
    ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
    c1, c2 = ts.Context(g.make_desc(b)), ts.Context(g.make_desc(b))
    c1.set_option("decode_prefetch_tiles", 4)
    c1.set_option("decode_split_pages", 16)
    c1.set_option("mixed_mode", 0)
    assert c1.get_option("decode_prefetch_tiles") == 4 and c2.get_option("decode_prefetch_tiles") == 2
    assert c1.get_option("decode_split_pages") == 16 and c2.get_option("decode_split_pages") == 0
    assert c1.get_option("mixed_mode") == 0 and c2.get_option("mixed_mode") == 2
    for _ in range(2):
        for c in (c1, c2):
            out, gk, gv = g.run_batch(b, ctx=c)
            assert same_bytes(gk, rk) and same_bytes(gv, rv)
            assert float(np.max(np.abs(out - ref))) <= TOL["bf16"]
    assert c1.get_option("decode_prefetch_tiles") == 4 and c2.get_option("decode_prefetch_tiles") == 2
    c1.close()
    c2.close()


def test_side_stream_probe_settles_with_many_contexts_alive():
    """The co-resident launch needs its side stream to run next to the caller's stream.  Twelve contexts alive
    at once (so that some side streams share a hardware queue with the caller's stream), five passes each:
    every context has an answer from its probe after the second pass, ends either side by side or after the
    most probes it may send, and every pass of every context gives the same bytes (and matches the oracle)."""
    import paper_2512_03416_amd as ts
    g = gpu()
    shape = AttnShape(32, 8, 128, "bf16", "bf16")
    rng = np.random.default_rng(9)
    q = [1] * 40 + [1000, 150]
    c = list(rng.integers(200, 3000, size=40)) + [1000 + 1500, 150]
    mk = lambda: make_batch(shape, q, c, seed=73, pool_rule=1.25, value_mult=0.5)
    b = g.to_dev(mk())
    ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
    assert ts.plan_describe(g.make_desc(b), b.q_lens, b.ctx_lens).mixed_mode == 2
    ctxs = [ts.Context(g.make_desc(b)) for _ in range(12)]
    first = None
    for rep in range(5):
        for i, ctx in enumerate(ctxs):
            out, gk, gv = g.run_batch(b, ctx=ctx)
            if first is None:
                first = out
                assert same_bytes(gk, rk) and same_bytes(gv, rv)
                assert float(np.max(np.abs(out - ref))) <= TOL["bf16"]
            assert np.array_equal(out, first), f"context {i}, pass {rep}"
            if rep >= 1:
                assert ctx.get_option("side_stream_probes") >= 1
    states = [(ctx.get_option("side_stream_overlap"), ctx.get_option("side_stream_probes")) for ctx in ctxs]
    print(f"[case] side stream probes (answer, probes): {states}", flush=True)
    for ans, n in states:
        assert (ans == 1 and 1 <= n <= 4) or (ans == 2 and n == 4)
    for ctx in ctxs:
        ctx.close()


def test_reserve_then_no_growth_and_kernel_timing_counts():
    """ts_reserve sizes the scratch for the largest batch to come (a pass within it matches the oracle);
    with kernel timing on every pass, ts_kernel_times counts one launch of each kernel the batch
    needs per pass, reports positive means, and forgets them on reset."""
    import paper_2512_03416_amd as ts
    from paper_2512_03416_amd import binding
    g = gpu()
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    mk = lambda: make_batch(shape, [1, 1, 200, 1], [3000, 555, 420, 64], seed=71, value_mult=0.5)
    b = g.to_dev(mk())
    ctx = ts.Context(g.make_desc(b))
    with pytest.raises(ts.TokenScaleError) as e:
        ctx.reserve(-1, 4, 100)
    assert e.value.code == binding.TS_ERR_INVALID_ARG
    ctx.set_option("decode_split_pages", 8)                  # split rows: decode, combine and prefill all run
    ctx.set_option("mixed_mode", 0)
    ctx.reserve(4096, 64, 4096)                              # (sized for the options in force)
    n_alloc = ctx.get_option("scratch_allocations")
    ctx.set_option("kernel_timing", 1)
    ref, rk, rv = oracle.run_batch(W.to_cpu(mk()))
    for _ in range(3):
        out, gk, gv = g.run_batch(b, ctx=ctx)
    assert ctx.get_option("scratch_allocations") == n_alloc  # nothing grew
    with pytest.raises(ts.TokenScaleError):
        ctx.get_option("no_such_option")
    assert same_bytes(gk, rk) and same_bytes(gv, rv)
    assert float(np.max(np.abs(out - ref))) <= TOL["bf16"]
    kt = ctx.kernel_times()
    # each run_batch = one prefix append + one pass (append, decode, combine, prefill)
    assert kt["append"][0] == 6 and kt["decode"][0] == 3 and kt["combine"][0] == 3 and kt["prefill"][0] == 3
    assert kt["mixed"][0] == 0 and kt["rows"][0] == 0
    assert all(v[1] > 0 for k, v in kt.items() if v[0])
    again = ctx.kernel_times(reset=True)
    assert again == kt
    assert all(v == (0, 0.0) for v in ctx.kernel_times().values())
    ctx.set_option("kernel_timing", 0)
    g.run_batch(b, ctx=ctx)
    assert all(v == (0, 0.0) for v in ctx.kernel_times().values())
    ctx.close()
