"""CPU-only checks of the boundary: exported symbols, descriptor/batch validation, planner."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2512_03416_amd as ts
from paper_2512_03416_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tokenscale.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ts_[a-z_0-9]+)\s*\(", hdr))
    assert {"ts_kv_append", "ts_mixed_paged_attention", "ts_token_velocity"} <= declared
    lib = ctypes.CDLL(ts.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


def test_library_exports_every_policy_symbol():
    from paper_2512_03416_amd import policy
    hdr = open(os.path.join(ROOT, "include", "tokenscale_policy.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ts_[a-z_0-9]+)\s*\(", hdr))
    lib = ctypes.CDLL(ts.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(policy.EXPORTS)
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert headers == ["tokenscale.h", "tokenscale_calib.h", "tokenscale_policy.h"]   # each has a symbol test


def test_library_exports_every_calibration_symbol():
    hdr = open(os.path.join(ROOT, "include", "tokenscale_calib.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ts_[a-z_0-9]+)\s*\(", hdr))
    lib = ctypes.CDLL(ts.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(binding.CALIB_EXPORTS)


def D(**kw):
    base = dict(Hq=32, Hkv=8, D=128, q_dtype="bf16", kv_dtype="bf16", num_pages=1000, max_pages_per_seq=64)
    base.update(kw)
    return ts.Desc.make(**base)


def test_check_desc_accepts_and_rejects():
    assert ts.check_desc(D()) == 0
    assert ts.check_desc(D(q_dtype="f32", kv_dtype="f32", D=64, Hq=4, Hkv=1)) == 0
    assert ts.check_desc(D(kv_dtype="fp8", Hq=64)) == 0
    assert ts.check_desc(D(page_size=32)) == binding.TS_ERR_INVALID_ARG
    assert ts.check_desc(D(Hq=30)) == binding.TS_ERR_INVALID_ARG
    assert ts.check_desc(D(num_pages=0)) == binding.TS_ERR_INVALID_ARG
    assert ts.check_desc(D(D=96)) == binding.TS_ERR_UNSUPPORTED
    assert ts.check_desc(D(q_dtype="f32", kv_dtype="bf16")) == binding.TS_ERR_UNSUPPORTED
    assert ts.check_desc(D(q_dtype=7)) == binding.TS_ERR_INVALID_ARG
    assert ts.check_desc(D(Hq=8 * 17)) == binding.TS_ERR_UNSUPPORTED


def test_cache_bytes():
    assert ts.cache_bytes(D()) == 1000 * 8 * 16 * 128 * 2
    assert ts.cache_bytes(D(kv_dtype="fp8")) == 1000 * 8 * 16 * 128
    assert ts.cache_bytes(D(q_dtype="f32", kv_dtype="f32", D=64)) == 1000 * 8 * 16 * 64 * 4
    assert ts.cache_bytes(D(D=96)) == 0


@pytest.mark.parametrize("ql,cl", [([-1], [4]), ([5], [4]), ([1], [64 * 16 + 1])])
def test_plan_rejects_bad_lengths(ql, cl):
    with pytest.raises(ts.TokenScaleError) as e:
        ts.plan_describe(D(), ql, cl)
    assert e.value.code == binding.TS_ERR_INVALID_ARG


def test_plan_counts_and_decode_items_cover_every_page_once():
    rng = np.random.default_rng(5)
    ctx = rng.integers(1, 1024, size=40)
    ql = np.ones(40, dtype=np.int32)
    ql[::7] = 0
    ql[3] = 37
    ctx[3] = 112
    ql[9] = 300
    ctx[9] = 300
    for split in (0, 8, 13, 128):
        info = ts.plan_describe(D(), ql, ctx, split)
        n_dec = int((ql == 1).sum())
        assert info.total_tokens == ql.sum() and info.decode_tokens == n_dec
        assert info.prefill_tokens == 337
        assert info.n_generic_rows == 0
        assert info.tile_tokens == 64
        assert info.n_prefill_tiles == -(-37 // 64) + -(-300 // 64)
        items = ts.plan_decode_items(D(), ql, ctx, split)
        assert len(items) == info.n_decode_items
        cover = {}
        for row, seq, n_keys, pb, pe in items:
            assert ql[seq] == 1 and n_keys == ctx[seq] and 0 <= pb < pe <= -(-n_keys // 16)
            assert pe - pb <= max(info.split_pages, 1)
            assert row == ql[:seq].sum()
            cover.setdefault(seq, []).extend(range(pb, pe))
        assert set(cover) == {s for s in range(40) if ql[s] == 1}
        for seq, pages in cover.items():
            assert sorted(pages) == list(range(-(-ctx[seq] // 16)))
        lens = items[:, 4] - items[:, 3]
        assert np.all(np.diff(lens) <= 0)                 # longest first
        n_split_rows = sum(1 for s in cover if len([1 for it in items if it[1] == s]) > 1)
        assert info.n_combine_rows == n_split_rows
        assert info.partial_slots == sum(len([1 for it in items if it[1] == s]) for s in cover
                                         if len([1 for it in items if it[1] == s]) > 1)


def test_plan_append_pages_cover_every_new_token_of_the_chunks_once():
    """Page-wise append work: each new token of a sequence with >= 8 new tokens lies in exactly one
    (page, slot range) record, and the record's row arithmetic points at that token's input row."""
    from paper_2512_03416_amd import binding
    rng = np.random.default_rng(5)
    q_lens = rng.integers(0, 70, size=60).astype(np.int32)
    q_lens[:6] = [0, 1, 7, 8, 16, 17]
    prefix = rng.integers(0, 50, size=60).astype(np.int32)
    ctx = q_lens + prefix
    desc = binding.Desc.make(8, 2, 128, "bf16", "bf16", 4096, 16)
    rec = binding.plan_export(desc, q_lens, ctx, "append")
    q_off = np.concatenate([[0], np.cumsum(q_lens)])
    seen = {}
    for seq, pg, lo, hi, row0, *_ in rec:
        assert q_lens[seq] >= 8 and 0 <= lo < hi <= 16
        for slot in range(lo, hi):
            pos = pg * 16 + slot
            assert prefix[seq] <= pos < ctx[seq]
            assert row0 + slot == q_off[seq] + pos - prefix[seq]
            assert (seq, pos) not in seen
            seen[(seq, pos)] = True
    assert len(seen) == int(q_lens[q_lens >= 8].sum())
    # the other tokens, and all tokens of shapes the page-wise kernel does not take, go one by one
    rows = binding.plan_export(desc, q_lens, ctx, "append_rows")
    want = [(q_off[s] + i, s, prefix[s] + i, 0) for s in range(len(q_lens)) if q_lens[s] < 8 for i in range(q_lens[s])]
    assert [tuple(r) for r in rows] == want
    d64 = binding.Desc.make(4, 1, 64, "f32", "f32", 4096, 16)
    assert len(binding.plan_export(d64, q_lens, ctx, "append")) == 0
    assert len(binding.plan_export(d64, q_lens, ctx, "append_rows")) == int(q_lens.sum())
    # head dim 64 with bf16 inputs is appended page-wise like head dim 128 (same lists)
    for kv in ("bf16", "fp8"):
        d64b = binding.Desc.make(8, 2, 64, "bf16", kv, 4096, 16)
        assert np.array_equal(binding.plan_export(d64b, q_lens, ctx, "append"), rec)
        assert np.array_equal(binding.plan_export(d64b, q_lens, ctx, "append_rows"), rows)


def test_plan_routes_fp32_to_generic_rows_and_head_dim_64_to_the_matrix_cores():
    d = D(q_dtype="f32", kv_dtype="f32", D=64, Hq=4, Hkv=1)
    info = ts.plan_describe(d, [1, 37, 64], [5, 37, 112])
    assert info.n_generic_rows == 102 and info.n_decode_items == 0 and info.n_prefill_tiles == 0
    # head dim 64, bf16 cache: decode rows are matrix-core items, chunks matrix-core tiles, one launch per class
    info = ts.plan_describe(D(D=64), [1, 4], [5, 4])
    assert info.n_generic_rows == 0 and info.n_decode_items == 1 and info.n_prefill_tiles == 1 and info.mixed_mode == 0
    # head dim 64, e4m3 cache: the tiles read widened pages; without them the chunk rows take the generic kernel
    info = ts.plan_describe(D(D=64, kv_dtype="fp8"), [1, 1, 40], [5, 1000, 17 + 40])
    assert info.n_generic_rows == 0 and info.n_decode_items >= 2 and info.n_prefill_tiles >= 1 and info.widened_pages == 4
    rows = binding.plan_export(D(D=64, kv_dtype="fp8", max_pages_per_seq=20000), [40], [40 + 16 * 16384], "rows")
    assert len(rows) == 40                                    # more pages than the widening scratch takes


def test_plan_sizes_the_co_resident_launch_from_the_two_costs():
    """A mixed batch is launched co-resident with as many resident prefill workgroups as the ratio of the two
    classes' estimated times asks for (all CUs when the tiles dominate, fewer -- in multiples of the die count --
    when the decode scan outlasts them); a batch in which either class is short goes class by class."""
    rng = np.random.default_rng(3)
    dec = rng.integers(1024, 8193, 128).tolist()
    d = D(max_pages_per_seq=2048, num_pages=200000)

    def plan(chunks):
        q = [1] * len(dec) + [c for c, _ in chunks]
        ctx = dec + [c + p for c, p in chunks]
        return ts.plan_describe(d, q, ctx)
    burst = plan([(2048, 0), (2048, 1500), (2048, 3000), (2048, 4096)])            # tiles ~ as long as the scan
    assert burst.mixed_mode == 2 and 160 <= burst.prefill_workgroups < 256 and burst.prefill_workgroups % 8 == 0
    heavy = plan([(4096, 4096)] * 4)                                                 # tiles dominate
    assert heavy.mixed_mode == 2 and heavy.prefill_workgroups == 256
    one = plan([(1920, 4096)])                                                       # the scan dominates
    assert one.mixed_mode == 2 and 64 <= one.prefill_workgroups <= 160 and one.prefill_workgroups % 8 == 0
    small = plan([(384, 4096)])
    assert small.mixed_mode == 2 and 8 <= small.prefill_workgroups <= 96
    assert plan([(128, 0)]).mixed_mode == 0 and plan([(128, 0)]).prefill_workgroups == 0
    few = ts.plan_describe(d, [1, 1, 2048], [100, 200, 2048])                        # hardly any decode pages
    assert few.mixed_mode == 0 and few.prefill_workgroups == 0
    # monotone in the prefill work
    sizes = [plan([(n, 4096)]).prefill_workgroups for n in (512, 1024, 2048, 4096, 8192)]
    assert sizes == sorted(sizes) and sizes[-1] == 256


def test_create_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(ts.TokenScaleError) as e:
        ts.Context(D())
    assert e.value.code == binding.TS_ERR_HIP


def test_calibration_helpers_reject_bad_arguments_before_touching_a_gpu():
    lib = binding.load_library()
    flops = ctypes.c_int64(-1)
    one = ctypes.c_void_p(16)                                  # never dereferenced: the checks come first
    assert lib.ts_calib_mfma(None, None, one, 10, 0, ctypes.byref(flops)) == -1
    assert lib.ts_calib_mfma(None, one, None, 10, 0, ctypes.byref(flops)) == -1
    assert lib.ts_calib_mfma(None, one, one, 0, 0, ctypes.byref(flops)) == -1
    assert lib.ts_calib_mfma(None, one, one, 200001, 1, ctypes.byref(flops)) == -1
    assert lib.ts_calib_mfma(None, one, one, 10, 1, None) == -1
    assert flops.value == -1
    assert lib.ts_calib_copy(None, one, one, 24) == -1         # not a multiple of 16
    assert lib.ts_calib_read(None, one, None, 32) == -1


@pytest.mark.parametrize("seed", range(6))
def test_plan_invariants_on_seeded_random_batches(seed):
    """Every list of the planner against what the batch demands, for random mixes of empty sequences,
    decode rows and chunks: each cache page of a decode row in exactly one item, partial slots
    contiguous per split row, each chunk token in exactly one tile, each (tile, head) once in the launch
    order and once in the queues, each (decode item, head) once in the queues, append work covering each
    new token once."""
    rng = np.random.default_rng(4000 + seed)
    hkv = int(rng.choice([1, 2, 8]))
    group = int(rng.choice([1, 4, 8]))
    desc = binding.Desc.make(hkv * group, hkv, 128, "bf16", str(rng.choice(["bf16", "fp8"])), 1 << 16, 1024)
    n = int(rng.integers(1, 40))
    kinds = rng.choice(["empty", "decode", "decode", "chunk"], size=n)
    ql = np.array([0 if k == "empty" else 1 if k == "decode" else int(rng.integers(2, 900)) for k in kinds], dtype=np.int32)
    ctx = ql + rng.integers(0, 6000, size=n).astype(np.int32)
    split = int(rng.choice([0, 0, 8, 37]))
    slots = int(rng.choice([0, 96, 768]))
    mode = int(rng.choice([-1, 0, 1, 2]))
    exp = lambda which: binding.plan_export(desc, ql, ctx, which, split, slots, mode)
    q_off = np.concatenate([[0], np.cumsum(ql)])
    pages = -(-ctx // 16)
    tile_tokens = 256 // group

    dec, cmb = exp("decode"), exp("combine")
    cover, slots_of = {}, {}
    for row, seq, n_keys, pb, pe, part, *_ in dec:
        assert ql[seq] == 1 and row == q_off[seq] and n_keys == ctx[seq] and 0 <= pb < pe <= pages[seq]
        cover.setdefault(seq, []).extend(range(pb, pe))
        slots_of.setdefault(seq, []).append(part)
    assert set(cover) == {s for s in range(n) if ql[s] == 1}
    for s, pg in cover.items():
        assert sorted(pg) == list(range(pages[s]))
    split_rows = {s for s, p in slots_of.items() if len(p) > 1}
    assert all(p == [-1] for s, p in slots_of.items() if s not in split_rows)
    used = []
    assert len(cmb) == len(split_rows)
    for row, begin, n_split, _ in cmb:
        s = int(np.searchsorted(q_off, row, side="right") - 1)
        while ql[s] == 0:
            s += 1
        assert s in split_rows and sorted(slots_of[s]) == list(range(begin, begin + n_split))
        used.extend(range(begin, begin + n_split))
    assert sorted(used) == list(range(len(used)))

    pf = exp("prefill")
    toks, part_keys = {}, {}
    for seq, row0, q_len, prefix, t0, cnt, ctx_len, part, kv_b, kv_e, *_ in pf:
        assert ql[seq] > 1 and row0 == q_off[seq] and q_len == ql[seq] and prefix == ctx[seq] - ql[seq] and ctx_len == ctx[seq]
        assert t0 % tile_tokens == 0 and 0 < cnt <= tile_tokens
        hi = prefix + t0 + cnt                                    # keys the tile's last row sees
        if part < 0:
            assert kv_b == 0 and kv_e >= hi
            toks.setdefault(seq, []).extend(range(t0, t0 + cnt))
        else:                                                     # a part of a tile cut along the keys
            assert kv_b % 64 == 0 and kv_b <= prefix + t0 and kv_b < min(kv_e, hi)
            assert kv_e % 64 == 0 or kv_e >= hi
            part_keys.setdefault((seq, t0, cnt), []).append((kv_b, min(kv_e, hi), part))
    for (seq, t0, cnt), parts in part_keys.items():               # the parts of a tile cover its keys exactly once
        parts.sort()
        assert len(parts) > 1 and parts[0][0] == 0 and parts[-1][1] == ctx[seq] - ql[seq] + t0 + cnt
        assert all(a[1] == b[0] for a, b in zip(parts, parts[1:]))
        assert all(e <= ctx[seq] - ql[seq] + t0 for _, e, _ in parts[:-1])        # only the last part meets the diagonal
        assert [p for _, _, p in parts] == list(range(parts[0][2], parts[0][2] + len(parts)))
        toks.setdefault(seq, []).extend(range(t0, t0 + cnt))
    pfc = exp("pfcombine")
    assert len(pfc) == len(part_keys)
    for item, p0, n_part, _ in pfc:
        seq, _, _, _, t0, cnt, *_ = pf[item]
        assert len(part_keys[(seq, t0, cnt)]) == n_part and min(p for _, _, p in part_keys[(seq, t0, cnt)]) == p0
    assert set(toks) == {s for s in range(n) if ql[s] > 1}
    for s, t in toks.items():
        assert sorted(t) == list(range(ql[s]))

    pfmap = exp("pfmap")
    live = [(int(t), int(g)) for t, g in pfmap if t >= 0]
    assert sorted(live) == sorted((t, g) for t in range(len(pf)) for g in range(hkv))      # (every part is a work item)

    queue, qoff = exp("queue"), exp("qoff")[:, 0]
    if len(dec) and len(pf) and mode == 1:
        assert len(queue)                                     # (asked for by name: no other launch form is chosen)
    if len(dec) and len(pf) and mode != 0 and len(queue):     # a mixed batch has per-die queues, unless the planner
        assert len(qoff) == 9 and qoff[0] == 0 and qoff[-1] == len(queue) and np.all(np.diff(qoff) >= 0)
        d_entries = sorted((int(i), int(g)) for k, i, g, _ in queue if k == 0)
        p_entries = sorted((int(i), int(g)) for k, i, g, _ in queue if k == 1)
        # launches it class by class (either class too short for the co-resident launch to pay).
        # One persistent kernel: both kinds are queued; co-resident launch: the tiles only
        assert d_entries in ([], sorted((i, g) for i in range(len(dec)) for g in range(hkv)))
        assert mode != 1 or d_entries
        assert p_entries == sorted((t, g) for t in range(len(pf)) for g in range(hkv))
    else:
        assert len(queue) == 0

    seen = set()
    for seq, pg, lo, hi, row0, *_ in exp("append"):
        for slot in range(lo, hi):
            pos = pg * 16 + slot
            assert (seq, pos) not in seen and row0 + slot == q_off[seq] + pos - (ctx[seq] - ql[seq])
            seen.add((seq, pos))
    for row, seq, pos, _ in exp("append_rows"):
        assert (seq, pos) not in seen and row == q_off[seq] + pos - (ctx[seq] - ql[seq])
        seen.add((seq, pos))
    assert seen == {(s, p) for s in range(n) for p in range(ctx[s] - ql[s], ctx[s])}


def test_kernels_fit_their_register_budget_without_spilling():
    """The co-resident launch rests on register budgets: resident prefill workgroups at <= 192 vector registers
    per lane (two waves per SIMD) next to a lean decode workgroup at <= 128, and no kernel may spill (a spill
    reload waits for every load in flight, the stage copies included).  Compiles the kernel sources for gfx950
    with the library's flags and reads the compiler's resource remarks."""
    import subprocess
    from paper_2512_03416_amd import build as B
    budgets = {"prefill_resident_kernel": 192, "prefill_kernel": 192, "decode_kernel_lean": 128, "mixed_kernel": 256,
               "decode_kernel": 256}
    seen = set()
    for src in ("ts_kernels_mixed.hip", "ts_kernels_prefill.hip", "ts_kernels_decode.hip"):
        r = subprocess.run([B.HIPCC] + B.FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-x", "hip", "-c",
                                                 os.path.join(B.CSRC, src), "-o", os.devnull],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        name = None
        for line in r.stderr.splitlines():
            m = re.search(r"Function Name: (\S+)", line)
            if m:
                name = m.group(1)
            m = re.search(r" VGPRs: (\d+)", line)
            if m and name:
                key = next((k for k in sorted(budgets, key=len, reverse=True) if k in name), None)
                if key:
                    assert int(m.group(1)) <= budgets[key], (name, line)
                    seen.add(key)
            m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
            if m and name:
                assert int(m.group(1)) == 0, f"{name} uses scratch memory (spills)"
    assert seen == set(budgets)
