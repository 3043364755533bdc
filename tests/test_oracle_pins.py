"""Pins for the fp64 oracle (CPU only).

The paper prints no number for the attention pass, so the oracle is pinned by what the
mathematics fixes: a dense brute-force evaluation built from the generator's logical K/V rows
(no paging, explicit boolean mask, naive exp/sum), closed forms, invariants, and an exhaustive
nearest-value search for the e4m3 encoder.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from workloads import AttnShape, make_batch

PAGE = 16


# ------------------------------------------------------------------------------------------
# independent helpers (numpy / torch library routines only)
# ------------------------------------------------------------------------------------------

def seq_logical_kv(batch, s):
    """[ctx, Hkv, D] float64 K and V rows of sequence s from the generator's tensors."""
    pre = batch.prefix_lens
    po = int(pre[:s].sum())
    qo = int(batch.q_lens[:s].sum())
    k = torch.cat([batch.k_prefix[po:po + pre[s]], batch.k_new[qo:qo + batch.q_lens[s]]]).double()
    v = torch.cat([batch.v_prefix[po:po + pre[s]], batch.v_new[qo:qo + batch.q_lens[s]]]).double()
    return k.numpy(), v.numpy()


def quantise_lib(x, scale):
    """Library e4m3 quantise->dequantise of rows x [n,Hkv,D] (in-range values only)."""
    xs = (torch.as_tensor(x).float() / scale.view(1, -1, 1).float())
    q8 = xs.to(torch.float8_e4m3fn)
    return (q8.double() * scale.view(1, -1, 1).double()).numpy()


def dense_bruteforce(batch):
    """Dense [q,c] scores with an explicit causal mask, naive exp(z)/sum exp(z), matmul."""
    sh = batch.shape
    G = sh.group
    outs = []
    for s in range(batch.num_seqs):
        ql, cl = int(batch.q_lens[s]), int(batch.ctx_lens[s])
        if ql == 0:
            continue
        k, v = seq_logical_kv(batch, s)
        if sh.kv_dtype == "fp8":
            k = quantise_lib(k, batch.k_scale)
            v = quantise_lib(v, batch.v_scale)
        qo = int(batch.q_lens[:s].sum())
        q = batch.q[qo:qo + ql].double().numpy()                      # [ql,Hq,D]
        rows = np.arange(ql)[:, None] + (cl - ql)                      # absolute position of row
        mask = np.arange(cl)[None, :] <= rows                          # [ql,cl] boolean
        o = np.zeros((ql, sh.num_q_heads, sh.head_dim))
        for h in range(sh.num_q_heads):
            z = batch.sm_scale * q[:, h, :] @ k[:, h // G, :].T        # [ql,cl]
            e = np.where(mask, np.exp(z), 0.0)
            p = e / e.sum(axis=1, keepdims=True)
            o[:, h, :] = p @ v[:, h // G, :]
        outs.append(o)
    return np.concatenate(outs) if outs else np.zeros((0, sh.num_q_heads, sh.head_dim))


def logical_view_k(cache, num_pages, Hkv, D, kv_dtype):
    """Documented K tile order [D/x][16][x] undone with numpy reshapes -> [page,Hkv,16,D]."""
    x = 16 // oracle.ELEM_SIZE[kv_dtype]
    return cache.reshape(num_pages, Hkv, D // x, PAGE, x).transpose(0, 1, 3, 2, 4).reshape(
        num_pages, Hkv, PAGE, D)


def logical_view_v(cache, num_pages, Hkv, D):
    return cache.reshape(num_pages, Hkv, D, PAGE).transpose(0, 1, 3, 2)


SHAPES = [
    AttnShape(4, 1, 64, "f32", "f32"),
    AttnShape(8, 2, 128, "bf16", "bf16"),
    AttnShape(6, 3, 32, "f32", "f32"),
    AttnShape(8, 2, 64, "bf16", "fp8"),
]


# ------------------------------------------------------------------------------------------
# whole result: brute force
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"{s.q_dtype}-{s.kv_dtype}-{s.num_q_heads}-{s.num_kv_heads}-{s.head_dim}")
def test_matches_dense_bruteforce(shape):
    b = make_batch(shape, [1, 1, 37, 64, 1, 5, 0], [1, 77, 37, 112, 16, 33, 9], seed=11,
                   pool_rule=1.5, value_mult=0.5, sm_scale=0.173)
    out, _, _ = oracle.run_batch(b)
    ref = dense_bruteforce(b)
    assert out.shape == ref.shape
    assert np.max(np.abs(out - ref)) <= 1e-12


def test_config1_matches_dense_bruteforce():
    b = W.config1()
    assert list(b.q_lens[6:]) == [37, 64] and list(b.ctx_lens[6:]) == [37, 112]
    assert np.all(b.q_lens[:6] == 1) and np.all((b.ctx_lens[:6] >= 1) & (b.ctx_lens[:6] <= 200))
    out, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(out - dense_bruteforce(b))) <= 1e-12


# ------------------------------------------------------------------------------------------
# softmax weights
# ------------------------------------------------------------------------------------------

def _filled(b):
    sh = b.shape
    out, kc, vc = oracle.run_batch(b)
    ks = None if b.k_scale is None else oracle.raw(b.k_scale)
    vs = None if b.v_scale is None else oracle.raw(b.v_scale)
    return out, kc, vc, ks, vs


@pytest.mark.parametrize("shape", SHAPES[:2] + SHAPES[3:], ids=["f32", "bf16", "fp8"])
def test_weight_rows_sum_to_one(shape):
    b = make_batch(shape, [1, 9], [50, 30], seed=3, pool_rule=1.3)
    out, kc, vc, ks, vs = _filled(b)
    sh = b.shape
    for (row, s, n) in [(0, 0, 50), (1, 1, 22), (9, 1, 30)]:
        for h in range(sh.num_q_heads):
            w, o = oracle.attention_row(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype,
                                        sh.kv_dtype, oracle.raw(b.q), kc, vc, ks, vs,
                                        b.block_table[s], n, row, h, b.sm_scale, b.num_pages)
            assert w.shape == (n,)
            assert np.all(w >= 0)
            assert abs(w.sum() - 1.0) <= 1e-14
            assert np.max(np.abs(o - out[row, h])) == 0.0


# ------------------------------------------------------------------------------------------
# special cases with closed forms
# ------------------------------------------------------------------------------------------

def test_single_key_returns_its_value_exactly():
    for shape in SHAPES[:3]:
        b = make_batch(shape, [1, 1], [1, 1], seed=5)
        out, _, _ = oracle.run_batch(b)
        G = shape.group
        for s in range(2):
            for h in range(shape.num_q_heads):
                assert np.array_equal(out[s, h], b.v_new[s, h // G].double().numpy())


def test_zero_query_gives_running_mean_of_values():
    shape = AttnShape(4, 2, 64, "f32", "f32")
    b = make_batch(shape, [23, 1], [40, 19], seed=6, q_zero=True)
    out, _, _ = oracle.run_batch(b)
    for s, (ql, cl) in enumerate(zip(b.q_lens, b.ctx_lens)):
        _, v = seq_logical_kv(b, s)
        qo = int(b.q_lens[:s].sum())
        for i in range(ql):
            n = cl - ql + i + 1
            for h in range(4):
                mean = v[:n, h // 2, :].mean(axis=0)
                assert np.max(np.abs(out[qo + i, h] - mean)) <= 1e-13


def test_constant_values_give_that_constant():
    shape = AttnShape(4, 2, 64, "f32", "f32")
    b = make_batch(shape, [7, 1], [30, 45], seed=7)
    b.v_new[:] = 0.625
    b.v_prefix[:] = 0.625
    out, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(out - 0.625)) <= 1e-14


def test_dominant_key_selects_its_value():
    shape = AttnShape(2, 1, 64, "f32", "f32")
    b = make_batch(shape, [1], [40], seed=8)
    # key 17 is aligned with both query heads and 60x longer than the rest
    qsum = b.q[0].sum(dim=0)
    b.k_prefix[17, 0] = 60.0 * qsum / qsum.norm()
    # make sure both heads have a positive projection on it
    b.q[0, 0] = qsum / 2
    b.q[0, 1] = qsum / 2
    out, _, _ = oracle.run_batch(b)
    for h in range(2):
        assert np.max(np.abs(out[0, h] - b.v_prefix[17, 0].double().numpy())) <= 1e-9


def test_linear_in_values():
    shape = AttnShape(4, 2, 64, "f32", "f32")
    b = make_batch(shape, [5, 1], [21, 33], seed=9)
    o12, _, _ = oracle.run_batch(b)
    v_new, v_pre = b.v_new.clone(), b.v_prefix.clone()
    # split V = V1 + V2 exactly (fp32 values with few mantissa bits so the split is exact)
    v1n, v1p = torch.round(v_new * 4) / 4, torch.round(v_pre * 4) / 4
    b.v_new, b.v_prefix = v1n, v1p
    o1, _, _ = oracle.run_batch(b)
    b.v_new, b.v_prefix = v_new - v1n, v_pre - v1p
    o2, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(o12 - (o1 + o2))) <= 1e-13


# ------------------------------------------------------------------------------------------
# paging
# ------------------------------------------------------------------------------------------

def test_page_permutation_leaves_output_bit_identical():
    shape = AttnShape(8, 2, 128, "bf16", "bf16")
    b = make_batch(shape, [1, 40, 1], [100, 75, 16], seed=10, pool_rule=2.0)
    o1, _, _ = oracle.run_batch(b)
    rng = np.random.default_rng(99)
    perm = rng.permutation(b.num_pages).astype(np.int32)
    bt = b.block_table.copy()
    bt[bt >= 0] = perm[bt[bt >= 0]]
    b.block_table = bt
    o2, _, _ = oracle.run_batch(b)
    assert np.array_equal(o1, o2)


def test_unused_slots_are_poison_and_never_read():
    b = make_batch(AttnShape(4, 2, 64, "bf16", "bf16"), [1, 3], [5, 19], seed=12, pool_rule=3.0)
    out, kc, vc = oracle.run_batch(b)
    assert np.all(np.isfinite(out))
    # the cache started as all-0xFF bytes: everything outside the written slots is still 0xFFFF
    kl = logical_view_k(kc, b.num_pages, 2, 64, "bf16")
    written = np.zeros((b.num_pages, PAGE), dtype=bool)
    for s in range(b.num_seqs):
        for pos in range(int(b.ctx_lens[s])):
            written[b.block_table[s, pos // PAGE], pos % PAGE] = True
    vl = logical_view_v(vc, b.num_pages, 2, 64)
    assert (~written).any()
    for g in range(2):
        assert np.all(kl[:, g][~written] == 0xFFFF)
        assert np.all(vl[:, g][~written] == 0xFFFF)
        assert not np.any(np.all(kl[:, g][written] == 0xFFFF, axis=-1))


# ------------------------------------------------------------------------------------------
# row sampling (the full-size GPU parity tests and the bench's CPU leg recompute a sample of rows)
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("kv", ["f32", "bf16", "fp8"])
def test_row_sampling_selects_exactly_the_strided_rows(kv):
    """row_stride = k, row_offset = o must give rows o, o+k, ... bit-identical to the same rows of
    the run over all rows (which the dense brute force pins), and leave every other row untouched."""
    shape = AttnShape(8, 2, 64, "f32" if kv == "f32" else "bf16", kv)
    b = make_batch(shape, [1, 9, 0, 1, 23, 1], [40, 9, 17, 1, 60, 33], seed=41, pool_rule=1.5)
    sh = b.shape
    args = (sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype, sh.kv_dtype)
    full, kc, vc = oracle.run_batch(b)
    T = b.total_q
    assert T == 35 and np.all(np.isfinite(full))
    assert np.max(np.abs(full - dense_bruteforce(b))) <= 1e-12
    ks = None if b.k_scale is None else oracle.raw(b.k_scale)
    vs = None if b.v_scale is None else oracle.raw(b.v_scale)
    for stride, off in [(1, 0), (2, 0), (2, 1), (3, 2), (7, 5), (7, 0), (34, 34), (35, 0), (100, 3), (1, 12),
                        (5, 35), (4, 1000), (0, 0)]:
        got = oracle.mixed_paged_attention(*args, oracle.raw(b.q), kc, vc, ks, vs, b.block_table, b.q_lens,
                                           b.ctx_lens, b.sm_scale, b.num_pages, row_stride=stride,
                                           row_offset=off)
        want_rows = list(range(off, T, max(stride, 1)))      # a stride below 1 means every row
        sel = np.zeros(T, dtype=bool)
        sel[want_rows] = True
        assert np.array_equal(got[sel], full[sel]), (stride, off)
        assert np.all(np.isnan(got[~sel])), (stride, off)
        assert int((~np.isnan(got[:, 0, 0])).sum()) == len(want_rows)


def test_row_sampling_rows_belong_to_the_right_sequence():
    """A sampled row must be computed with its own sequence's page list and key count: compare with
    the one-row entry point called with those, sequence by sequence."""
    b = make_batch(AttnShape(4, 2, 64, "bf16", "bf16"), [5, 1, 12], [21, 70, 12], seed=42, pool_rule=1.2)
    sh = b.shape
    args = (sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype, sh.kv_dtype)
    _, kc, vc = oracle.run_batch(b)
    got = oracle.mixed_paged_attention(*args, oracle.raw(b.q), kc, vc, None, None, b.block_table, b.q_lens,
                                       b.ctx_lens, b.sm_scale, b.num_pages, row_stride=4, row_offset=3)
    q_off = np.concatenate([[0], np.cumsum(b.q_lens)])
    n = 0
    for row in range(3, b.total_q, 4):
        s = int(np.searchsorted(q_off, row, side="right") - 1)
        n_keys = int(b.ctx_lens[s] - b.q_lens[s] + (row - q_off[s]) + 1)
        for h in range(sh.num_q_heads):
            _, o = oracle.attention_row(*args, oracle.raw(b.q), kc, vc, None, None, b.block_table[s], n_keys,
                                        row, h, b.sm_scale, b.num_pages)
            assert np.array_equal(got[row, h], o)
        n += 1
    assert n == 4


# ------------------------------------------------------------------------------------------
# chunking
# ------------------------------------------------------------------------------------------

def _run_chunks(shape, L, chunks, k_all, v_all, q_all, seed):
    """Prefill a prompt of L tokens in the given chunk sizes; returns [L,Hq,D]."""
    outs = []
    done = 0
    for c in chunks:
        b = make_batch(shape, [c], [done + c], seed=seed, pool_rule=1.0)
        b.k_prefix, b.v_prefix = k_all[:done].clone(), v_all[:done].clone()
        b.k_new, b.v_new = k_all[done:done + c].clone(), v_all[done:done + c].clone()
        b.q = q_all[done:done + c].clone()
        o, _, _ = oracle.run_batch(b)
        outs.append(o)
        done += c
    assert done == L
    return np.concatenate(outs)


def test_chunked_prefill_equals_whole_prompt_and_decode_rows():
    shape = AttnShape(4, 2, 64, "f32", "f32")
    L = 134
    g = torch.Generator().manual_seed(21)
    k_all = torch.randn(L, 2, 64, generator=g)
    v_all = torch.randn(L, 2, 64, generator=g)
    q_all = torch.randn(L, 4, 64, generator=g)
    whole = _run_chunks(shape, L, [L], k_all, v_all, q_all, 1)
    parts = _run_chunks(shape, L, [37, 64, 1, 15, 17], k_all, v_all, q_all, 2)
    assert np.max(np.abs(whole - parts)) <= 1e-14
    dec = _run_chunks(shape, L, [100] + [1] * 34, k_all, v_all, q_all, 3)
    assert np.max(np.abs(whole - dec)) <= 1e-14


# ------------------------------------------------------------------------------------------
# grouped-query mapping
# ------------------------------------------------------------------------------------------

def test_gqa_equals_replicated_kv_heads():
    shape = AttnShape(8, 2, 64, "f32", "f32")
    b = make_batch(shape, [1, 6], [44, 20], seed=13)
    o1, _, _ = oracle.run_batch(b)
    rep = AttnShape(8, 8, 64, "f32", "f32")
    b2 = make_batch(rep, [1, 6], [44, 20], seed=13)
    b2.block_table, b2.num_pages = b.block_table, b.num_pages
    b2.q = b.q
    for name in ("k_new", "v_new", "k_prefix", "v_prefix"):
        setattr(b2, name, getattr(b, name).repeat_interleave(4, dim=1).contiguous())
    o2, _, _ = oracle.run_batch(b2)
    assert np.array_equal(o1, o2)
    # head h depends only on kv head h // G: perturb kv head 1, heads 0..3 unchanged
    b.k_new[:, 1] += 1.0
    b.v_prefix[:, 1] -= 2.0
    o3, _, _ = oracle.run_batch(b)
    assert np.array_equal(o1[:, :4], o3[:, :4]) and not np.array_equal(o1[:, 4:], o3[:, 4:])


# ------------------------------------------------------------------------------------------
# append
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("shape", SHAPES[:3], ids=["f32-64", "bf16-128", "f32-32"])
def test_append_round_trip_and_layout(shape):
    b = make_batch(shape, [1, 37, 64, 3], [70, 37, 112, 16], seed=14, pool_rule=1.7)
    _, kc, vc = oracle.run_batch(b)
    Hkv, D = shape.num_kv_heads, shape.head_dim
    kl = logical_view_k(kc, b.num_pages, Hkv, D, shape.kv_dtype)
    vl = logical_view_v(vc, b.num_pages, Hkv, D)
    for s in range(b.num_seqs):
        k, v = seq_logical_kv(b, s)
        for pos in range(int(b.ctx_lens[s])):
            page = b.block_table[s, pos // PAGE]
            kr, vr = kl[page, :, pos % PAGE, :], vl[page, :, pos % PAGE, :]
            if shape.kv_dtype == "bf16":
                kr = torch.from_numpy(kr.astype(np.int16)).view(torch.bfloat16).double().numpy()
                vr = torch.from_numpy(vr.astype(np.int16)).view(torch.bfloat16).double().numpy()
            assert np.array_equal(kr, k[pos]) and np.array_equal(vr, v[pos])


def test_append_fp8_matches_library_quantiser_in_range():
    shape = AttnShape(8, 2, 64, "bf16", "fp8")
    b = make_batch(shape, [1, 20], [40, 20], seed=15)
    _, kc, vc = oracle.run_batch(b)
    kl = logical_view_k(kc, b.num_pages, 2, 64, "fp8")
    vl = logical_view_v(vc, b.num_pages, 2, 64)
    for s in range(b.num_seqs):
        k, v = seq_logical_kv(b, s)
        k8 = (torch.as_tensor(k).float() / b.k_scale.view(1, -1, 1)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        v8 = (torch.as_tensor(v).float() / b.v_scale.view(1, -1, 1)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        for pos in range(int(b.ctx_lens[s])):
            page = b.block_table[s, pos // PAGE]
            assert np.array_equal(kl[page, :, pos % PAGE, :], k8[pos])
            assert np.array_equal(vl[page, :, pos % PAGE, :], v8[pos])


# ------------------------------------------------------------------------------------------
# e4m3 codec: exhaustive
# ------------------------------------------------------------------------------------------

def _e4m3_table():
    """All 256 e4m3fn values from the format's definition (bias 7, no inf, S.1111.111 = NaN)."""
    vals = np.empty(256)
    for b in range(256):
        s, e, m = b >> 7, (b >> 3) & 15, b & 7
        if e == 15 and m == 7:
            v = math.nan
        elif e == 0:
            v = m * 2.0 ** -9
        else:
            v = (8 + m) * 2.0 ** (e - 10)
        vals[b] = -v if s else v
    return vals


def test_e4m3_decode_table_against_definition_and_library():
    tab = _e4m3_table()
    got = np.array([oracle.e4m3_to_double(b) for b in range(256)])
    assert np.array_equal(np.isnan(tab), np.isnan(got))
    ok = ~np.isnan(tab)
    assert np.array_equal(tab[ok], got[ok])
    assert np.signbit(got[0x80]) and got[0x80] == 0.0
    libv = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(libv[ok], got[ok])
    assert got[0x7E] == 448.0 and np.nanmax(got) == 448.0


def _nearest_search(y, tab_pos):
    """Brute-force nearest e4m3 magnitude index (0..126) for |y| < 464, ties -> even code."""
    a = abs(y)
    d = np.abs(tab_pos - a)
    best = np.flatnonzero(d == d.min())
    if len(best) == 1:
        return int(best[0])
    assert len(best) == 2
    return int(best[0] if best[0] % 2 == 0 else best[1])


def test_e4m3_encode_exhaustive_bf16_inputs():
    tab = _e4m3_table()
    tab_pos = tab[:127]                                  # 0x00..0x7E ascending, 0x7F is NaN
    scales = [1.0, 0.0078125, 0.0123, 3.7, 1.0 / 448.0]
    bits = np.arange(1 << 16, dtype=np.uint32)
    xs = (bits << 16).astype(np.uint32).view(np.float32)
    for sc in scales:
        ys = (xs / np.float32(sc)).astype(np.float32)    # IEEE single division
        for idx in range(0, 1 << 16, 1):
            x, y = float(xs[idx]), float(ys[idx])
            code = oracle.e4m3_encode(x, sc)
            sign = 0x80 if math.copysign(1.0, y) < 0 else 0
            if math.isnan(y):
                assert code == (sign | 0x7F)
            elif abs(y) >= 448.0:
                assert code == (sign | 0x7E)             # saturation, inf included
            else:
                assert code == (sign | _nearest_search(y, tab_pos)), (x, sc, y, code)


def test_e4m3_encode_properties():
    tab = _e4m3_table()
    # every representable value encodes to itself, -0 keeps its sign, monotone, half-ulp bound
    for b in range(256):
        if not math.isnan(tab[b]):
            assert oracle.e4m3_encode(float(tab[b]), 1.0) == b
    ys = np.linspace(-500, 500, 20001).astype(np.float32)
    codes = np.array([oracle.e4m3_encode(float(y), 1.0) for y in ys])
    dec = np.array([oracle.e4m3_to_double(int(c)) for c in codes])
    assert np.all(np.diff(dec) >= 0)
    inr = np.abs(ys) <= 448
    ulp = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(ys[inr]), 2.0 ** -6))) - 3), 2.0 ** -9)
    assert np.all(np.abs(dec[inr] - ys[inr]) <= ulp / 2 + 1e-12)
    assert dec[0] == -448 and dec[-1] == 448
    # exact ties go to the even mantissa: 17 is halfway between 16 (0x58) and 18 (0x59)
    assert oracle.e4m3_encode(17.0, 1.0) == 0x58 and oracle.e4m3_encode(19.0, 1.0) == 0x5A
    # the fp32 division is rounded once in single precision
    x, sc = np.float32(1.7), np.float32(0.3)
    assert oracle.e4m3_encode(float(x), float(sc)) == oracle.e4m3_encode(float(np.float32(x / sc)), 1.0)
