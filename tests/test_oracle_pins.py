"""Pins for the CPU oracle: closed forms, brute force, invariants, library routines.

None of these retypes the oracle's formula against itself: each compares it with
something the mathematics fixes (a closed form, a dense numpy evaluation over
contiguous unpaged tensors, an invariant of the split-range design, numpy's own
half-precision decoder, numpy fancy indexing for the layouts, a list model of
the allocator).  CPU only.
"""
import itertools
import os

import numpy as np
import pytest

import mc_inputs as mi
import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def shape_of(L=1, pages=8, P=16, Hkv=2, D=128, dtype=oracle.F16):
    return oracle.Shape(L, pages, P, Hkv, D, dtype)


def build_pool(shape, layer, k_bits, v_bits, pages):
    pool = oracle.new_pool(shape)
    oracle.append(pool, shape, layer, k_bits, v_bits, 0, pages)
    return pool


def dense_attention(q, k, v, begin, G, scale):
    """Textbook dense evaluation on contiguous fp64 tensors with an explicit -inf mask.
    q [q_len][Hq][D], k/v [n][Hkv][D].  Independent of the oracle's row-wise paged path."""
    q_len, Hq, D = q.shape
    n = k.shape[0]
    kk = np.repeat(k, G, axis=1)  # [n][Hq][D]
    vv = np.repeat(v, G, axis=1)
    s = scale * np.einsum("ihd,jhd->hij", q, kk)
    i = begin + np.arange(q_len)[:, None]
    j = np.arange(n)[None, :]
    s = np.where((j <= i)[None], s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=-1, keepdims=True)
    o = np.einsum("hij,jhd->ihd", e / z, vv)
    lse = (m + np.log(z))[..., 0].T  # [q_len][Hq]
    return o, lse


# ---------------------------------------------------------------- decode ----
def test_decode_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.decode(bits, oracle.F16)
    ref = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok], ref[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))
    got = oracle.decode(bits, oracle.BF16)
    ref = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok], ref[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))


# ---------------------------------------------------------------- golden ----
def test_golden_two_key_softmax():
    vals = {}
    for line in open(os.path.join(GOLDEN, "softmax_two_keys.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        vals[key] = [float(x) for x in rest]
    shape = oracle.Shape(1, 3, 2, 1, 4, oracle.F16)
    f = lambda *x: np.array(x, dtype=np.float16).view(np.uint16)
    k = np.stack([f(0, 0, 0, 0), f(vals["s"][0], 0, 0, 0)]).reshape(2, 1, 4)
    v = np.stack([f(3, 0, -6, 1), f(0, 3, 6, 1)]).reshape(2, 1, 4)
    pool = build_pool(shape, 0, k, v, [2])
    q = f(1, 0, 0, 0).reshape(1, 1, 4)
    o, lse = oracle.attention(pool, shape, 0, [2], q, 1, 1, 2, scale=1.0)
    assert abs(lse[0, 0] - vals["lse"][0]) < 1e-14
    assert np.allclose(o[0, 0], vals["o"], rtol=0, atol=1e-14)
    # range [0,1): the first token sees only itself
    o0, lse0 = oracle.attention(pool, shape, 0, [2], f(1, 0, 0, 0).reshape(1, 1, 4), 1, 0, 1,
                                scale=1.0)
    assert lse0[0, 0] == 0.0 and np.array_equal(o0[0, 0], [3, 0, -6, 1])


# ----------------------------------------------------------- closed forms ----
@pytest.mark.parametrize("dtype", [oracle.F16, oracle.BF16])
def test_equal_keys_give_running_mean_and_log_count(dtype):
    rng = mi.rng_for(11, dtype)
    n, b, Hq, Hkv, D = 45, 13, 4, 2, 128
    shape = shape_of(pages=8, Hkv=Hkv, dtype=dtype)
    krow = mi.normal_bits(rng, (1, Hkv, D), dtype)
    k = np.repeat(krow, n, axis=0)
    v = mi.normal_bits(rng, (n, Hkv, D), dtype)
    pages = [5, 0, 7]
    pool = build_pool(shape, 0, k, v, pages)
    q = mi.normal_bits(rng, (n - b, Hq, D), dtype)
    o, lse = oracle.attention(pool, shape, 0, pages, q, Hq, b, n)
    vd, kd, qd = oracle.decode(v, dtype), oracle.decode(krow, dtype), oracle.decode(q, dtype)
    scale = 1 / np.sqrt(D)
    for r in range(n - b):
        i = b + r
        for h in range(Hq):
            mean = vd[: i + 1, h // 2].mean(axis=0)
            s = scale * float(qd[r, h] @ kd[0, h // 2])
            assert np.allclose(o[r, h], mean, rtol=0, atol=1e-12)
            assert abs(lse[r, h] - (s + np.log(i + 1))) < 1e-12


def test_single_token_returns_its_value_and_score():
    rng = mi.rng_for(12)
    shape = shape_of(pages=4, Hkv=2, dtype=oracle.BF16)
    k = mi.normal_bits(rng, (1, 2, 128), mi.BF16)
    v = mi.normal_bits(rng, (1, 2, 128), mi.BF16)
    q = mi.normal_bits(rng, (1, 6, 128), mi.BF16)
    pool = build_pool(shape, 0, k, v, [3])
    o, lse = oracle.attention(pool, shape, 0, [3], q, 6, 0, 1, scale=0.25)
    kd, vd, qd = (oracle.decode(x, mi.BF16) for x in (k, v, q))
    for h in range(6):
        assert np.array_equal(o[0, h], vd[0, h // 3])
        assert abs(lse[0, h] - 0.25 * float(qd[0, h] @ kd[0, h // 3])) < 1e-13


def test_dominant_key_selects_its_value():
    rng = mi.rng_for(13)
    n, D = 40, 128
    shape = shape_of(pages=4, Hkv=1)
    k = np.zeros((n, 1, D), dtype=np.float16)
    k[17, 0, 0] = 60.0  # score 60 against q = e0 with scale 1; every other score is 0
    v = mi.normal_bits(rng, (n, 1, D), mi.F16)
    q = np.zeros((1, 1, D), dtype=np.float16)
    q[0, 0, 0] = 1.0
    pool = build_pool(shape, 0, k.view(np.uint16), v, [1, 2, 3])
    o, lse = oracle.attention(pool, shape, 0, [1, 2, 3], q.view(np.uint16), 1, n - 1, n, scale=1.0)
    assert np.allclose(o[0, 0], oracle.decode(v, mi.F16)[17, 0], rtol=0, atol=1e-20)
    assert abs(lse[0, 0] - 60.0) < 1e-12
    # the same key hidden behind the causal mask (query at position 16 < 17) has no effect
    o2, lse2 = oracle.attention(pool, shape, 0, [1, 2, 3], q.view(np.uint16), 1, 16, 17, scale=1.0)
    assert abs(lse2[0, 0] - np.log(17)) < 1e-12
    assert np.allclose(o2[0, 0], oracle.decode(v, mi.F16)[:17, 0].mean(axis=0), atol=1e-13)


def test_softmax_rows_sum_to_one():
    """V == 1 everywhere makes every output element the row sum of the probabilities."""
    rng = mi.rng_for(14)
    n, b, Hq, Hkv, D = 70, 21, 4, 4, 128
    shape = shape_of(pages=8, Hkv=Hkv, dtype=oracle.BF16)
    k = mi.normal_bits(rng, (n, Hkv, D), mi.BF16)
    v = mi.f32_to_bits(np.ones((n, Hkv, D), dtype=np.float32), mi.BF16)
    pages = [6, 1, 4, 2, 7]
    pool = build_pool(shape, 0, k, v, pages)
    q = mi.f32_to_bits(3 * rng.standard_normal((n - b, Hq, D), dtype=np.float32), mi.BF16)
    o, _ = oracle.attention(pool, shape, 0, pages, q, Hq, b, n)
    assert np.max(np.abs(o - 1.0)) < 1e-12


# ------------------------------------------------------------ brute force ----
@pytest.mark.parametrize("dtype,n,b,Hq,Hkv,P,D", [
    (oracle.F16, 64, 0, 4, 4, 16, 128),
    (oracle.BF16, 61, 23, 8, 2, 16, 128),
    (oracle.BF16, 33, 32, 4, 1, 16, 128),   # one new token (the "prefill the last token" case)
    (oracle.F16, 50, 7, 6, 3, 4, 32),       # other page size / head dim: layout arithmetic
])
def test_paged_rows_match_dense_contiguous_evaluation(dtype, n, b, Hq, Hkv, P, D):
    rng = mi.rng_for(20, dtype, n, b)
    n_pages = -(-n // P)
    shape = oracle.Shape(2, n_pages + 5, P, Hkv, D, dtype)
    pages = rng.permutation(n_pages + 5)[:n_pages].astype(np.int32)
    k = mi.normal_bits(rng, (n, Hkv, D), dtype)
    v = mi.normal_bits(rng, (n, Hkv, D), dtype)
    q = mi.normal_bits(rng, (n - b, Hq, D), dtype)
    pool = build_pool(shape, 1, k, v, pages)  # layer 1; layer 0 stays zero
    o, lse = oracle.attention(pool, shape, 1, pages, q, Hq, b, n)
    scale = 1 / np.sqrt(D)
    ro, rl = dense_attention(oracle.decode(q, dtype), oracle.decode(k, dtype),
                             oracle.decode(v, dtype), b, Hq // Hkv, scale)
    assert np.max(np.abs(o - ro)) < 1e-12
    assert np.max(np.abs(lse - rl)) < 1e-12
    # sampled interface returns the same numbers as the full one
    rows = np.array([0, (n - b) - 1, (n - b) // 2], dtype=np.int32)
    heads = np.array([Hq - 1, 0, 1], dtype=np.int32)
    so, sl = oracle.attention(pool, shape, 1, pages, q, Hq, b, n, sel_rows=rows, sel_heads=heads)
    assert np.array_equal(so, o[rows, heads]) and np.array_equal(sl, lse[rows, heads])


# -------------------------------------------------------------- invariants ----
def _seq(rng, n, Hq, Hkv, dtype, D=128, extra_pages=9, P=16):
    n_pages = -(-n // P)
    shape = oracle.Shape(1, n_pages + extra_pages, P, Hkv, D, dtype)
    pages = rng.permutation(n_pages + extra_pages)[:n_pages].astype(np.int32)
    k = mi.normal_bits(rng, (n, Hkv, D), dtype)
    v = mi.normal_bits(rng, (n, Hkv, D), dtype)
    q = mi.normal_bits(rng, (n, Hq, D), dtype)
    return shape, pages, k, v, q


def test_split_range_equals_single_pass():
    """attn([0,n)) rows == attn([0,m)) rows followed by attn([m,n)) over the cached [0,m)
    (Sec. 3.3: the decode engine continues with prompt[s:] after receiving KV of prompt[:s])."""
    rng = mi.rng_for(30)
    n, m, Hq, Hkv = 77, 29, 4, 2
    shape, pages, k, v, q = _seq(rng, n, Hq, Hkv, oracle.BF16)
    pool = build_pool(shape, 0, k, v, pages)
    o, lse = oracle.attention(pool, shape, 0, pages, q, Hq, 0, n)
    # pass A on a pool that holds only [0,m): nothing after m may be needed
    pool_a = build_pool(shape, 0, k[:m], v[:m], pages)
    oa, la = oracle.attention(pool_a, shape, 0, pages, q[:m], Hq, 0, m)
    # pass B: append [m,n) to the same pool, then attend the new range
    oracle.append(pool_a, shape, 0, k[m:], v[m:], m, pages)
    assert np.array_equal(pool_a, pool)
    ob, lb = oracle.attention(pool_a, shape, 0, pages, q[m:], Hq, m, n)
    assert np.array_equal(np.concatenate([oa, ob]), o)
    assert np.array_equal(np.concatenate([la, lb]), lse)


def test_kv_split_merged_by_lse_equals_single_pass():
    """Row i over keys [0,m) and over keys [m,i], merged by LSE, equals row i over [0,i]."""
    rng = mi.rng_for(31)
    n, m, Hq, Hkv, D = 59, 21, 2, 1, 128
    shape, pages, k, v, q = _seq(rng, n, Hq, Hkv, oracle.F16)
    pool = build_pool(shape, 0, k, v, pages)
    for i in (m, 40, n - 1):
        qi = q[i:i + 1]
        o, lse = oracle.attention(pool, shape, 0, pages, qi, Hq, i, i + 1)
        # keys [0,m): the same query placed at position m-1 of a cache holding [0,m)
        o1, l1 = oracle.attention(pool, shape, 0, pages, qi, Hq, m - 1, m)
        # keys [m,i]: a second sequence holding only those tokens, query at its last position
        cnt = i - m + 1
        pool2 = build_pool(shape, 0, k[m:i + 1], v[m:i + 1], pages)
        o2, l2 = oracle.attention(pool2, shape, 0, pages, qi, Hq, cnt - 1, cnt)
        om, lm = oracle.lse_merge(o1.reshape(-1, D), l1.ravel(), o2.reshape(-1, D), l2.ravel())
        assert np.max(np.abs(om - o.reshape(-1, D))) < 1e-12
        assert np.max(np.abs(lm - lse.ravel())) < 1e-12


def test_lse_merge_against_direct_formula_on_scalars():
    # two "partials" made of one key each: merging must give the two-key softmax
    o1, o2 = np.array([[2.0, -1.0]]), np.array([[0.5, 4.0]])
    l1, l2 = np.array([0.3]), np.array([-1.1])
    o, l = oracle.lse_merge(o1, l1, o2, l2)
    w = np.exp([0.3, -1.1])
    assert abs(l[0] - np.log(w.sum())) < 1e-14
    assert np.allclose(o[0], (w[0] * o1[0] + w[1] * o2[0]) / w.sum(), atol=1e-14)
    # merging with an empty partial (LSE = -inf) is the identity
    o, l = oracle.lse_merge(o1, l1, np.zeros((1, 2)), np.array([-np.inf]))
    assert np.array_equal(o, o1) and l[0] == l1[0]


def test_result_does_not_depend_on_physical_pages():
    rng = mi.rng_for(32)
    n, b, Hq, Hkv = 90, 37, 4, 2
    shape, pages, k, v, q = _seq(rng, n, Hq, Hkv, oracle.BF16)
    pool = build_pool(shape, 0, k, v, pages)
    o, lse = oracle.attention(pool, shape, 0, pages, q[b:], Hq, b, n)
    pages2 = rng.permutation(shape.num_pages)[: len(pages)].astype(np.int32)
    assert not np.array_equal(pages, pages2)
    pool2 = build_pool(shape, 0, k, v, pages2)
    o2, lse2 = oracle.attention(pool2, shape, 0, pages2, q[b:], Hq, b, n)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)


def test_heads_of_one_group_share_kv():
    rng = mi.rng_for(33)
    n, b, Hq, Hkv = 48, 16, 8, 2
    shape, pages, k, v, q = _seq(rng, n, Hq, Hkv, oracle.BF16)
    q[:, 1] = q[:, 3]      # same group (heads 0-3 -> kv head 0)
    q[:, 5] = q[:, 3]      # other group (heads 4-7 -> kv head 1)
    pool = build_pool(shape, 0, k, v, pages)
    o, lse = oracle.attention(pool, shape, 0, pages, q[b:], Hq, b, n)
    assert np.array_equal(o[:, 1], o[:, 3]) and np.array_equal(lse[:, 1], lse[:, 3])
    assert not np.allclose(o[:, 5], o[:, 3])


def test_causal_mask_future_tokens_do_not_matter():
    rng = mi.rng_for(34)
    n, b, Hq, Hkv = 50, 20, 2, 2
    shape, pages, k, v, q = _seq(rng, n, Hq, Hkv, oracle.F16)
    pool = build_pool(shape, 0, k, v, pages)
    o, lse = oracle.attention(pool, shape, 0, pages, q[b:], Hq, b, n)
    k2, v2 = k.copy(), v.copy()
    k2[41:] = mi.normal_bits(rng, k2[41:].shape, mi.F16)
    v2[41:] = mi.normal_bits(rng, v2[41:].shape, mi.F16)
    pool2 = build_pool(shape, 0, k2, v2, pages)
    o2, lse2 = oracle.attention(pool2, shape, 0, pages, q[b:], Hq, b, n)
    assert np.array_equal(o[: 41 - b], o2[: 41 - b]) and np.array_equal(lse[: 41 - b], lse2[: 41 - b])
    assert not np.allclose(o[41 - b:], o2[41 - b:])


# ------------------------------------------------------------------ copies ----
def test_append_places_rows_where_numpy_indexing_says():
    rng = mi.rng_for(40)
    L, NP, P, Hkv, D = 3, 11, 16, 4, 128
    shape = oracle.Shape(L, NP, P, Hkv, D, oracle.BF16)
    pool = rng.integers(0, 65536, size=shape.pool_elems(), dtype=np.uint16)  # canary bytes
    before = pool.copy()
    pages = np.array([9, 2, 5, 0], dtype=np.int32)
    b, n = 13, 55
    k = mi.normal_bits(rng, (n - b, Hkv, D), mi.BF16)
    v = mi.normal_bits(rng, (n - b, Hkv, D), mi.BF16)
    oracle.append(pool, shape, 2, k, v, b, pages)
    view = pool.reshape(shape.pool_dims())
    ref = before.reshape(shape.pool_dims()).copy()
    pos = np.arange(b, n)
    ref[2, pages[pos // P], 0, :, pos % P, :] = k
    ref[2, pages[pos // P], 1, :, pos % P, :] = v
    assert np.array_equal(view, ref)


@pytest.mark.parametrize("s0,s1", [(0, 55), (13, 40), (16, 48), (7, 8), (20, 20)])
def test_pack_layout_and_unpack_identity(s0, s1):
    rng = mi.rng_for(41, s0, s1)
    L, NP, P, Hkv, D = 4, 9, 16, 2, 128
    shape = oracle.Shape(L, NP, P, Hkv, D, oracle.F16)
    pool = mi.normal_bits(rng, shape.pool_elems(), mi.F16)   # finite, so it can be attended
    pages = np.array([7, 3, 8, 1], dtype=np.int32)
    buf = oracle.pack(pool, shape, 1, 4, pages, s0, s1)
    pos = np.arange(s0, s1)
    view = pool.reshape(shape.pool_dims())
    # [layer][kv][token][head][d] by fancy indexing
    ref = np.stack([np.stack([view[l, pages[pos // P], kv, :, pos % P, :].reshape(-1, Hkv, D)
                              for kv in range(2)]) for l in range(1, 4)])
    assert buf.shape == ref.shape and np.array_equal(buf, ref)
    # unpack into another pool with another table: addressed slots equal, the rest untouched
    pool_b = rng.integers(0, 65536, size=shape.pool_elems(), dtype=np.uint16)
    before = pool_b.copy()
    pages_b = np.array([0, 4, 2, 6], dtype=np.int32)
    oracle.unpack(pool_b, shape, 1, 4, pages_b, s0, s1, buf)
    vb = pool_b.reshape(shape.pool_dims())
    expect = before.reshape(shape.pool_dims()).copy()
    for li, l in enumerate(range(1, 4)):
        for kv in range(2):
            expect[l, pages_b[pos // P], kv, :, pos % P, :] = buf[li, kv]
    assert np.array_equal(vb, expect)
    # and packing pool_b again returns the very same bytes
    assert np.array_equal(oracle.pack(pool_b, shape, 1, 4, pages_b, s0, s1), buf)
    # attention over the received pages equals attention over the source pages
    if s0 == 0 and s1 == 55:
        q = mi.normal_bits(rng, (1, 4, D), mi.F16)
        o1, l1 = oracle.attention(pool, shape, 2, pages, q, 4, s1 - 1, s1)
        o2, l2 = oracle.attention(pool_b, shape, 2, pages_b, q, 4, s1 - 1, s1)
        assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


# --------------------------------------------------------------- allocator ----
class ListModel:
    def __init__(self, n):
        self.free = list(range(n - 1, -1, -1))
        self.used = set()
        self.n = n

    def take(self, k):
        if k > len(self.free):
            return None
        out = [self.free.pop() for _ in range(k)]
        self.used.update(out)
        return out

    def give(self, pages):
        if len(set(pages)) != len(pages) or any(p not in self.used for p in pages):
            return False
        for p in pages:
            self.used.discard(p)
            self.free.append(p)
        return True


def test_allocator_first_pages_and_exhaustion():
    a = oracle.Allocator(4)
    assert a.take(3) == [0, 1, 2]
    assert a.take(2) is None and a.num_free == 1      # all-or-nothing
    assert a.take(1) == [3]
    assert a.give([1, 3]) and a.take(2) == [3, 1]     # last freed comes back first
    assert not a.give([0, 0]) and not a.give([2, 2])
    assert not a.give([7]) and not a.give([-1])
    assert a.take(0) == []


def test_allocator_exhaustive_on_four_pages():
    """Every sequence of up to 5 operations on a 4-page pool against a Python list model."""
    ops = [("take", k) for k in range(0, 5)] + [("give_first", k) for k in (1, 2)] + \
          [("give_last", 1), ("give_dup", 0), ("give_free", 0)]
    for seq in itertools.product(ops, repeat=4):
        a, m = oracle.Allocator(4), ListModel(4)
        held = []
        for op, k in seq:
            if op == "take":
                got, ref = a.take(k), m.take(k)
                assert got == ref
                if got:
                    held += got
            else:
                if op == "give_first":
                    pages = held[:k]
                elif op == "give_last":
                    pages = held[-1:]
                elif op == "give_dup":
                    pages = held[:1] * 2
                else:
                    pages = [p for p in range(4) if p not in held][:1]
                if not pages:
                    continue
                ok, ref = a.give(pages), m.give(pages)
                assert ok == ref
                if ok:
                    held = [p for p in held if p not in pages]
            assert a.num_free == len(m.free)
        a.close()


# ---------------------------------------------------------- input generator ----
def test_bf16_rounding_of_generator_is_nearest_even():
    import torch
    x = mi.rng_for(50).standard_normal(size=20000, dtype=np.float32)
    x[:4] = [1.00390625, 1.01171875, 0.0, -2.5]   # two exact ties: round to even mantissa
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mi.f32_to_bits(x, mi.BF16), ref)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_config_shapes(idx):
    w = mi.config(idx)
    assert w.head_dim == 128 and w.page_size == 16
    assert np.all(w.b <= w.n) and np.all(w.b >= 0)
    flat = w.flat_page_table
    assert len(np.unique(flat)) == len(flat) and flat.max() < w.num_pages
    for t, n in zip(w.page_tables, w.n):
        assert len(t) == -(-int(n) // 16)
    if idx == 1:
        assert (w.dtype, w.num_q_heads, w.num_kv_heads, int(w.n[0]), int(w.b[0])) == (0, 8, 8, 512, 256)
        assert w.useful_flops() == 4 * 128 * 8 * (256 * 256 + 256 * 257 // 2)
    if idx == 2:
        assert w.batch == 8 and w.num_pages == 65536 and w.n.min() >= 1024 and w.n.max() <= 4096
        assert np.all(w.b <= 0.75 * w.n)
    if idx == 4:
        assert int(w.b[0]) == 7372 and w.num_q_heads == 64
    if idx == 5:
        assert list(w.n) == [16384, 32768] and w.num_layers == 32


# ---- host arithmetic of remote_send (Sec. 3.5) ----
def test_send_plan_case1_sender_matched_more():
    # sender cached 300 tokens, receiver 100, request [0, 500): 100..299 exist only on the
    # sender and go as they are; 300..499 exist nowhere: computed, then sent
    p = oracle.send_plan(300, 100, 0, 500)
    assert p["copy"] == list(range(100, 300))
    assert p["prefill"] == list(range(300, 500))
    assert p["send"] == list(range(300, 500))


def test_send_plan_case2_receiver_matched_more():
    # sender cached 100, receiver 300: nothing can be copied; the sender computes everything it
    # lacks (100..499) and sends only what the receiver lacks (300..499)
    p = oracle.send_plan(100, 300, 0, 500)
    assert p["copy"] == []
    assert p["prefill"] == list(range(100, 500))
    assert p["send"] == list(range(300, 500))


def test_send_plan_degenerate_cases():
    assert oracle.send_plan(500, 0, 0, 500) == {"copy": list(range(500)), "prefill": [], "send": []}
    assert oracle.send_plan(0, 500, 0, 500) == {"copy": [], "prefill": [], "send": []}
    assert oracle.send_plan(0, 0, 0, 0) == {"copy": [], "prefill": [], "send": []}
    # a request that starts above what the receiver has: the gap below begin is not sent
    p = oracle.send_plan(50, 10, 40, 60)
    assert p["copy"] == list(range(40, 50)) and p["send"] == list(range(50, 60))
    # everything the receiver gets is exactly what it lacked in [begin, end), once
    for s, r, b, e in [(7, 3, 2, 11), (3, 7, 0, 11), (5, 5, 5, 9), (20, 1, 4, 9)]:
        p = oracle.send_plan(s, r, b, e)
        assert sorted(p["copy"] + p["send"]) == [t for t in range(b, e) if t >= r]


def test_addr_runs():
    assert oracle.addr_runs([]) == []
    assert oracle.addr_runs([5, 6, 7, 9, 10, 3, 4, 4]) == [(5, 3), (9, 2), (3, 2), (4, 1)]
    assert oracle.addr_runs([2, 1, 0]) == [(2, 1), (1, 1), (0, 1)]


# ---- context cache index behind prep_recv (Sec. 3.1) ----
def test_prefix_index_hand_cases():
    ix = oracle.PrefixIndex()
    a = list(range(100, 150))                  # 50 tokens: 3 whole pages
    ix.insert(a, [7, 8, 9])
    assert ix.match(a) == (48, [7, 8, 9])
    assert ix.match(a[:47]) == (32, [7, 8])    # the third page is not whole in the query
    b = a[:32] + [999] + a[33:]                # differs in the third page
    assert ix.match(b) == (32, [7, 8])
    c = [5] + a[1:]                            # differs in the first token: nothing in common
    assert ix.match(c) == (0, [])
    # same block tokens under another prefix are another block
    d = [1] * 16 + a[16:32]
    ix.insert(d, [20, 21])
    assert ix.match(d) == (32, [20, 21]) and ix.match(a[:32]) == (32, [7, 8])
    # a block recorded earlier keeps its page
    ix.insert(a, [70, 80, 90])
    assert ix.match(a) == (48, [7, 8, 9])


def test_prep_recv_oracle_allocates_only_the_unmatched_part():
    ix, al = oracle.PrefixIndex(), oracle.Allocator(16)
    prompt = list(range(200))
    pages, m = oracle.prep_recv(ix, al, prompt, 100)      # nothing cached: 7 fresh pages
    assert m == 0 and pages == [0, 1, 2, 3, 4, 5, 6] and al.num_free == 9
    ix.insert(prompt[:100], pages)                         # 6 whole pages recorded
    pages2, m2 = oracle.prep_recv(ix, al, prompt, 200)    # 96 tokens matched, 13 - 6 fresh
    assert m2 == 96 and pages2[:6] == pages[:6] and pages2[6:] == [7, 8, 9, 10, 11, 12, 13]
    assert oracle.prep_recv(ix, al, [9] * 64, 64) is None and al.num_free == 2   # all or nothing


# ---- fork_sequence (Sec. 3.5) ----
def test_fork_sequence_oracle_hand_cases():
    al = oracle.Allocator(10)
    parent = al.take(7)                                  # pages 0..6 hold 100 tokens
    child, copy = oracle.fork_sequence(al, parent, 100)  # 6 whole pages, 4 slots in the seventh
    assert child == [0, 1, 2, 3, 4, 5, 7] and copy == (6, 7, 4)
    assert oracle.fork_sequence(al, parent, 96) == ([0, 1, 2, 3, 4, 5], (-1, -1, 0))
    assert oracle.fork_sequence(al, parent, 0) == ([], (-1, -1, 0))
    assert al.num_free == 2


def test_copy_page_oracle_moves_exactly_the_slots():
    shape = oracle.Shape(2, 4, 16, 3, 128, oracle.BF16)
    rng = np.random.default_rng(0)
    pool = rng.integers(0, 65536, size=shape.pool_elems(), dtype=np.uint16)
    before = pool.copy()
    oracle.copy_page(pool, shape, 0, 2, 1, 3, 5)
    v, b = pool.reshape(shape.pool_dims()), before.reshape(shape.pool_dims())
    for layer in range(2):
        for page in range(4):
            for kv in range(2):
                for head in range(3):
                    for slot in range(16):
                        src = (1 if (page == 3 and slot < 5) else page)
                        assert np.array_equal(v[layer, page, kv, head, slot], b[layer, src, kv, head, slot])
