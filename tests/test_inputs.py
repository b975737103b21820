"""CPU checks of the seeded input generators (mc_inputs.py): the shapes of the five workload
configurations, the flop count, forked sequences."""
import numpy as np

import mc_inputs as mi


def test_config_shapes():
    w = mi.config(1)
    assert (w.dtype, w.num_q_heads, w.num_kv_heads, w.num_pages) == (mi.F16, 8, 8, 64)
    assert list(w.n) == [512] and list(w.b) == [256] and sorted(w.page_tables[0]) == sorted(set(w.page_tables[0]))
    w = mi.config(2)
    assert (w.dtype, w.num_q_heads, w.num_kv_heads, w.num_pages, w.batch) == (mi.BF16, 32, 8, 65536, 8)
    assert np.all((w.n >= 1024) & (w.n <= 4096)) and np.all(w.b <= 0.75 * w.n) and np.all(w.b >= 0)
    flat = w.flat_page_table
    assert len(set(flat.tolist())) == len(flat) and flat.min() >= 0 and flat.max() < 65536
    assert [len(t) for t in w.page_tables] == [-(-int(x) // 16) for x in w.n]
    w = mi.config(4)
    assert (w.num_q_heads, w.num_kv_heads, w.batch) == (64, 8, 4)
    assert list(w.n) == [8192] * 4 and list(w.b) == [7372] * 4 and 7372 % 16 == 12
    w = mi.config(5, num_layers=1)
    assert list(w.n) == [16384, 32768] and list(w.b) == [8192, 16384]
    for cached in (500, 2500, 4500):
        w = mi.paper_point(cached)
        assert list(w.b) == [cached] and list(w.n - w.b) == [500]


def test_same_seed_same_data_and_prefix_of_longer_sequence():
    a, b = mi.config(2, seed=7), mi.config(2, seed=7)
    assert np.array_equal(a.n, b.n) and np.array_equal(a.kv(3)[0], b.kv(3)[0])
    short = a.with_ranges(np.zeros_like(a.b), a.b)           # the cached prefixes only
    k_full, _ = a.kv(0)
    k_short, _ = short.kv(0)
    assert np.array_equal(k_short, k_full[: short.n[0]])     # a prefix keeps its values


def test_useful_flops_is_the_count_of_visible_pairs():
    w = mi.Workload("t", 1, mi.BF16, 1, 4, 2, 64, np.array([37, 5, 9]), np.array([20, 0, 9]))
    pairs = 0
    for n, b in zip(w.n, w.b):
        for i in range(int(b), int(n)):
            pairs += i + 1                                    # keys 0..i
    assert w.useful_flops() == 4 * 128 * 4 * pairs


def test_layer_variant_permutes_tokens_and_flips_signs():
    x = mi.normal_bits(mi.rng_for(3), (50, 2, 128), mi.BF16)
    assert np.array_equal(mi.layer_variant(x, 0), x)
    y = mi.layer_variant(x, 1)
    assert y.shape == x.shape and not np.array_equal(x, y)
    assert np.array_equal(np.sort((y ^ np.uint16(0x8000)).reshape(-1)), np.sort(x.reshape(-1)))


def test_share_prefix_makes_a_fork():
    n = np.array([300, 260, 100])
    w = mi.Workload("f", 5, mi.F16, 1, 8, 2, 64, n, n - 1)
    w.page_tables = mi.scatter_page_tables(mi.rng_for(5, mi.KIND_TABLE), 64, n)
    own = w.page_tables[1].copy()
    w.share_prefix(1, 0, 160)
    k0, v0 = w.kv(0)
    k1, v1 = w.kv(1)
    assert np.array_equal(k1[:160], k0[:160]) and np.array_equal(v1[:160], v0[:160])
    assert not np.array_equal(k1[160:], k0[160:260])
    assert np.array_equal(w.page_tables[1][:10], w.page_tables[0][:10])
    assert np.array_equal(w.page_tables[1][10:], own[10:])
    assert np.array_equal(w.with_ranges(w.b, w.n).kv(1)[0], k1)      # forks survive a change of ranges


def test_sample_rows_covers_the_whole_range():
    q_len, begin, tile = 8192 + 13, 8192 + 5, 32
    rows, heads = mi.sample_rows(mi.rng_for(9), q_len, begin, 32, 4096, tile, num_kv_heads=8)
    assert rows.size == heads.size >= 4096 and rows.min() == 0 and rows.max() == q_len - 1
    # every row comes with one head of each kv head's group
    assert np.array_equal(np.unique(heads.reshape(-1, 8) // 4, axis=0), np.arange(8)[None, :])
    pos = begin + np.unique(rows)
    thirds = [pos[(pos >= begin + k * q_len // 3) & (pos < begin + (k + 1) * q_len // 3)] for k in range(3)]
    for part in thirds:                      # start, middle and end of the range alike
        assert np.sum(part % 16 == 0) >= 8 and np.sum(part % 16 == 15) >= 8       # page boundaries
        r = part - begin
        assert np.sum(r % tile == 0) >= 8 and np.sum(r % tile == tile - 1) >= 8   # q tile edges
    last0 = (q_len - 1) // tile * tile       # the ragged last tile: its first, its last, more
    assert last0 in rows and np.sum(np.unique(rows) >= last0) >= 3
    # one head per row without kv groups; short ranges are taken whole at most
    rows, heads = mi.sample_rows(mi.rng_for(9), 5, 3, 8, 64)
    assert rows.size == heads.size and set(rows.tolist()) <= set(range(5)) and {0, 4} <= set(rows.tolist())
