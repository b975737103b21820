"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, its host allocator agrees with the oracle's, and argument validation
rejects bad calls before anything would be launched (no compute call is made here)."""
import os
import re

import numpy as np
import pytest

import mc_inputs as mi
import oracle
import paper_2412_12488_amd as mc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a non-null, 16-byte aligned "device address" that is never dereferenced


def header_symbols():
    text = open(os.path.join(ROOT, "include", "mc_kv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_symbols()
    assert "mc_prefix_prefill_attn" in names and "mc_kv_pack_range" in names
    L = mc.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(mc.EXPORTS) == names
    assert mc.mc_abi_version() == 2
    assert mc.status_string(0) == "MC_OK" and mc.status_string(3) == "MC_ERR_RANGE"


def test_allocator_matches_oracle_on_random_traffic():
    rng = mi.rng_for(60)
    for num_pages in (0, 1, 4, 64, 1000):
        a = mc.mc_kv_allocator_create(num_pages)
        o = oracle.Allocator(num_pages)
        held = []
        for _ in range(300):
            if rng.random() < 0.55 or not held:
                n = int(rng.integers(0, max(2, num_pages // 3 + 2)))
                ref = o.take(n)
                if ref is None:
                    with pytest.raises(mc.McError) as e:
                        mc.mc_kv_alloc_pages(a, n)
                    assert e.value.status == mc.MC_ERR_NO_PAGES
                else:
                    assert mc.mc_kv_alloc_pages(a, n) == ref
                    held += ref
            else:
                k = int(rng.integers(1, len(held) + 1))
                idx = rng.permutation(len(held))[:k]
                pages = [held[i] for i in idx]
                assert o.give(pages)
                mc.mc_kv_free_pages(a, pages)
                held = [p for i, p in enumerate(held) if i not in set(idx.tolist())]
            assert mc.mc_kv_allocator_num_free(a) == o.num_free
        # double free / foreign page / duplicate are rejected and change nothing
        free_before = mc.mc_kv_allocator_num_free(a)
        for bad in ([num_pages], [-1], held[:1] * 2 if held else [0, 0]):
            with pytest.raises(mc.McError) as e:
                mc.mc_kv_free_pages(a, bad)
            assert e.value.status == mc.MC_ERR_INVALID
            assert not o.give(bad)
        assert mc.mc_kv_allocator_num_free(a) == free_before
        mc.mc_kv_allocator_destroy(a)


def test_first_allocations_are_0_1_2_and_lifo():
    a = mc.mc_kv_allocator_create(8)
    assert mc.mc_kv_alloc_pages(a, 3) == [0, 1, 2]
    mc.mc_kv_free_pages(a, [1, 0])
    assert mc.mc_kv_alloc_pages(a, 3) == [0, 1, 3]
    with pytest.raises(mc.McError):
        mc.mc_kv_alloc_pages(a, 5)
    assert mc.mc_kv_allocator_num_free(a) == 4
    mc.mc_kv_allocator_destroy(a)


def test_check_page_table():
    assert mc.mc_kv_check_page_table([3, 1, 2], 4) == mc.MC_OK
    assert mc.mc_kv_check_page_table([3, 1, 3], 4) == mc.MC_ERR_ALIAS
    assert mc.mc_kv_check_page_table([4], 4) == mc.MC_ERR_RANGE
    assert mc.mc_kv_check_page_table([-1], 4) == mc.MC_ERR_RANGE
    assert mc.mc_kv_check_page_table([], 4) == mc.MC_OK


def _pool(**kw):
    d = dict(base=FAKE, num_layers=2, num_pages=8, num_kv_heads=8, dtype=mc.MC_BF16)
    d.update(kw)
    return mc.pool_desc(d.pop("base"), d.pop("num_layers"), d.pop("num_pages"),
                        d.pop("num_kv_heads"), d.pop("dtype"), **d)


def test_copy_check_needs_a_counter():
    # without a counter, or with a misaligned one, nothing is read from the device
    L = mc.lib()
    import ctypes as C
    assert L.mc_kv_copy_check(None, None, None) == mc.MC_ERR_INVALID
    assert L.mc_kv_copy_check(C.byref(_pool()), None, None) == mc.MC_ERR_INVALID
    assert L.mc_kv_copy_check(C.byref(_pool(skipped=FAKE + 2)), None, None) == mc.MC_ERR_INVALID
    # a misaligned counter is refused by every call that takes the pool
    assert _status(mc.mc_kv_pack_range, _pool(skipped=FAKE + 2), 0, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_INVALID


def _status(fn, *args):
    try:
        fn(*args, stream=0)
    except mc.McError as e:
        return e.status
    return mc.MC_OK


def test_validation_rejects_before_launch():
    ok = _pool()
    pk = mc.mc_kv_pack_range
    assert _status(pk, _pool(head_dim=64), 0, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_UNSUPPORTED
    assert _status(pk, _pool(page_size=32), 0, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_UNSUPPORTED
    assert _status(pk, _pool(dtype=7), 0, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_UNSUPPORTED
    assert _status(pk, _pool(base=0), 0, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_INVALID
    assert _status(pk, _pool(base=FAKE + 2), 0, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_INVALID
    assert _status(pk, ok, 0, 3, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_RANGE      # layer_end > L
    assert _status(pk, ok, 1, 0, FAKE, 4, 0, 16, FAKE) == mc.MC_ERR_RANGE      # reversed layers
    assert _status(pk, ok, 0, 1, FAKE, 4, 9, 8, FAKE) == mc.MC_ERR_RANGE       # s0 > s1
    assert _status(pk, ok, 0, 1, FAKE, 4, 0, 65, FAKE) == mc.MC_ERR_RANGE      # table too short
    assert _status(pk, ok, 0, 1, None, 4, 0, 16, FAKE) == mc.MC_ERR_INVALID
    assert _status(pk, ok, 0, 1, FAKE, 4, 0, 16, FAKE + 8) == mc.MC_ERR_INVALID
    # empty ranges are fine and launch nothing
    assert _status(pk, ok, 0, 1, FAKE, 4, 5, 5, FAKE) == mc.MC_OK
    assert _status(mc.mc_kv_unpack_range, ok, 1, 1, FAKE, 4, 0, 16, FAKE) == mc.MC_OK
    pb = mc.mc_kv_pack_batch
    assert _status(pb, ok, 0, 3, 2, FAKE, FAKE, FAKE, FAKE, FAKE, 4, FAKE) == mc.MC_ERR_RANGE
    assert _status(pb, ok, 0, 1, -1, FAKE, FAKE, FAKE, FAKE, FAKE, 4, FAKE) == mc.MC_ERR_INVALID
    assert _status(pb, ok, 0, 1, 2, FAKE, FAKE, None, FAKE, FAKE, 4, FAKE) == mc.MC_ERR_INVALID
    assert _status(pb, ok, 0, 1, 2, FAKE, FAKE, FAKE, FAKE, FAKE + 4, 4, FAKE) == mc.MC_ERR_INVALID
    assert _status(pb, ok, 0, 1, 2, FAKE, FAKE, FAKE, FAKE, FAKE, 4, FAKE + 8) == mc.MC_ERR_INVALID
    assert _status(pb, ok, 0, 1, 0, FAKE, FAKE, FAKE, FAKE, FAKE, 4, FAKE) == mc.MC_OK
    assert _status(mc.mc_kv_unpack_batch, ok, 0, 1, 2, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE) == mc.MC_OK
    ap = mc.mc_kv_append
    assert _status(ap, ok, 2, FAKE, FAKE, 1, 16, FAKE, FAKE, FAKE, FAKE) == mc.MC_ERR_RANGE
    assert _status(ap, ok, 0, None, FAKE, 1, 16, FAKE, FAKE, FAKE, FAKE) == mc.MC_ERR_INVALID
    assert _status(ap, ok, 0, FAKE, FAKE, 1, -1, FAKE, FAKE, FAKE, FAKE) == mc.MC_ERR_INVALID
    assert _status(ap, ok, 0, FAKE, FAKE, 1, 0, FAKE, FAKE, FAKE, FAKE) == mc.MC_OK
    aps = mc.mc_kv_append_send
    assert _status(aps, ok, 0, FAKE, FAKE, 1, 16, FAKE, FAKE, FAKE, FAKE, 1, FAKE, FAKE, FAKE, FAKE) == mc.MC_ERR_RANGE
    assert _status(aps, ok, 0, FAKE, FAKE, 1, 16, FAKE, FAKE, FAKE, FAKE, 0, None, FAKE, FAKE, FAKE) == mc.MC_ERR_INVALID
    assert _status(aps, ok, 0, FAKE, FAKE, 1, 16, FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE + 4, FAKE) == mc.MC_ERR_INVALID
    assert _status(aps, ok, 0, FAKE, FAKE, 1, 16, FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, FAKE + 8) == mc.MC_ERR_INVALID
    assert _status(aps, ok, 0, FAKE, FAKE, 1, 0, FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, FAKE) == mc.MC_OK
    at = mc.mc_prefix_prefill_attn
    base = [ok, 0, FAKE, 32, 1, 16, FAKE, FAKE, FAKE, FAKE, 0.0, FAKE, FAKE, FAKE, 1 << 20]

    def attn(kw):
        a = list(base)
        for k, v in kw.items():
            a[k] = v
        return _status(at, *a)
    assert attn({3: 24}) == mc.MC_ERR_UNSUPPORTED     # 24 q heads over 8 kv heads: G = 3
    assert attn({3: 12}) == mc.MC_ERR_UNSUPPORTED     # not a multiple
    assert attn({1: 2}) == mc.MC_ERR_RANGE            # layer
    assert attn({10: -1.0}) == mc.MC_ERR_INVALID      # negative scale
    assert attn({10: float("nan")}) == mc.MC_ERR_INVALID
    assert attn({14: 16}) == mc.MC_ERR_INVALID        # workspace too small
    assert attn({11: None}) == mc.MC_ERR_INVALID
    assert attn({5: 0}) == mc.MC_OK                   # no new tokens: nothing to do
    pa = mc.mc_attn_plan_ahead
    assert _status(pa, ok, 32, 1, 16, FAKE, FAKE, FAKE, FAKE, -1, FAKE, 1 << 30) == mc.MC_ERR_RANGE
    assert _status(pa, ok, 32, 1, 16, FAKE, FAKE, FAKE, FAKE, 4, FAKE, 8) == mc.MC_ERR_INVALID
    pl = mc.mc_attn_plan
    assert _status(pl, ok, 32, 1, 16, FAKE, FAKE, FAKE, FAKE, FAKE, 8) == mc.MC_ERR_INVALID
    assert _status(pl, ok, 32, 1, 16, FAKE, FAKE, FAKE, FAKE, None, 1 << 20) == mc.MC_ERR_INVALID


def test_workspace_size():
    assert mc.mc_attn_workspace_size(1, 16, 32, 8) >= 64 + 8
    assert mc.mc_attn_workspace_size(8, 20000, 32, 8) < (1 << 20)      # many q tiles: no partials
    assert mc.mc_attn_workspace_size(8, 8, 32, 8) < (80 << 20)          # decode step: room for chunks
    assert mc.mc_attn_workspace_size(4, 3280, 64, 8) < (130 << 20)      # never more than the cap
    assert mc.mc_attn_workspace_size(1, 16, 24, 8) == 0
    assert mc.mc_attn_workspace_size(-1, 16, 32, 8) == 0
    s1 = mc.mc_attn_workspace_size(4, 1000, 32, 8)
    s2 = mc.mc_attn_workspace_size(4, 2000, 32, 8)
    assert s2 > s1 and s1 % 16 == 0


def _as_range(tokens, empty_at):
    if not tokens:
        return (empty_at, empty_at)
    assert tokens == list(range(tokens[0], tokens[-1] + 1))
    return (tokens[0], tokens[-1] + 1)


def test_plan_remote_send_matches_oracle_exhaustively():
    hi = 10
    for s in range(hi):
        for r in range(hi):
            for b in range(hi):
                for e in range(b, hi):
                    got = mc.mc_plan_remote_send(s, r, b, e)
                    want = oracle.send_plan(s, r, b, e)
                    for key in ("copy", "prefill", "send"):
                        lo, up = got[key]
                        assert lo <= up
                        if want[key]:
                            assert (lo, up) == _as_range(want[key], 0), (s, r, b, e, key, got)
                        else:
                            assert lo == up, (s, r, b, e, key, got)


def test_plan_remote_send_errors():
    for bad in [(-1, 0, 0, 1), (0, -1, 0, 1), (0, 0, -1, 1), (0, 0, 2, 1)]:
        with pytest.raises(mc.McError) as e:
            mc.mc_plan_remote_send(*bad)
        assert e.value.status == mc.MC_ERR_RANGE
    assert mc.lib().mc_plan_remote_send(1, 1, 0, 1, None) == mc.MC_ERR_INVALID


def test_addr_compress_expand():
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(0, 40))
        pages, p = [], int(rng.integers(0, 50))
        for _ in range(n):
            p = p + 1 if rng.random() < 0.6 else int(rng.integers(0, 1000))
            pages.append(p)
        runs = mc.mc_addr_compress(pages)
        assert runs == oracle.addr_runs(pages)
        assert mc.mc_addr_expand(runs) == pages
    with pytest.raises(mc.McError) as e:
        mc.mc_addr_compress([3, -1])
    assert e.value.status == mc.MC_ERR_RANGE
    for bad in ([(0, 0)], [(-1, 2)], [(2**31 - 2, 5)]):
        with pytest.raises(mc.McError) as e:
            mc.mc_addr_expand(bad, capacity=16)
        assert e.value.status == mc.MC_ERR_RANGE
    with pytest.raises(mc.McError) as e:
        mc.mc_addr_expand([(0, 5)], capacity=4)
    assert e.value.status == mc.MC_ERR_RANGE


def test_prefix_index_and_prep_recv_match_oracle():
    rng = np.random.default_rng(11)
    ix, oix = mc.mc_prefix_index_create(), oracle.PrefixIndex()
    al, oal = mc.mc_kv_allocator_create(4096), oracle.Allocator(4096)
    stems = [list(rng.integers(0, 50, size=int(rng.integers(0, 200)))) for _ in range(6)]
    try:
        for step in range(300):
            stem = stems[int(rng.integers(0, len(stems)))]
            cut = int(rng.integers(0, len(stem) + 1))
            prompt = [int(x) for x in stem[:cut]] + [int(x) for x in rng.integers(0, 50, size=int(rng.integers(0, 80)))]
            assert mc.mc_prefix_index_match(ix, prompt) == oix.match(prompt)
            end = int(rng.integers(0, len(prompt) + 1))
            want = oracle.prep_recv(oix, oal, prompt, end)
            if want is None:
                with pytest.raises(mc.McError) as e:
                    mc.mc_prep_recv(ix, al, prompt, end)
                assert e.value.status == mc.MC_ERR_NO_PAGES
                continue
            pages, m = mc.mc_prep_recv(ix, al, prompt, end)
            assert (pages, m) == want
            assert m % 16 == 0 and m <= end
            if step % 2 == 0:                  # the sequence's whole pages become matchable
                mc.mc_prefix_index_insert(ix, prompt[:end], pages)
                oix.insert(prompt[:end], pages)
            else:                              # or it goes away: only its fresh pages are returned
                fresh = pages[m // 16:]
                mc.mc_kv_free_pages(al, fresh)
                oal.give(fresh)
        assert mc.mc_kv_allocator_num_free(al) == oal.num_free
    finally:
        mc.mc_prefix_index_destroy(ix)
        mc.mc_kv_allocator_destroy(al)


def test_prefix_index_errors():
    ix = mc.mc_prefix_index_create()
    L = mc.lib()
    assert L.mc_prefix_index_insert(None, None, 0, None) == mc.MC_ERR_INVALID
    assert L.mc_prefix_index_insert(ix, None, -1, None) == mc.MC_ERR_RANGE
    assert L.mc_prefix_index_insert(ix, None, 16, None) == mc.MC_ERR_INVALID
    assert L.mc_prefix_index_insert(ix, None, 15, None) == mc.MC_OK       # no whole page: nothing to do
    with pytest.raises(mc.McError) as e:
        mc.mc_prefix_index_insert(ix, list(range(16)), [-3])
    assert e.value.status == mc.MC_ERR_RANGE
    assert L.mc_prefix_index_match(ix, None, 0, None, None) == mc.MC_ERR_INVALID
    assert L.mc_prep_recv(ix, None, None, 0, None, None) == mc.MC_ERR_INVALID
    assert mc.mc_prefix_index_match(ix, []) == (0, [])
    mc.mc_prefix_index_destroy(ix)


def test_fork_sequence_matches_oracle():
    al, oal = mc.mc_kv_allocator_create(12), oracle.Allocator(12)
    parent = mc.mc_kv_alloc_pages(al, 7)
    assert oal.take(7) == parent
    for n in (0, 1, 16, 17, 100, 112):
        got = mc.mc_kv_fork_sequence(al, parent, n)
        want = oracle.fork_sequence(oal, parent, n)
        assert got == want, (n, got, want)
        child, (src, dst, slots) = got
        assert child[: n // 16] == parent[: n // 16] and slots == n % 16
        if slots:
            assert src == parent[n // 16] and dst == child[-1] and dst not in parent
    # 3 pages went to forks with a partly filled last page (1, 17 and 100 tokens); two are left
    assert mc.mc_kv_allocator_num_free(al) == oal.num_free == 2
    mc.mc_kv_fork_sequence(al, parent, 5)
    mc.mc_kv_fork_sequence(al, parent, 5)
    with pytest.raises(mc.McError) as e:
        mc.mc_kv_fork_sequence(al, parent, 5)
    assert e.value.status == mc.MC_ERR_NO_PAGES
    assert mc.mc_kv_fork_sequence(al, parent, 32) == (parent[:2], (-1, -1, 0))    # needs no page
    ok = _pool()
    cp = mc.mc_kv_copy_page
    assert _status(cp, ok, 0, 3, 1, 2, 5) == mc.MC_ERR_RANGE
    assert _status(cp, ok, 0, 2, 8, 2, 5) == mc.MC_ERR_RANGE
    assert _status(cp, ok, 0, 2, 1, 2, 17) == mc.MC_ERR_RANGE
    assert _status(cp, ok, 0, 2, 1, 1, 5) == mc.MC_ERR_ALIAS
    assert _status(cp, ok, 0, 2, 1, 2, 0) == mc.MC_OK
    mc.mc_kv_allocator_destroy(al)
