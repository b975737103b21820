"""GPU parity on seeded random ragged batches: every row of every sequence against the oracle.
Shapes the other tests do not list one by one: random head groupings and dtypes, short prefill
ranges, short ranges over long contexts, decode rows mixed with prefill (some of them forks of
their neighbour), empty and one-token ranges."""
import numpy as np
import pytest

import mc_inputs as mi
from test_gpu_parity import check_attention, small_workload

pytestmark = pytest.mark.gpu

HEADS = [(8, 8), (8, 2), (16, 2), (32, 8), (4, 2), (16, 16), (64, 8)]


def random_workload(case, rng):
    Hq, Hkv = HEADS[int(rng.integers(0, len(HEADS)))]
    dtype = [mi.F16, mi.BF16][int(rng.integers(0, 2))]
    kind = int(rng.integers(0, 4))
    batch = int(rng.integers(1, 9)) if kind != 2 else int(rng.integers(2, 40))
    lens, begins = [], []
    for _ in range(batch):
        if kind == 0:      # short prefill ranges
            n = int(rng.integers(1, 400))
            b = int(rng.integers(0, n + 1))
        elif kind == 1:    # long contexts, short ranges
            n = int(rng.integers(300, 3000))
            b = n - int(rng.integers(0, 40))
        elif kind == 2:    # decode rows with a few prefill ranges
            n = int(rng.integers(1, 2500))
            b = n - 1 if rng.random() < 0.8 else int(rng.integers(0, n + 1))
        else:
            n = int(rng.integers(1, 1200))
            b = int(rng.integers(0, n + 1))
        lens.append(n)
        begins.append(b)
    if sum(n - b for n, b in zip(lens, begins)) == 0:
        begins[0] = max(0, lens[0] - 1)
    w = small_workload(9000 + case, dtype, Hq, Hkv, lens, begins)
    if kind == 2 and rng.random() < 0.5:       # neighbouring decode rows forked from one another
        for s in range(1, batch):
            both_decode = lens[s] - begins[s] == 1 and lens[s - 1] - begins[s - 1] == 1
            if both_decode and rng.random() < 0.7:
                pages = min(begins[s], begins[s - 1]) // 16
                shared = int(rng.integers(0, pages + 1)) * 16
                if shared:
                    w.share_prefix(s, s - 1, shared)
    return w


@pytest.mark.parametrize("chunk", range(6))
def test_random_batches(chunk):
    rng = np.random.default_rng(4000 + chunk)
    for i in range(10):
        check_attention(random_workload(10 * chunk + i, rng))


def test_random_copies():
    """append, batched pack and batched unpack on seeded random shapes (1..3 layers, 1..16 kv
    heads, ragged ranges): pools and buffers byte for byte, canary bytes everywhere else."""
    import torch

    import oracle
    import paper_2412_12488_amd as mc
    from gpu_harness import DEV, DevBatch, DevPool, bits, dev, gpu_append
    from test_gpu_parity import canary
    rng = np.random.default_rng(77)
    for case in range(30):
        L, Hkv, dtype = int(rng.integers(1, 4)), int(rng.choice([1, 2, 3, 8, 16])), int(rng.integers(0, 2))
        B = int(rng.integers(1, 7))
        lens = [int(rng.integers(1, 600)) for _ in range(B)]
        begins = [int(rng.integers(0, n + 1)) for n in lens]
        w = small_workload(20000 + case, dtype, Hkv, Hkv, lens, begins, layers=L)
        init = canary(case, DevPool(w).elems)
        pool, opool = DevPool(w, fill=init), init.copy()
        db = DevBatch(w)
        if db.total_q:
            for layer in range(L):
                ks = np.concatenate([w.kv(s, layer)[0][begins[s]:lens[s]] for s in range(B)])
                vs = np.concatenate([w.kv(s, layer)[1][begins[s]:lens[s]] for s in range(B)])
                gpu_append(pool, layer, dev(ks), dev(vs), db)
                for s in range(B):
                    if lens[s] > begins[s]:
                        k, v = w.kv(s, layer)
                        oracle.append(opool, pool.shape, layer, k[begins[s]:lens[s]],
                                      v[begins[s]:lens[s]], begins[s], w.page_tables[s])
            torch.cuda.synchronize()
            assert np.array_equal(bits(pool.t), opool), case
        s0 = [int(rng.integers(0, n + 1)) for n in lens]
        s1 = [int(rng.integers(a, n + 1)) for a, n in zip(s0, lens)]
        lb = int(rng.integers(0, L))
        le = int(rng.integers(lb, L + 1))
        sizes = [(le - lb) * 2 * (b - a) * Hkv * 128 for a, b in zip(s0, s1)]
        offs, at = [], 64
        for n in sizes:
            offs.append(at)
            at += n + 64 + (-n % 8)
        raw = canary(case + 1, at)
        send = dev(raw)
        d_s0, d_s1 = dev(np.array(s0, np.int32)), dev(np.array(s1, np.int32))
        d_off = torch.tensor([2 * o for o in offs], dtype=torch.int64, device=DEV)
        max_pages = max(((b - 1) // 16 - a // 16 + 1) if b > a else 0 for a, b in zip(s0, s1))
        mc.mc_kv_pack_batch(pool.desc, lb, le, B, db.page_table, db.cu_pages, d_s0, d_s1, d_off,
                            max_pages, send)
        torch.cuda.synchronize()
        expect, refs = raw.copy(), []
        for i in range(B):
            refs.append(oracle.pack(opool, pool.shape, lb, le, w.page_tables[i], s0[i], s1[i]))
            expect[offs[i]:offs[i] + sizes[i]] = refs[i].ravel()
        assert np.array_equal(bits(send), expect), case
        init_b = canary(case + 2, pool.elems)
        pool_b = DevPool(w, fill=init_b)
        tables_b = mi.scatter_page_tables(mi.rng_for(case, 5), w.num_pages, w.n)
        wb = mi.Workload("b", w.seed, w.dtype, L, Hkv, Hkv, w.num_pages, w.n, w.b, tables_b)
        dbb = DevBatch(wb)
        mc.mc_kv_unpack_batch(pool_b.desc, lb, le, B, dbb.page_table, dbb.cu_pages, d_s0, d_s1,
                              d_off, max_pages, send)
        torch.cuda.synchronize()
        ob = init_b.copy()
        for i in range(B):
            oracle.unpack(ob, pool.shape, lb, le, tables_b[i], s0[i], s1[i], refs[i])
        assert np.array_equal(bits(pool_b.t), ob), case
