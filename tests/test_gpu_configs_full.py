"""Configs 3 and 5 at full size on the GPU, in the launch configuration the benchmark uses.

The oracle checks, per config, every row and q head of one layer of the smallest sequence and
a seeded sample of more than 4096 (sequence, q head, row) triples spread over all sequences and
several layers: range ends, first and last rows of q tiles from the start to the end of the
range, the ragged last tile, both sides of page boundaries, one q head of every kv head's group
per row.  Whole layers of the copies are compared byte for byte; properties that hold at any
size cover every layer: split passes against the single pass, and pool B against pool A through
the two page tables."""
import numpy as np
import pytest
import torch

import mc_inputs as mi
import oracle
import paper_2412_12488_amd as mc
from gpu_harness import DEV, DevBatch, DevPool, bits, dev, gpu_append, gpu_attention, layer_variant_dev

pytestmark = pytest.mark.gpu
O_TOL, LSE_TOL = 2e-2, 1e-3


def host_layer(w, s, layer, base):
    k0, v0, q0 = base[s]
    return mi.layer_variant(k0, layer), mi.layer_variant(v0, layer), mi.layer_variant(q0, layer)


def check_rows(w, opool, shape, layer, seq, q_bits, begin, end, out_rows, lse_rows, seed, count):
    """out_rows / lse_rows: device tensors of the rows [begin, end) of sequence seq; count = number
    of (row, q head) pairs to check, or None for every row and head.  Returns the pairs checked."""
    q_len = end - begin
    if count is None:
        rr, hh = np.meshgrid(np.arange(q_len, dtype=np.int32),
                             np.arange(w.num_q_heads, dtype=np.int32), indexing="ij")
        rows, heads = rr.ravel(), hh.ravel()
    else:
        rows, heads = mi.sample_rows(mi.rng_for(seed, seq, layer), q_len, begin, w.num_q_heads, count,
                                     tile_tokens=128 // (w.num_q_heads // w.num_kv_heads),
                                     num_kv_heads=w.num_kv_heads)
    ro, rl = oracle.attention(opool, shape, layer, w.page_tables[seq], q_bits, w.num_q_heads, begin,
                              end, sel_rows=rows, sel_heads=heads)
    go = oracle.decode(bits(out_rows)[rows, heads], w.dtype)
    gl = lse_rows.cpu().numpy().astype(np.float64)[rows, heads]
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    eo, el = float(np.max(np.abs(go - ro))), float(np.max(np.abs(gl - rl)))
    assert eo <= O_TOL, (layer, seq, eo)
    assert el <= LSE_TOL, (layer, seq, el)
    return int(rows.size)


def pools_agree(pool_a, table_a, pool_b, table_b, w, upto):
    """Every (layer, K|V, head) row of tokens [0, upto) is the same in both pools."""
    pages = -(-upto // 16)
    dims = (pool_a.num_layers, -1, 2, w.num_kv_heads, 16, 128)
    a = pool_a.t.view(dims)[:, table_a[:pages].long()]
    b = pool_b.t.view((pool_b.num_layers, -1, 2, w.num_kv_heads, 16, 128))[:, table_b[:pages].long()]
    full = upto // 16
    ok = torch.equal(a[:, :full], b[:, :full])
    if upto % 16:
        ok = ok and torch.equal(a[:, full, :, :, : upto % 16], b[:, full, :, :, : upto % 16])
    return bool(ok)


def test_config3_balanced_split_32_layers():
    w = mi.config(3)
    L, B = w.num_layers, w.batch
    m = (w.n // 2).astype(np.int64)
    base = [(*w.kv(s, 0), mi.normal_bits(mi.rng_for(w.seed, s, mi.KIND_Q),
                                         (int(w.n[s]), w.num_q_heads, 128), w.dtype)) for s in range(B)]
    dk = [dev(k) for k, _, _ in base]
    dv = [dev(v) for _, v, _ in base]
    dq = [dev(q) for _, _, q in base]
    pool = DevPool(w)
    pool.t.fill_(0x7fc1)
    w_a = w.with_ranges(np.zeros_like(m), m)          # pass A: [0, m), nothing cached
    w_b = w.with_ranges(m, w.n)                        # pass B: [m, n) over the cached [0, m)
    w_c = w.with_ranges(np.zeros_like(m), w.n)         # check pass: [0, n)
    db_a, db_b, db_c = DevBatch(w_a), DevBatch(w_b), DevBatch(w_c)
    oracle_layers = (0, 17, L - 1)
    opool = np.full(pool.elems, 0x7fc1, dtype=np.uint16)
    worst_split_o = worst_split_l = 0.0
    triples = 0
    for layer in range(L):
        kl = [layer_variant_dev(t, layer) for t in dk]
        vl = [layer_variant_dev(t, layer) for t in dv]
        ql = [layer_variant_dev(t, layer) for t in dq]
        cat = lambda ts, lo, hi: torch.cat([t[lo[s]:hi[s]] for s, t in enumerate(ts)])
        zero = np.zeros(B, dtype=np.int64)
        gpu_append(pool, layer, cat(kl, zero, m), cat(vl, zero, m), db_a)
        o_a, l_a = gpu_attention(pool, layer, cat(ql, zero, m), db_a, check_plan=(layer == 0))
        gpu_append(pool, layer, cat(kl, m, w.n), cat(vl, m, w.n), db_b)
        o_b, l_b = gpu_attention(pool, layer, cat(ql, m, w.n), db_b, check_plan=(layer == 0))
        o_c, l_c = gpu_attention(pool, layer, cat(ql, zero, w.n), db_c, check_plan=(layer == 0))
        # rows of A followed by rows of B are the rows of the single pass (every layer, all rows)
        f = lambda t: t.view(torch.bfloat16).float()
        for s in range(B):
            a0, b0, c0 = int(w_a.cu_q[s]), int(w_b.cu_q[s]), int(w_c.cu_q[s])
            ms, ns = int(m[s]), int(w.n[s])
            parts_o = torch.cat([f(o_a[a0:a0 + ms]), f(o_b[b0:b0 + ns - ms])])
            parts_l = torch.cat([l_a[a0:a0 + ms], l_b[b0:b0 + ns - ms]])
            worst_split_o = max(worst_split_o, float((parts_o - f(o_c[c0:c0 + ns])).abs().max()))
            worst_split_l = max(worst_split_l, float((parts_l - l_c[c0:c0 + ns]).abs().max()))
        if layer in oracle_layers:
            for s in range(B):
                k, v, q = host_layer(w, s, layer, base)
                oracle.append(opool, pool.shape, layer, k, v, 0, w.page_tables[s])
            smallest = int(np.argmin(w.n))
            for s in range(B):       # every sequence: 256 pairs of the second pass, 256 of the single pass
                _, _, q = host_layer(w, s, layer, base)
                ms, ns = int(m[s]), int(w.n[s])
                b0, c0 = int(w_b.cu_q[s]), int(w_c.cu_q[s])
                # the smallest sequence, first layer: every row and q head of both passes
                every = layer == oracle_layers[0] and s == smallest
                triples += check_rows(w, opool, pool.shape, layer, s, q[ms:], ms, ns,
                                      o_b[b0:b0 + ns - ms], l_b[b0:b0 + ns - ms], 3,
                                      None if every else 256)
                triples += check_rows(w, opool, pool.shape, layer, s, q, 0, ns, o_c[c0:c0 + ns],
                                      l_c[c0:c0 + ns], 33, None if every else 256)
    assert triples >= 4096 + 32 * int(np.min(w.n)), triples
    assert worst_split_o <= O_TOL, worst_split_o
    assert worst_split_l <= LSE_TOL, worst_split_l
    # ---- ship [0, m) of every sequence, all 32 layers, into a second pool ----
    pool_b = DevPool(w)
    pool_b.t.fill_(0x1234)
    tables_b = mi.scatter_page_tables(mi.rng_for(w.seed, 55), w.num_pages, w.n)
    for s in range(B):
        ms = int(m[s])
        send = torch.empty(L * 2 * ms * w.num_kv_heads * 128, dtype=torch.int16, device=DEV)
        ta, tb = db_c.tables[s], dev(tables_b[s])
        mc.mc_kv_pack_range(pool.desc, 0, L, ta, len(w.page_tables[s]), 0, ms, send)
        mc.mc_kv_unpack_range(pool_b.desc, 0, L, tb, len(tables_b[s]), 0, ms, send)
        torch.cuda.synchronize()
        assert pools_agree(pool, ta, pool_b, tb, w, ms)
        if s in (0, B - 1):      # bytes of the transfer buffer against the oracle, sampled layers
            per_layer = 2 * ms * w.num_kv_heads * 128
            got = bits(send).reshape(L, per_layer)
            for layer in oracle_layers:
                ref = oracle.pack(opool, pool.shape, layer, layer + 1, w.page_tables[s], 0, ms)
                assert np.array_equal(got[layer], ref.ravel()), (s, layer)
        del send
    # nothing outside the addressed slots of pool B was written
    used = torch.zeros(w.num_pages, dtype=torch.bool, device=DEV)
    for s in range(B):
        used[dev(tables_b[s])[: -(-int(m[s]) // 16)].long()] = True
    untouched = pool_b.t.view(L, w.num_pages, -1)[:, ~used]
    assert bool((untouched == 0x1234).all())


def test_config5_long_context():
    w = mi.config(5)
    L = w.num_layers
    base = [(*w.kv(s, 0), w.q(s, 0)) for s in range(2)]
    pool = DevPool(w)
    pool.t.fill_(0x7fc1)
    opool = np.full(pool.elems, 0x7fc1, dtype=np.uint16)
    whole = w.with_ranges(np.zeros(2, dtype=np.int64), w.n)
    db_fill, db = DevBatch(whole), DevBatch(w)
    dk = [dev(b[0]) for b in base]
    dv = [dev(b[1]) for b in base]
    dq = [dev(b[2]) for b in base]
    for layer in range(L):
        gpu_append(pool, layer, torch.cat([layer_variant_dev(t, layer) for t in dk]),
                   torch.cat([layer_variant_dev(t, layer) for t in dv]), db_fill)
    triples = 0
    for layer in (0, L - 1):
        q_dev = torch.cat([layer_variant_dev(t, layer) for t in dq])
        out, lse = gpu_attention(pool, layer, q_dev, db)
        for s in range(2):
            k, v, q = host_layer(w, s, layer, base)
            oracle.append(opool, pool.shape, layer, k, v, 0, w.page_tables[s])
            lo, ql = int(w.cu_q[s]), int(w.n[s] - w.b[s])
            # the 16384-token sequence, first layer: every row and q head; else 2048 pairs
            every = layer == 0 and s == 0
            triples += check_rows(w, opool, pool.shape, layer, s, q, int(w.b[s]), int(w.n[s]),
                                  out[lo:lo + ql], lse[lo:lo + ql], 5, None if every else 2048)
    assert triples >= 3 * 2048 + 32 * 8192, triples
    # ---- 32768 tokens x 32 layers (4 GiB of KV) to a second pool ----
    s, n = 1, int(w.n[1])
    pool_b = DevPool(w)
    pool_b.t.fill_(0x1234)
    table_b = mi.rng_for(w.seed, 56).permutation(w.num_pages)[: len(w.page_tables[s])].astype(np.int32)
    send = torch.empty(L * 2 * n * w.num_kv_heads * 128, dtype=torch.int16, device=DEV)
    ta, tb = db.tables[s], dev(table_b)
    mc.mc_kv_pack_range(pool.desc, 0, L, ta, len(w.page_tables[s]), 0, n, send)
    mc.mc_kv_unpack_range(pool_b.desc, 0, L, tb, len(table_b), 0, n, send)
    torch.cuda.synchronize()
    assert pools_agree(pool, ta, pool_b, tb, w, n)
    per_layer = 2 * n * w.num_kv_heads * 128
    for layer in (0, L - 1):
        ref = oracle.pack(opool, pool.shape, layer, layer + 1, w.page_tables[s], 0, n)
        got = bits(send[layer * per_layer:(layer + 1) * per_layer])
        assert np.array_equal(got, ref.ravel()), layer
    used = torch.zeros(w.num_pages, dtype=torch.bool, device=DEV)
    used[tb.long()] = True
    assert bool((pool_b.t.view(L, w.num_pages, -1)[:, ~used] == 0x1234).all())
