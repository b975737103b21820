"""Per-layer overlap of the KV transfer with the next layer's computation (paper Sec. 3.6:
a computation stream and a communication stream, a layer's KV leaves as soon as the layer has
produced it), on one GPU: layer l's KV goes pool A -> transfer buffer -> pool B on a side
stream while layer l+1 appends and attends on the main stream.  Both streams have the default
priority.  Every layer's O and LSE, every byte of the transfer buffers and every byte of the
receiving pool are compared with the oracle."""
import numpy as np
import pytest
import torch

import mc_inputs as mi
import oracle
import paper_2412_12488_amd as mc
from gpu_harness import DEV, DevBatch, DevPool, bits, dev, layer_variant_dev

pytestmark = pytest.mark.gpu
O_TOL, LSE_TOL = 2e-2, 1e-3


def _workload(seed, layers, Hq, Hkv, lens, begins):
    n, b = np.array(lens), np.array(begins)
    pages = int(sum(-(-int(t) // 16) for t in n)) + 9
    w = mi.Workload(f"overlap-{seed}", seed, mi.BF16, layers, Hq, Hkv, pages, n, b)
    w.page_tables = mi.scatter_page_tables(mi.rng_for(seed, mi.KIND_TABLE), pages, n)
    return w


@pytest.mark.parametrize("fused_send", [False, True])
def test_transfer_of_layer_l_runs_beside_layer_l_plus_1(fused_send):
    """fused_send: the new range reaches the transfer buffer from the append itself
    (mark_send, mc_kv_append_send) and only the cached part is packed on the side stream."""
    L, Hq, Hkv = 5, 32, 8
    lens, begins = [700, 333, 1200, 90, 257], [130, 0, 1199, 45, 256]
    w = _workload(1201, L, Hq, Hkv, lens, begins)
    B = w.batch
    canary = lambda seed, n: mi.rng_for(seed, 99).integers(0, 65536, size=n, dtype=np.uint16)
    init_a, init_b = canary(1, DevPool(w).elems), canary(2, DevPool(w).elems)
    pool_a, pool_b = DevPool(w, fill=init_a), DevPool(w, fill=init_b)
    opool_a, opool_b = init_a.copy(), init_b.copy()
    tables_b = mi.scatter_page_tables(mi.rng_for(1202), w.num_pages, w.n)
    wb = mi.Workload("recv", w.seed, w.dtype, L, Hq, Hkv, w.num_pages, w.n, w.b, tables_b)
    db, dbb = DevBatch(w), DevBatch(wb)
    cached = DevBatch(w.with_ranges(np.zeros_like(w.b), w.b))
    k0 = [dev(w.kv(s)[0]) for s in range(B)]
    v0 = [dev(w.kv(s)[1]) for s in range(B)]
    q0 = [dev(w.q(s)) for s in range(B)]
    cat = lambda ts, lo, hi, layer: torch.cat(
        [layer_variant_dev(t, layer)[int(lo[s]):int(hi[s])] for s, t in enumerate(ts)])
    zero = np.zeros(B, dtype=np.int64)
    # the cached prefixes of every layer are in pool A before the pass starts
    for layer in range(L):
        mc.mc_kv_append(pool_a.desc, layer, cat(k0, zero, w.b, layer), cat(v0, zero, w.b, layer),
                        B, cached.total_q, cached.cu_q, cached.begin, cached.page_table,
                        cached.cu_pages)
        for s in range(B):
            k, v = w.kv(s, layer)
            if w.b[s]:
                oracle.append(opool_a, pool_a.shape, layer, k[: w.b[s]], v[: w.b[s]], 0,
                              w.page_tables[s])
    # One transfer buffer per layer, one slice [2][tokens][Hkv][D] per sequence with guard
    # elements around it.  Plain: the slice holds the whole sequence [0, n), packed after the
    # layer's append.  Fused: the cached part [0, b) of all layers is copied ahead, on the side
    # stream, while the first layers compute (it needs no computation: the range a sender "sends
    # as it is", Sec. 3.5); the per-layer slice holds only the new range [b, n), written by the
    # append itself.
    lo_tok = w.b if fused_send else np.zeros_like(w.b)
    sizes = [2 * int(n - lo) * Hkv * 128 for n, lo in zip(w.n, lo_tok)]
    guard, offs, at = 64, [], 64
    for sz in sizes:
        offs.append(at)
        at += sz + guard
    raw = canary(3, at)
    sends = [dev(raw) for _ in range(L)]
    d_off = torch.tensor([2 * o for o in offs], dtype=torch.int64, device=DEV)
    d_zero = dev(np.zeros(B, np.int32))
    d_b, d_n = dev(w.b.astype(np.int32)), dev(w.n.astype(np.int32))
    d_lo = d_b if fused_send else d_zero
    max_pages = int(max(-(-int(n) // 16) for n in w.n))
    ws_bytes = mc.mc_attn_workspace_size(B, db.total_q, Hq, Hkv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    outs = [torch.full((db.total_q, Hq, 128), 0x7fc1, dtype=torch.int16, device=DEV) for _ in range(L)]
    lses = [torch.full((db.total_q, Hq), float("nan"), dtype=torch.float32, device=DEV) for _ in range(L)]
    kn = [cat(k0, w.b, w.n, layer) for layer in range(L)]
    vn = [cat(v0, w.b, w.n, layer) for layer in range(L)]
    qn = [cat(q0, zero, w.n - w.b, layer) for layer in range(L)]
    # cached part, all layers in one buffer [L][2][b][Hkv][D] per sequence
    c_sizes = [L * 2 * int(b) * Hkv * 128 for b in w.b]
    c_offs = np.concatenate([[0], np.cumsum(c_sizes)[:-1]]).astype(np.int64)
    c_send = torch.zeros(max(int(sum(c_sizes)), 8), dtype=torch.int16, device=DEV)
    d_coff = torch.from_numpy(c_offs * 2).to(DEV)
    torch.cuda.synchronize()

    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    appended = [torch.cuda.Event() for _ in range(L)]
    side.wait_stream(main)
    if fused_send:
        mc.mc_kv_pack_batch(pool_a.desc, 0, L, B, db.page_table, db.cu_pages, d_zero, d_b, d_coff,
                            max_pages, c_send, stream=side)
        mc.mc_kv_unpack_batch(pool_b.desc, 0, L, B, dbb.page_table, dbb.cu_pages, d_zero, d_b,
                              d_coff, max_pages, c_send, stream=side)
    # begin_forward: one plan for all layers
    mc.mc_attn_plan(pool_a.desc, Hq, B, db.total_q, db.cu_q, db.begin, db.page_table, db.cu_pages,
                    ws, ws_bytes, stream=main)
    for layer in range(L):
        # main stream: the layer's new K/V into the pages, then its attention
        if fused_send:
            mc.mc_kv_append_send(pool_a.desc, layer, kn[layer], vn[layer], B, db.total_q, db.cu_q,
                                 db.begin, db.page_table, db.cu_pages, layer, d_b, d_n, d_off,
                                 sends[layer], stream=main)
        else:
            mc.mc_kv_append(pool_a.desc, layer, kn[layer], vn[layer], B, db.total_q, db.cu_q,
                            db.begin, db.page_table, db.cu_pages, stream=main)
        appended[layer].record(main)
        mc.mc_prefix_prefill_attn(pool_a.desc, layer, qn[layer], Hq, B, db.total_q, db.cu_q,
                                  db.begin, db.page_table, db.cu_pages, 0.0, outs[layer],
                                  lses[layer], ws, ws_bytes, stream=main)
        # side stream: as soon as the layer's KV is in the pages (or in the buffer) it leaves
        # for pool B, beside this layer's attention and the next layer's append
        side.wait_event(appended[layer])
        if not fused_send:
            mc.mc_kv_pack_batch(pool_a.desc, layer, layer + 1, B, db.page_table, db.cu_pages,
                                d_zero, d_n, d_off, max_pages, sends[layer], stream=side)
        mc.mc_kv_unpack_batch(pool_b.desc, layer, layer + 1, B, dbb.page_table, dbb.cu_pages,
                              d_lo, d_n, d_off, max_pages, sends[layer], stream=side)
    main.wait_stream(side)
    torch.cuda.synchronize()
    mc.mc_attn_plan_check(ws)

    # ---- oracle: append, attention, pack, unpack, layer by layer ----
    for layer in range(L):
        for s in range(B):
            k, v = w.kv(s, layer)
            if w.n[s] > w.b[s]:
                oracle.append(opool_a, pool_a.shape, layer, k[w.b[s]:], v[w.b[s]:], int(w.b[s]),
                              w.page_tables[s])
    assert np.array_equal(bits(pool_a.t), opool_a)
    for layer in range(L):
        expect = raw.copy()
        for s in range(B):
            lo, n = int(lo_tok[s]), int(w.n[s])
            ref = oracle.pack(opool_a, pool_a.shape, layer, layer + 1, w.page_tables[s], lo, n)
            expect[offs[s]:offs[s] + sizes[s]] = ref.ravel()
            oracle.unpack(opool_b, pool_b.shape, layer, layer + 1, tables_b[s], lo, n, ref)
            if fused_send and w.b[s]:
                ref = oracle.pack(opool_a, pool_a.shape, layer, layer + 1, w.page_tables[s], 0, lo)
                oracle.unpack(opool_b, pool_b.shape, layer, layer + 1, tables_b[s], 0, lo, ref)
        assert np.array_equal(bits(sends[layer]), expect), layer     # slices and guard elements
        for s in range(B):
            q_len = int(w.n[s] - w.b[s])
            if q_len == 0:
                continue
            lo = int(w.cu_q[s])
            ro, rl = oracle.attention(opool_a, pool_a.shape, layer, w.page_tables[s], w.q(s, layer),
                                      Hq, int(w.b[s]), int(w.n[s]))
            go = oracle.decode(bits(outs[layer][lo:lo + q_len]), w.dtype)
            gl = lses[layer][lo:lo + q_len].cpu().numpy().astype(np.float64)
            assert float(np.max(np.abs(go - ro))) <= O_TOL, (layer, s)
            assert float(np.max(np.abs(gl - rl))) <= LSE_TOL, (layer, s)
    assert np.array_equal(bits(pool_b.t), opool_b)     # every addressed slot, every other byte
