"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on
the same seeded inputs.  Bars: bit-exact for every byte the copies touch or must not
touch; max abs error <= 2e-2 on fp16/bf16 attention outputs; LSE within 1e-3."""
import numpy as np
import pytest
import torch

import mc_inputs as mi
import oracle
import paper_2412_12488_amd as mc
from gpu_harness import (DEV, DevBatch, DevPool, bits, dev, fill_both, gpu_append, gpu_attention,
                         oracle_rows)

pytestmark = pytest.mark.gpu
O_TOL, LSE_TOL = 2e-2, 1e-3


def small_workload(seed, dtype, Hq, Hkv, lens, begins, num_pages=None, layers=1):
    n, b = np.array(lens), np.array(begins)
    need = int(sum(-(-int(t) // 16) for t in n))
    num_pages = num_pages or need + 7
    w = mi.Workload(f"small-{seed}", seed, dtype, layers, Hq, Hkv, num_pages, n, b)
    w.page_tables = mi.scatter_page_tables(mi.rng_for(seed, mi.KIND_TABLE), num_pages, n)
    return w


def canary(seed, elems):
    return mi.rng_for(seed, 99).integers(0, 65536, size=elems, dtype=np.uint16)


# ------------------------------------------------------------------ append ----
@pytest.mark.parametrize("case", [
    dict(dtype=mi.F16, Hkv=8, lens=[512], begins=[256]),
    dict(dtype=mi.BF16, Hkv=8, lens=[45, 1, 300, 16, 77], begins=[13, 0, 299, 16, 0]),
    dict(dtype=mi.BF16, Hkv=2, lens=[100, 64], begins=[33, 48]),
    dict(dtype=mi.BF16, Hkv=12, lens=[70], begins=[5]),
])
def test_append_bytes(case):
    w = small_workload(101, case["dtype"], case["Hkv"], case["Hkv"], case["lens"], case["begins"],
                       layers=2)
    init = canary(1, DevPool(w).elems)
    pool = DevPool(w, fill=init)
    opool = init.copy()
    db = DevBatch(w)
    ks, vs = [], []
    for s in range(w.batch):
        k, v = w.kv(s, 1)
        k, v = k[w.b[s]:], v[w.b[s]:]
        ks.append(k), vs.append(v)
        if len(k):
            oracle.append(opool, pool.shape, 1, k, v, int(w.b[s]), w.page_tables[s])
    gpu_append(pool, 1, dev(np.concatenate(ks)), dev(np.concatenate(vs)), db)
    torch.cuda.synchronize()
    assert np.array_equal(bits(pool.t), opool)          # addressed slots and every other byte
    assert not np.array_equal(opool, init)


def test_copies_report_what_they_skip():
    """Tokens and pages a copy kernel leaves out because a table index or a page id is out of
    bounds are counted (mc_kv_copy_check); well-formed calls count nothing, and what is left out
    is neither read nor written."""
    w = small_workload(106, mi.BF16, 8, 8, [45, 100, 33], [13, 0, 32], layers=2)
    init = canary(12, DevPool(w).elems)
    counter = torch.zeros(1, dtype=torch.int32, device=DEV)
    pool = DevPool(w, fill=init)
    pool.desc = mc.pool_desc(pool.t, 2, w.num_pages, 8, w.dtype, skipped=counter)
    db = DevBatch(w)
    k = dev(np.concatenate([w.kv(s, 1)[0][w.b[s]:] for s in range(3)]))
    v = dev(np.concatenate([w.kv(s, 1)[1][w.b[s]:] for s in range(3)]))
    gpu_append(pool, 1, k, v, db)
    assert mc.mc_kv_copy_check(pool.desc) == (mc.MC_OK, 0)
    # a page id outside the pool in sequence 1 (tokens 16..31) and a table one entry too short
    # for sequence 2 (its token 32 has no page): 16 + 1 tokens are left out
    good = bits(pool.t).copy()
    pool.t.copy_(dev(init))
    table = w.flat_page_table.copy()
    table[int(w.cu_pages[1]) + 1] = w.num_pages + 3
    cu_pages = w.cu_pages.copy()
    cu_pages[3] -= 1
    mc.mc_kv_append(pool.desc, 1, k, v, 3, db.total_q, db.cu_q, db.begin, dev(table), dev(cu_pages))
    assert mc.mc_kv_copy_check(pool.desc) == (mc.MC_ERR_RANGE, 17)
    assert mc.mc_kv_copy_check(pool.desc) == (mc.MC_OK, 0)          # the check set it back to zero
    got = bits(pool.t)
    shape5 = (2, w.num_pages, 2, 8, 16, 128)
    g5, ok5, i5 = got.reshape(shape5), good.reshape(shape5), init.reshape(shape5)
    bad_page, short_page = int(w.page_tables[1][1]), int(w.page_tables[2][2])
    for page in range(w.num_pages):          # skipped tokens leave their slots as they were
        ref = i5 if page in (bad_page, short_page) else ok5
        assert np.array_equal(g5[:, page], ref[:, page]), page
    # pack with the bad table: the page is counted once, its slice of the buffer stays untouched
    send = dev(canary(13, 2 * 2 * 100 * 8 * 128))
    before = bits(send).copy()
    mc.mc_kv_pack_range(pool.desc, 0, 2, dev(table[w.cu_pages[1]:w.cu_pages[2]]), 7, 0, 100, send)
    assert mc.mc_kv_copy_check(pool.desc) == (mc.MC_ERR_RANGE, 1)
    after = bits(send).reshape(2, 2, 100, 8 * 128)
    assert np.array_equal(after[:, :, 16:32], before.reshape(2, 2, 100, 8 * 128)[:, :, 16:32])
    assert not np.array_equal(after[:, :, :16], before.reshape(2, 2, 100, 8 * 128)[:, :, :16])
    # batched unpack: a sequence with a misaligned buffer offset is left out and counted once;
    # an empty range is not counted
    s0, s1 = dev(np.array([0, 0, 5], np.int32)), dev(np.array([45, 100, 5], np.int32))
    off = torch.tensor([0, 8, 0], dtype=torch.int64, device=DEV)
    mc.mc_kv_unpack_batch(pool.desc, 0, 1, 3, db.page_table, db.cu_pages, s0, s1, off, 7, send)
    assert mc.mc_kv_copy_check(pool.desc) == (mc.MC_ERR_RANGE, 1)


def test_append_nothing_is_a_no_op():
    w = small_workload(102, mi.BF16, 8, 8, [32], [32])
    init = canary(2, DevPool(w).elems)
    pool = DevPool(w, fill=init)
    db = DevBatch(w)
    gpu_append(pool, 0, dev(np.zeros(16, np.uint16)), dev(np.zeros(16, np.uint16)), db)
    torch.cuda.synchronize()
    assert np.array_equal(bits(pool.t), init)


# ------------------------------------------------------------- pack / unpack ----
@pytest.mark.parametrize("s0,s1", [(0, 256), (0, 512), (13, 40), (7, 8), (16, 48), (250, 507),
                                   (511, 512), (100, 100)])
@pytest.mark.parametrize("Hkv", [8, 3])
def test_pack_unpack_bytes(s0, s1, Hkv):
    L = 3
    w = small_workload(103, mi.F16, Hkv, Hkv, [512], [0], num_pages=64, layers=L)
    init = canary(3, DevPool(w).elems)
    pool_a = DevPool(w, fill=init)
    table = w.page_tables[0]
    T = s1 - s0
    guard = 64
    payload = (L - 1) * 2 * T * Hkv * 128
    raw = canary(4, payload + 2 * guard)
    send = dev(raw)
    mc.mc_kv_pack_range(pool_a.desc, 1, L, dev(table), len(table), s0, s1, send[guard:])
    torch.cuda.synchronize()
    got = bits(send)
    ref = oracle.pack(init, pool_a.shape, 1, L, table, s0, s1)
    assert np.array_equal(got[guard:guard + payload], ref.ravel())
    assert np.array_equal(got[:guard], raw[:guard]) and np.array_equal(got[guard + payload:],
                                                                      raw[guard + payload:])
    assert np.array_equal(bits(pool_a.t), init)                      # pack writes no page
    # receiver: a second pool with its own table and canaries
    init_b = canary(5, pool_a.elems)
    pool_b = DevPool(w, fill=init_b)
    table_b = mi.rng_for(6).permutation(64)[: len(table)].astype(np.int32)
    mc.mc_kv_unpack_range(pool_b.desc, 1, L, dev(table_b), len(table_b), s0, s1, send[guard:])
    torch.cuda.synchronize()
    opool_b = init_b.copy()
    oracle.unpack(opool_b, pool_a.shape, 1, L, table_b, s0, s1, ref)
    assert np.array_equal(bits(pool_b.t), opool_b)


def test_pack_unpack_batch_bytes():
    """One launch for several sequences gives, for each, the bytes of the single-sequence call."""
    L, Hkv = 3, 8
    lens = [300, 16, 77, 1, 130]
    s0 = [0, 3, 16, 0, 129]
    s1 = [300, 16, 70, 1, 130]
    w = small_workload(105, mi.BF16, Hkv, Hkv, lens, [0] * 5, layers=L)
    init = canary(8, DevPool(w).elems)
    pool_a = DevPool(w, fill=init)
    B = len(lens)
    sizes = [(L - 1) * 2 * (s1[i] - s0[i]) * Hkv * 128 for i in range(B)]     # elements
    guard = 64
    offs, at = [], guard
    for n in sizes:
        offs.append(at)
        at += n + guard                      # guard elements between and around the slices
    raw = canary(9, at)
    send = dev(raw)
    db = DevBatch(w)
    d_s0, d_s1 = dev(np.array(s0, np.int32)), dev(np.array(s1, np.int32))
    d_off = torch.tensor([2 * o for o in offs], dtype=torch.int64, device=DEV)   # bytes
    max_pages = max((b - 1) // 16 - a // 16 + 1 for a, b in zip(s0, s1))
    mc.mc_kv_pack_batch(pool_a.desc, 1, L, B, db.page_table, db.cu_pages, d_s0, d_s1, d_off,
                        max_pages, send)
    torch.cuda.synchronize()
    got = bits(send)
    expect = raw.copy()
    refs = []
    for i in range(B):
        ref = oracle.pack(init, pool_a.shape, 1, L, w.page_tables[i], s0[i], s1[i])
        refs.append(ref)
        expect[offs[i]:offs[i] + sizes[i]] = ref.ravel()
    assert np.array_equal(got, expect)                  # slices and every guard byte
    assert np.array_equal(bits(pool_a.t), init)
    # receiver: other tables, same launch shape
    init_b = canary(10, pool_a.elems)
    pool_b = DevPool(w, fill=init_b)
    tables_b = mi.scatter_page_tables(mi.rng_for(11), w.num_pages, w.n)
    wb = mi.Workload("b", w.seed, w.dtype, L, Hkv, Hkv, w.num_pages, w.n, w.b, tables_b)
    dbb = DevBatch(wb)
    mc.mc_kv_unpack_batch(pool_b.desc, 1, L, B, dbb.page_table, dbb.cu_pages, d_s0, d_s1, d_off,
                          max_pages, send)
    torch.cuda.synchronize()
    opool_b = init_b.copy()
    for i in range(B):
        oracle.unpack(opool_b, pool_a.shape, 1, L, tables_b[i], s0[i], s1[i], refs[i])
    assert np.array_equal(bits(pool_b.t), opool_b)
    # a malformed sequence (reversed range) is skipped, the others still move
    send2 = dev(raw)
    bad_s1 = dev(np.array([300, 2, 70, 1, 130], np.int32))      # sequence 1: s1 < s0
    mc.mc_kv_pack_batch(pool_a.desc, 1, L, B, db.page_table, db.cu_pages, d_s0, bad_s1, d_off,
                        max_pages, send2)
    torch.cuda.synchronize()
    expect2 = expect.copy()
    expect2[offs[1]:offs[1] + sizes[1]] = raw[offs[1]:offs[1] + sizes[1]]
    assert np.array_equal(bits(send2), expect2)


def test_transfer_then_attend_equals_local_attention():
    """KV sent to a second pool is attended there exactly as at home (Sec. 3.4)."""
    w = small_workload(104, mi.BF16, 32, 8, [200], [150], num_pages=40)
    pool_a, opool = DevPool(w), None
    opool = oracle.new_pool(pool_a.shape)
    fill_both(w, pool_a, opool)
    table = w.page_tables[0]
    send = torch.zeros(2 * 200 * 8 * 128, dtype=torch.int16, device=DEV)
    mc.mc_kv_pack_range(pool_a.desc, 0, 1, dev(table), len(table), 0, 200, send)
    pool_b = DevPool(w)
    table_b = mi.rng_for(7).permutation(40)[: len(table)].astype(np.int32)
    mc.mc_kv_unpack_range(pool_b.desc, 0, 1, dev(table_b), len(table_b), 0, 200, send)
    wb = mi.Workload("b", w.seed, w.dtype, 1, 32, 8, 40, w.n, w.b, [table_b])
    q = w.q(0)
    oa, la = gpu_attention(pool_a, 0, dev(q), DevBatch(w))
    ob, lb = gpu_attention(pool_b, 0, dev(q), DevBatch(wb))
    assert torch.equal(oa, ob) and torch.equal(la, lb)


# ---------------------------------------------------------------- attention ----
def peaked_o_tol(w, layer=0):
    """Bar for data whose softmax can put all its weight on one key (scores many units wide):
    O then is one V row times a weight that entered the P.V product rounded to 2 bytes, and is
    itself rounded to 2 bytes on the way out - two relative errors of one unit roundoff u each
    (2^-8 for bf16, 2^-11 for fp16), so |error| <= 2 u max|V|.  On scores a few units wide, as
    in every named config, a row averages many keys and the absolute bar O_TOL holds."""
    vmax = max(float(np.max(np.abs(oracle.decode(w.kv(s, layer)[1], w.dtype))))
               for s in range(w.batch))
    u = 2.0 ** -8 if w.dtype == mi.BF16 else 2.0 ** -11
    return max(O_TOL, 2 * u * vmax)


def check_attention(w, layer=0, scale=None, sample=None, seed=0, o_tol=O_TOL):
    # every slot that is never appended holds NaN bit patterns: unwritten slots of a
    # sequence's last page and foreign pages must not leak into the result
    pool = DevPool(w)
    pool.t.fill_(0x7fc1)
    opool = np.full(pool.elems, 0x7fc1, dtype=np.uint16)
    fill_both(w, pool, opool, layers=(layer,))
    db = DevBatch(w)
    qs = [w.q(s, layer) for s in range(w.batch)]
    out, lse = gpu_attention(pool, layer, dev(np.concatenate(qs)), db,
                             sm_scale=0.0 if scale is None else scale)
    out_b, lse_h = bits(out), lse.cpu().numpy().astype(np.float64)
    worst_o = worst_l = 0.0
    for s in range(w.batch):
        q_len = int(w.n[s] - w.b[s])
        if q_len == 0:
            continue
        lo = int(w.cu_q[s])
        go = oracle.decode(out_b[lo:lo + q_len], w.dtype)
        gl = lse_h[lo:lo + q_len]
        if sample is None:
            ro, rl = oracle_rows(w, opool, pool.shape, layer, s, qs[s], scale=scale)
        else:
            rows, heads = mi.sample_rows(mi.rng_for(seed, s, 5), q_len, int(w.b[s]),
                                         w.num_q_heads, sample,
                                         tile_tokens=128 // (w.num_q_heads // w.num_kv_heads),
                                         num_kv_heads=w.num_kv_heads)
            ro, rl = oracle_rows(w, opool, pool.shape, layer, s, qs[s], rows, heads, scale=scale)
            go, gl = go[rows, heads], gl[rows, heads]
        assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
        worst_o = max(worst_o, float(np.max(np.abs(go - ro))))
        worst_l = max(worst_l, float(np.max(np.abs(gl - rl))))
    assert worst_o <= o_tol, worst_o
    assert worst_l <= LSE_TOL, worst_l
    return worst_o, worst_l


@pytest.mark.parametrize("dtype", [mi.F16, mi.BF16])
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (4, 2), (32, 8), (16, 2)])
def test_attention_small_all_rows(dtype, Hq, Hkv):
    # several q tiles and KV tiles, ragged tails, unaligned prefixes, one-token and
    # no-prefix sequences, and a sequence with nothing new
    lens = [333, 64, 130, 1, 257, 90]
    begins = [77, 0, 129, 0, 256, 90]
    w = small_workload(200 + Hq, dtype, Hq, Hkv, lens, begins)
    check_attention(w)


def test_attention_custom_scale_and_layer():
    w = small_workload(210, mi.BF16, 32, 8, [150, 40], [31, 8], layers=3)
    check_attention(w, layer=2, scale=0.05)


def test_attention_writes_only_its_rows():
    w = small_workload(211, mi.BF16, 32, 8, [100, 0 + 50], [40, 50])   # second sequence: nothing new
    pool = DevPool(w)
    opool = oracle.new_pool(pool.shape)
    fill_both(w, pool, opool)
    db = DevBatch(w)
    out, lse = gpu_attention(pool, 0, dev(w.q(0)), db)
    assert out.shape[0] == 60 and torch.isfinite(lse).all()


def test_plan_reports_bad_tables():
    w = small_workload(212, mi.BF16, 32, 8, [100], [40])
    pool = DevPool(w)
    db = DevBatch(w)
    ws_bytes = mc.mc_attn_workspace_size(1, 60, 32, 8)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV)
    bad = db.page_table.clone()
    bad[3] = w.num_pages            # page id outside the pool
    mc.mc_attn_plan(pool.desc, 32, 1, 60, db.cu_q, db.begin, bad, db.cu_pages, ws, ws_bytes)
    with pytest.raises(mc.McError) as e:
        mc.mc_attn_plan_check(ws)
    assert e.value.status == mc.MC_ERR_RANGE
    short = dev(np.array([0, 3], dtype=np.int32))   # 3 pages cannot hold 100 tokens
    mc.mc_attn_plan(pool.desc, 32, 1, 60, db.cu_q, db.begin, db.page_table, short, ws, ws_bytes)
    with pytest.raises(mc.McError):
        mc.mc_attn_plan_check(ws)
    # attention over the failed plan launches but writes nothing
    out = torch.full((60, 32, 128), 0x7fc1, dtype=torch.int16, device=DEV)
    lse = torch.full((60, 32), -7.0, dtype=torch.float32, device=DEV)
    mc.mc_prefix_prefill_attn(pool.desc, 0, dev(w.q(0)), 32, 1, 60, db.cu_q, db.begin,
                              db.page_table, short, 0.0, out, lse, ws, ws_bytes)
    torch.cuda.synchronize()
    assert (lse == -7.0).all() and (out == 0x7fc1).all()


def test_split_range_equals_single_pass_on_gpu():
    """Pass A over [0,m) then pass B over [m,n) against the cached [0,m) reproduces the
    single [0,n) pass row for row (Sec. 3.3)."""
    n = [300, 170]
    m = [150, 85]
    w_full = small_workload(213, mi.BF16, 32, 8, n, [0, 0])
    pool = DevPool(w_full)
    opool = oracle.new_pool(pool.shape)
    fill_both(w_full, pool, opool)
    q_full = [w_full.q(s) for s in range(2)]
    o_full, l_full = gpu_attention(pool, 0, dev(np.concatenate(q_full)), DevBatch(w_full))
    w_a = w_full.with_ranges([0, 0], m)
    w_b = w_full.with_ranges(m, n)
    o_a, l_a = gpu_attention(pool, 0, dev(np.concatenate([q_full[s][: m[s]] for s in range(2)])),
                             DevBatch(w_a))
    o_b, l_b = gpu_attention(pool, 0, dev(np.concatenate([q_full[s][m[s]:] for s in range(2)])),
                             DevBatch(w_b))
    f = lambda t: oracle.decode(bits(t), mi.BF16)
    full, la_full = f(o_full), l_full.cpu().numpy()
    parts = np.concatenate([f(o_a)[:150], f(o_b)[:150], f(o_a)[150:], f(o_b)[150:]])
    lparts = np.concatenate([l_a.cpu().numpy()[:150], l_b.cpu().numpy()[:150],
                             l_a.cpu().numpy()[150:], l_b.cpu().numpy()[150:]])
    # different tilings of the same rows: equal within the tolerance, not bit-wise
    assert np.max(np.abs(parts - full)) <= O_TOL
    assert np.max(np.abs(lparts - la_full)) <= LSE_TOL


# ------------------------------------------------------- the five configs ----
def test_config1_full():
    w = mi.config(1)
    check_attention(w)


def test_config2_full():
    check_attention(mi.config(2))          # every row and q head: 0.27 TFLOP of fp64 on the host


def test_config4_full():
    check_attention(mi.config(4))          # every row and q head: 0.84 TFLOP of fp64 on the host


def test_paper_shaped_points():
    for cached in (500, 2500, 4500):
        check_attention(mi.paper_point(cached))


# ------------------------------------------------- cut KV ranges (decode rows, short batches) ----
def plan_header(w):
    pool = DevPool(w)
    db = DevBatch(w)
    ws_bytes = mc.mc_attn_workspace_size(db.batch, db.total_q, w.num_q_heads, w.num_kv_heads)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan(pool.desc, w.num_q_heads, db.batch, db.total_q, db.cu_q, db.begin,
                    db.page_table, db.cu_pages, ws, ws_bytes)
    mc.mc_attn_plan_check(ws)
    h = ws[:64].view(torch.int32).cpu().numpy()
    return {"num_items": int(h[2]), "tile_tokens": int(h[3]), "num_merges": int(h[6]),
            "chunk_tiles": int(h[7]), "num_groups_rows": int(h[8])}


@pytest.mark.parametrize("Hq,Hkv,dtype", [(32, 8, mi.BF16), (8, 8, mi.F16), (64, 8, mi.BF16)])
def test_decode_rows_fused_with_prefill(Hq, Hkv, dtype):
    # decode steps (one new token over contexts of 1..5000 tokens) in one ragged batch with two
    # prefill ranges and an idle sequence (Sec. 3.3: the prefill of the rest of a prompt runs
    # fused with decode).  Too few q tiles to fill the GPU: the planner cuts the long contexts
    # into chunks and the chunks' partial results are merged by their LSE.
    lens = [1, 17, 64, 65, 1000, 2047, 2049, 5000, 1500, 700, 90]
    begins = [0, 16, 63, 64, 999, 2046, 2048, 4999, 300, 0, 90]
    w = small_workload(300 + Hq, dtype, Hq, Hkv, lens, begins)
    h = plan_header(w)
    assert h["chunk_tiles"] >= 8 and h["chunk_tiles"] % 2 == 0 and h["num_merges"] > 0, h
    check_attention(w)


def test_pure_decode_batch():
    rng = mi.rng_for(321)
    lens = [int(x) for x in rng.integers(1, 4097, size=48)]
    w = small_workload(322, mi.BF16, 32, 8, lens, [n - 1 for n in lens])
    h = plan_header(w)
    assert h["num_merges"] > 0 and h["num_items"] > 48, h
    check_attention(w)


def test_large_batch_is_not_cut():
    h = plan_header(mi.config(2))
    assert h["chunk_tiles"] == 0 and h["num_merges"] == 0 and h["num_items"] >= 300, h


@pytest.mark.parametrize("dtype,Hq,Hkv", [(mi.BF16, 32, 8), (mi.F16, 32, 8), (mi.BF16, 64, 8),
                                          (mi.BF16, 16, 8), (mi.F16, 8, 8)])
def test_wide_q_tiles_on_long_contexts(dtype, Hq, Hkv):
    """Long new ranges over long cached prefixes: the planner takes q tiles of 256 rows (the
    kernel variant with two row blocks per wavefront).  Unaligned begins and lengths, a ragged
    last tile; a sample spread over both sequences against the oracle."""
    G = Hq // Hkv
    lens, begins = {1: ([42013], [9005]), 2: ([26511], [10003]), 4: ([17013, 13107], [12001, 9007]),
                    8: ([14113], [10007])}[G]
    w = small_workload(790 + Hq + dtype, dtype, Hq, Hkv, lens, begins)
    h = plan_header(w)
    assert h["tile_tokens"] == 256 // G and h["num_merges"] == 0, h
    check_attention(w, sample=4096, seed=79)


def test_wide_q_tiles_fall_back_on_overflowing_scores():
    # scaled scores ~ N(0, 60^2) on the wide-tile kernel: rows whose later keys beat the first
    # half tile's best by more than 2^60 send their workgroup through the moving-reference pass
    w = small_workload(795, mi.BF16, 64, 8, [14113], [10007])
    _scaled_kv(w, k_gain=60.0)
    assert plan_header(w)["tile_tokens"] == 32
    check_attention(w, sample=2048, seed=80, o_tol=peaked_o_tol(w))


def test_short_range_over_long_context_is_cut():
    w = mi.paper_point(4500)
    h = plan_header(w)
    assert h["num_merges"] > 0, h
    check_attention(w, sample=256, seed=9)


# ------------------------------------------------------------- shared prefixes ----
def forked_decode_workload(seed, Hq, Hkv, dtype, groups, extra=()):
    """groups: lists of (total tokens, tokens shared with the group's first sequence); every
    sequence is a decode step (one new token).  extra: (n, b) of other sequences placed between
    the groups (they break the neighbourhood)."""
    lens, begins, forks = [], [], []
    for gi, g in enumerate(groups):
        first = len(lens)
        for n, shared in g:
            if len(lens) > first:
                forks.append((len(lens), first, shared))
            lens.append(n)
            begins.append(n - 1)
        if gi < len(extra):
            lens.append(extra[gi][0])
            begins.append(extra[gi][1])
    w = small_workload(seed, dtype, Hq, Hkv, lens, begins)
    for s, src, shared in forks:
        w.share_prefix(s, src, shared)
    return w


@pytest.mark.parametrize("Hq,Hkv,dtype", [(32, 8, mi.BF16), (8, 8, mi.F16)])
def test_decode_rows_sharing_a_prefix(Hq, Hkv, dtype):
    # forks of a common prompt (Sec. 3.5 fork_sequence): their page tables start with the same
    # pages.  Neighbouring decode rows attend the shared prefix together and their own
    # remainders alone; results must equal plain per-sequence attention.
    groups = [
        [(1100, 0), (1500, 1024), (3000, 1024), (1040, 1024), (2000, 1024)],   # 64 shared pages
        [(900, 0), (700, 592), (1300, 592)],                                   # 37 shared pages
        [(800, 0), (900, 160)],                                                # too few: no group
    ]
    w = forked_decode_workload(400 + Hq, Hq, Hkv, dtype, groups, extra=[(700, 300), (90, 90)])
    pool = DevPool(w)
    db = DevBatch(w)
    ws_bytes = mc.mc_attn_workspace_size(db.batch, db.total_q, w.num_q_heads, w.num_kv_heads)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan(pool.desc, w.num_q_heads, db.batch, db.total_q, db.cu_q, db.begin,
                    db.page_table, db.cu_pages, ws, ws_bytes)
    mc.mc_attn_plan_check(ws)
    h = ws[:64].view(torch.int32).cpu().numpy()
    assert int(h[8]) > 0, h[:9]          # shared-prefix items were planned
    check_attention(w)


@pytest.mark.parametrize("dtype", [mi.BF16, mi.F16])
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (32, 8), (64, 8)])
def test_short_ranges_sharing_a_prefix(dtype, Hq, Hkv):
    """Forks of one 2048-token prompt that each bring a few new tokens (3..40), after own middle
    parts of different lengths: those whose new tokens fit a q tile together attend the shared
    prefix as one tile; an unrelated sequence in between ends a run.  Every row vs the oracle."""
    rng = mi.rng_for(760 + Hq)
    new = [int(x) for x in rng.integers(3, 15, size=9)]
    new[7] = 40                                        # too long for a shared tile of 32 tokens
    own = [int(x) for x in rng.integers(0, 200, size=9)]
    begins = [2048 + o for o in own]
    begins[4] = 700                                    # sequence 4 is not a fork
    lens = [b + q for b, q in zip(begins, new)]
    w = small_workload(761, dtype, Hq, Hkv, lens, begins)
    for s in range(1, 9):
        if s != 4:
            w.share_prefix(s, 0, 2048)
    h = plan_header(w)
    if 128 // (Hq // Hkv) > 16:                        # tiles of 16 tokens hold few of these ranges
        assert h["num_groups_rows"] > 0, h
    check_attention(w)


def test_more_forks_than_a_tile_holds():
    # 40 forks of one 2048-token prompt with G = 4 (32 tokens a tile): two groups
    groups = [[(2100 + 7 * i, 0 if i == 0 else 2048) for i in range(40)]]
    w = forked_decode_workload(450, 32, 8, mi.BF16, groups)
    check_attention(w)


def test_batch_larger_than_the_planner_keeps_in_lds():
    # 1500 sequences (the planner keeps per-sequence offsets in LDS up to 1024): decode rows and
    # short prefill ranges over short contexts
    rng = mi.rng_for(460)
    lens = [int(x) for x in rng.integers(1, 41, size=1500)]
    begins = [n - 1 if i % 3 else int(rng.integers(0, n)) for i, n in enumerate(lens)]
    w = small_workload(461, mi.BF16, 32, 8, lens, begins)
    check_attention(w)


# ------------------------------------------------------------------ HIP graph ----
def test_decode_step_under_graph_capture():
    """append + plan + attention (+ merge) of a decode step captured in a HIP graph: the calls
    allocate nothing and never synchronise, so they can be captured; every replay, with fresh
    Q/K/V in the same buffers, must give what the eager calls give."""
    lens = [1500, 700, 2300, 64, 65, 3000, 999, 1200]
    w = small_workload(470, mi.BF16, 32, 8, lens, [n - 1 for n in lens])
    pool = DevPool(w)
    opool = oracle.new_pool(pool.shape)
    fill_both(w, pool, opool, upto_end=False)          # the cached prefixes
    db = DevBatch(w)
    Hq, Hkv = w.num_q_heads, w.num_kv_heads
    ws_bytes = mc.mc_attn_workspace_size(db.batch, db.total_q, Hq, Hkv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    q = torch.zeros((db.total_q, Hq, 128), dtype=torch.int16, device=DEV)
    k = torch.zeros((db.total_q, Hkv, 128), dtype=torch.int16, device=DEV)
    v = torch.zeros((db.total_q, Hkv, 128), dtype=torch.int16, device=DEV)
    out = torch.zeros((db.total_q, Hq, 128), dtype=torch.int16, device=DEV)
    lse = torch.zeros((db.total_q, Hq), dtype=torch.float32, device=DEV)

    def step():
        mc.mc_kv_append(pool.desc, 0, k, v, db.batch, db.total_q, db.cu_q, db.begin,
                        db.page_table, db.cu_pages)
        mc.mc_attn_plan(pool.desc, Hq, db.batch, db.total_q, db.cu_q, db.begin, db.page_table,
                        db.cu_pages, ws, ws_bytes)
        mc.mc_prefix_prefill_attn(pool.desc, 0, q, Hq, db.batch, db.total_q, db.cu_q, db.begin,
                                  db.page_table, db.cu_pages, 0.0, out, lse, ws, ws_bytes)

    def fresh(seed):
        g = torch.Generator(device=DEV).manual_seed(seed)
        for t in (q, k, v):
            t.copy_(torch.randn(t.shape, generator=g, device=DEV).to(torch.bfloat16).view(torch.int16))

    fresh(1)
    step()                                   # eager once (also warms the library up)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for seed in (2, 3, 4):
        fresh(seed)
        graph.replay()
        torch.cuda.synchronize()
        got_o, got_l = out.clone(), lse.clone()
        out.zero_()
        lse.zero_()
        step()                               # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(got_o, out) and torch.equal(got_l, lse), seed
    assert torch.isfinite(lse).all()


# ------------------------------------------------- the calls together: one prompt, two engines ----
@pytest.mark.parametrize("sender_cached,receiver_cached", [(192, 64), (64, 192), (0, 0), (384, 0),
                                                           (128, 128)])
def test_remote_send_flow_for_the_prefix_matching_cases(sender_cached, receiver_cached):
    """prep_recv on the receiver, remote_send on the sender (copy what is cached, prefill the
    rest, send what the receiver lacks), start_generate on the receiver (Sec. 3.1, Sec. 3.2,
    Sec. 3.5 cases 1 and 2): afterwards the receiver holds exactly the prompt's KV and its
    last-token attention equals the oracle's."""
    Hq, Hkv, n, pages_total = 32, 8, 400, 64
    end = n - 1                                             # the receiver prefills the last token
    w = small_workload(500 + sender_cached + receiver_cached, mi.BF16, Hq, Hkv, [n], [0],
                       num_pages=pages_total)
    prompt = [int(x) for x in mi.rng_for(w.seed, 42).integers(0, 32000, size=n)]
    k_all, v_all = w.kv(0)

    def engine(cached):
        """An engine that already served prompt[:cached]: pool, allocator, index, that KV."""
        pool = DevPool(w)
        pool.t.fill_(0x7fc1)
        al, ix = mc.mc_kv_allocator_create(pages_total), mc.mc_prefix_index_create()
        mc.mc_kv_alloc_pages(al, 3)                         # the engines' page ids differ
        if cached:
            pages, m = mc.mc_prep_recv(ix, al, prompt, cached)
            assert m == 0
            wc = mi.Workload("c", w.seed, w.dtype, 1, Hq, Hkv, pages_total, np.array([cached]),
                             np.array([0]), [np.array(pages, dtype=np.int32)])
            gpu_append(pool, 0, dev(k_all[:cached]), dev(v_all[:cached]), DevBatch(wc))
            mc.mc_prefix_index_insert(ix, prompt[:cached], pages)
        return pool, al, ix

    pool_a, al_a, ix_a = engine(sender_cached)
    pool_b, al_b, ix_b = engine(receiver_cached)
    # receiver: prep_recv(prompt, end) -> where to send, and how much it already has
    pages_b, match_b = mc.mc_prep_recv(ix_b, al_b, prompt, end)
    assert match_b == receiver_cached
    # sender: remote_send(prompt, kv_addr_info, begin = 0, end)
    pages_a, match_a = mc.mc_prep_recv(ix_a, al_a, prompt, end)
    assert match_a == sender_cached
    plan = mc.mc_plan_remote_send(match_a, match_b, 0, end)
    tab_a, tab_b = np.array(pages_a, dtype=np.int32), np.array(pages_b, dtype=np.int32)
    # the compressed address list travels and comes back unchanged
    assert mc.mc_addr_expand(mc.mc_addr_compress(pages_b)) == pages_b
    p0, p1 = plan["prefill"]
    if p1 > p0:                                             # KV of what the sender lacks
        wp = mi.Workload("p", w.seed, w.dtype, 1, Hq, Hkv, pages_total, np.array([p1]),
                         np.array([p0]), [tab_a])
        gpu_append(pool_a, 0, dev(k_all[p0:p1]), dev(v_all[p0:p1]), DevBatch(wp))
        out_p, lse_p = gpu_attention(pool_a, 0, dev(w.q(0)[p0:p1]), DevBatch(wp))
        assert torch.isfinite(lse_p).all()
    for s0, s1 in (plan["copy"], plan["send"]):             # pack -> wire -> unpack
        if s1 > s0:
            buf = torch.zeros(2 * (s1 - s0) * Hkv * 128, dtype=torch.int16, device=DEV)
            mc.mc_kv_pack_range(pool_a.desc, 0, 1, dev(tab_a), len(tab_a), s0, s1, buf)
            mc.mc_kv_unpack_range(pool_b.desc, 0, 1, dev(tab_b), len(tab_b), s0, s1, buf)
    # the receiver now holds prompt[0, end): packed out of its pool it is the prompt's KV, bit for bit
    got = torch.zeros(2 * end * Hkv * 128, dtype=torch.int16, device=DEV)
    mc.mc_kv_pack_range(pool_b.desc, 0, 1, dev(tab_b), len(tab_b), 0, end, got)
    want = np.concatenate([k_all[:end].reshape(-1), v_all[:end].reshape(-1)])
    assert np.array_equal(bits(got), want)
    # receiver: start_generate(prompt, begin = end): the last token over everything before it
    wl = mi.Workload("l", w.seed, w.dtype, 1, Hq, Hkv, pages_total, np.array([n]), np.array([end]),
                     [tab_b])
    gpu_append(pool_b, 0, dev(k_all[end:n]), dev(v_all[end:n]), DevBatch(wl))
    out, lse = gpu_attention(pool_b, 0, dev(w.q(0)[end:n]), DevBatch(wl))
    # oracle: the same sequence in a pool of its own
    wo = mi.Workload("o", w.seed, w.dtype, 1, Hq, Hkv, pages_total, np.array([n]), np.array([end]),
                     [w.page_tables[0]])
    opool = oracle.new_pool(pool_b.shape)
    oracle.append(opool, pool_b.shape, 0, k_all, v_all, 0, w.page_tables[0])
    ro, rl = oracle_rows(wo, opool, pool_b.shape, 0, 0, w.q(0)[end:n])
    assert np.max(np.abs(oracle.decode(bits(out), w.dtype) - ro)) <= O_TOL
    assert np.max(np.abs(lse.cpu().numpy().astype(np.float64) - rl)) <= LSE_TOL
    for h in (ix_a, ix_b):
        mc.mc_prefix_index_destroy(h)
    for h in (al_a, al_b):
        mc.mc_kv_allocator_destroy(h)


# ------------------------------------------------------- value distributions ----
def _scaled_kv(w, k_gain=None, v_gain=1.0, ramp=0.0, const_k=False):
    """Replace the workload's K/V by a transformed copy: K x k_gain (wide score range), K plus
    a ramp along the token axis in the direction of a fixed vector (scores that keep rising, so
    the running max moves tile after tile), K constant (uniform softmax), V x v_gain."""
    base = w.kv
    dt = w.dtype

    def kv(seq, layer=0):
        k, v = base(seq, layer)
        kf = oracle.decode(k, dt)
        vf = oracle.decode(v, dt) * v_gain
        if const_k:
            kf = np.broadcast_to(kf[:1], kf.shape).copy()
        if k_gain is not None:
            kf = kf * k_gain
        if ramp:
            kf = kf + ramp * np.arange(kf.shape[0])[:, None, None] * np.sign(kf[:1])
        return (mi.f32_to_bits(kf.astype(np.float32), dt), mi.f32_to_bits(vf.astype(np.float32), dt))
    w.kv = kv
    return w


@pytest.mark.parametrize("kind", ["wide", "rising", "uniform", "big_v", "huge"])
@pytest.mark.parametrize("dtype", [mi.BF16, mi.F16])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (8, 8), (16, 2)])
def test_attention_value_distributions(kind, dtype, Hq, Hkv):
    lens, begins = [700, 333, 1], [130, 0, 0]
    w = small_workload(600 + len(kind) + Hq, dtype, Hq, Hkv, lens, begins)
    if kind == "wide":        # scaled scores ~ N(0, 6^2): exp2 range of dozens between keys
        _scaled_kv(w, k_gain=6.0)
    elif kind == "rising":    # every tile's max exceeds the last one's: the reference max keeps moving
        _scaled_kv(w, ramp=0.02)
    elif kind == "uniform":   # all keys equal: softmax is uniform, LSE = s + ln(i + 1)
        _scaled_kv(w, const_k=True)
    elif kind == "huge":      # scaled scores ~ N(0, 60^2): later keys beat the first tile's best by
        _scaled_kv(w, k_gain=60.0)   # more than 2^60, so a reference fixed there cannot serve
    else:                     # V x 3: the output and its 2-byte rounding scale with V, so does the bar
        _scaled_kv(w, v_gain=3.0)
    peaked = kind in ("wide", "huge", "big_v")
    check_attention(w, o_tol=peaked_o_tol(w) if peaked else O_TOL)


@pytest.mark.parametrize("dtype", [mi.BF16, mi.F16])
def test_wide_scores_through_chunks_and_merge(dtype):
    # decode rows and a short range over long contexts (the planner cuts them into chunks) with
    # scores spanning dozens of powers of two: chunk LSEs far apart, weights down to exactly 0
    lens = [2500, 1800, 3000, 900]
    begins = [2499, 1799, 2900, 899]
    w = small_workload(640, dtype, 32, 8, lens, begins)
    _scaled_kv(w, k_gain=6.0)
    assert plan_header(w)["num_merges"] > 0
    check_attention(w, o_tol=peaked_o_tol(w))


def test_decode_over_a_128k_context():
    # one new token over 131071 cached ones (2048 KV tiles, cut into many chunks) next to a short
    # sequence: large tile indices, many partial rows per token
    n = 131072
    w = small_workload(650, mi.BF16, 32, 8, [n, 40], [n - 1, 39])
    h = plan_header(w)
    assert h["num_merges"] >= 1 and h["num_items"] > 8, h
    check_attention(w)


def test_append_send_writes_pool_and_marked_rows():
    """mark_send: the append of the new range also writes the marked tokens to the transfer
    buffer, byte for byte what pack writes for them after a plain append, and nothing else."""
    L, Hkv = 3, 8
    lens = [300, 64, 77, 130, 40]
    begins = [100, 0, 20, 129, 40]            # the last sequence has nothing new
    s0 = [100, 5, 30, 129, 0]                 # whole new range / inside it / inside / one token / nothing new
    s1 = [300, 60, 70, 130, 40]
    s0[2], s1[2] = 10, 77                     # starts below begin: rows of [10, 20) stay untouched
    w = small_workload(700, mi.BF16, Hkv, Hkv, lens, begins, layers=L)
    init = canary(20, DevPool(w).elems)
    pool, ref_pool = DevPool(w, fill=init), DevPool(w, fill=init)
    opool = init.copy()
    B = len(lens)
    first_layer = 1                           # the buffer holds layers 1 and 2
    sizes = [(L - first_layer) * 2 * (s1[i] - s0[i]) * Hkv * 128 for i in range(B)]
    guard, offs, at = 64, [], 64
    for n in sizes:
        offs.append(at)
        at += n + guard
    raw = canary(21, at)
    send = dev(raw)
    db = DevBatch(w)
    d_s0, d_s1 = dev(np.array(s0, np.int32)), dev(np.array(s1, np.int32))
    d_off = torch.tensor([2 * o for o in offs], dtype=torch.int64, device=DEV)
    for layer in range(L):
        ks = np.concatenate([w.kv(s, layer)[0][begins[s]:lens[s]] for s in range(B)])
        vs = np.concatenate([w.kv(s, layer)[1][begins[s]:lens[s]] for s in range(B)])
        if layer >= first_layer:
            mc.mc_kv_append_send(pool.desc, layer, dev(ks), dev(vs), db.batch, db.total_q, db.cu_q,
                                 db.begin, db.page_table, db.cu_pages, first_layer, d_s0, d_s1,
                                 d_off, send)
        else:
            gpu_append(pool, layer, dev(ks), dev(vs), db)
        gpu_append(ref_pool, layer, dev(ks), dev(vs), db)
        for s in range(B):
            if lens[s] > begins[s]:
                k, v = w.kv(s, layer)
                oracle.append(opool, pool.shape, layer, k[begins[s]:lens[s]], v[begins[s]:lens[s]],
                              begins[s], w.page_tables[s])
    torch.cuda.synchronize()
    assert np.array_equal(bits(pool.t), opool)               # the pool: exactly a plain append
    assert np.array_equal(bits(ref_pool.t), opool)
    expect = raw.copy()
    for i in range(B):
        if s1[i] <= s0[i]:
            continue
        full = oracle.pack(opool, pool.shape, first_layer, L, w.page_tables[i], s0[i], s1[i])
        lo = max(begins[i], s0[i]) - s0[i]                   # rows of tokens below begin are not new
        hi = min(lens[i], s1[i]) - s0[i]
        cur = expect[offs[i]:offs[i] + sizes[i]].reshape(full.shape).copy()
        cur[:, :, lo:hi] = full[:, :, lo:hi]
        expect[offs[i]:offs[i] + sizes[i]] = cur.ravel()
    assert np.array_equal(bits(send), expect)                # marked rows, holes and guards


def test_fork_sequence_copies_the_partial_page_and_forks_diverge():
    """fork_sequence (Sec. 3.5): the child shares the parent's whole pages and gets a copy of the
    partly filled one; both then append their own next token and attend: each sees the common
    100 tokens and only its own new one."""
    Hq, Hkv, L, n = 32, 8, 2, 100
    w = small_workload(710, mi.BF16, Hq, Hkv, [n + 1, n + 1], [n, n], num_pages=32, layers=L)
    init = canary(30, DevPool(w).elems)
    pool = DevPool(w, fill=init)
    opool = init.copy()
    al = mc.mc_kv_allocator_create(32)
    parent = mc.mc_kv_alloc_pages(al, 7)                      # 100 tokens: 6 whole pages + 4 slots
    kp = [w.kv(0, l) for l in range(L)]
    wp = mi.Workload("p", w.seed, w.dtype, L, Hq, Hkv, 32, np.array([n]), np.array([0]),
                     [np.array(parent, np.int32)])
    for l in range(L):
        gpu_append(pool, l, dev(kp[l][0][:n]), dev(kp[l][1][:n]), DevBatch(wp))
        oracle.append(opool, pool.shape, l, kp[l][0][:n], kp[l][1][:n], 0, parent)
    child, (src, dst, slots) = mc.mc_kv_fork_sequence(al, parent, n)
    assert child[:6] == parent[:6] and (src, slots) == (parent[6], 4) and dst == child[6]
    mc.mc_kv_copy_page(pool.desc, 0, L, src, dst, slots)
    oracle.copy_page(opool, pool.shape, 0, L, src, dst, slots)
    torch.cuda.synchronize()
    assert np.array_equal(bits(pool.t), opool)                # the copy and nothing else
    # both sequences append their own token 100 and attend it
    wf = mi.Workload("f", w.seed, w.dtype, L, Hq, Hkv, 32, np.array([n + 1, n + 1]),
                     np.array([n, n]), [np.array(parent, np.int32), np.array(child, np.int32)])
    kc = [w.kv(1, l) for l in range(L)]
    db = DevBatch(wf)
    for l in range(L):
        k_new = np.concatenate([kp[l][0][n:n + 1], kc[l][0][n:n + 1]])
        v_new = np.concatenate([kp[l][1][n:n + 1], kc[l][1][n:n + 1]])
        gpu_append(pool, l, dev(k_new), dev(v_new), db)
        oracle.append(opool, pool.shape, l, kp[l][0][n:n + 1], kp[l][1][n:n + 1], n, parent)
        oracle.append(opool, pool.shape, l, kc[l][0][n:n + 1], kc[l][1][n:n + 1], n, child)
    torch.cuda.synchronize()
    assert np.array_equal(bits(pool.t), opool)
    for l in range(L):
        q = np.concatenate([w.q(0, l), w.q(1, l)])
        out, lse = gpu_attention(pool, l, dev(q), db)
        for s, tab in enumerate((parent, child)):
            ro, rl = oracle.attention(opool, pool.shape, l, np.array(tab, np.int32), q[s:s + 1],
                                      Hq, n, n + 1)
            assert np.max(np.abs(oracle.decode(bits(out[s:s + 1]), w.dtype) - ro)) <= O_TOL
            assert np.max(np.abs(lse[s:s + 1].cpu().numpy() - rl)) <= LSE_TOL
    # the child's last page holds the parent's first 4 slots and its own fifth
    view = opool.reshape(pool.shape.pool_dims())
    assert np.array_equal(view[:, child[6], :, :, :4], view[:, parent[6], :, :, :4])
    assert not np.array_equal(view[:, child[6], :, :, 4], view[:, parent[6], :, :, 4])
    mc.mc_kv_allocator_destroy(al)


def test_one_plan_for_many_decode_steps():
    """mc_attn_plan_ahead: a plan made once serves decode step after decode step while the
    sequences grow (begin is read again by every attention call), up to the number of tokens it
    was made for; the page tables already list the pages of the tokens to come."""
    steps, Hq, Hkv = 70, 32, 8
    start = [1000, 63, 1, 2047, 500]                      # lengths before the first step
    final = [n + steps for n in start]
    w_full = small_workload(720, mi.BF16, Hq, Hkv, final, [0] * len(start))   # tables for the final lengths
    B = len(start)
    pool = DevPool(w_full)
    opool = oracle.new_pool(pool.shape)
    kv = [w_full.kv(s) for s in range(B)]
    # the contexts before the first step
    w0 = w_full.with_ranges(np.zeros(B, dtype=np.int64), np.array(start))
    gpu_append(pool, 0, dev(np.concatenate([kv[s][0][:start[s]] for s in range(B)])),
               dev(np.concatenate([kv[s][1][:start[s]] for s in range(B)])), DevBatch(w0))
    for s in range(B):
        oracle.append(opool, pool.shape, 0, kv[s][0][:start[s]], kv[s][1][:start[s]], 0,
                      w_full.page_tables[s])
    # one plan at the lengths of step 0, good for `steps` more tokens
    w_step = w_full.with_ranges(np.array(start), np.array(start) + 1)
    db = DevBatch(w_step)
    ws_bytes = mc.mc_attn_workspace_size(B, B, Hq, Hkv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan_ahead(pool.desc, Hq, B, B, db.cu_q, db.begin, db.page_table, db.cu_pages, steps,
                          ws, ws_bytes)
    mc.mc_attn_plan_check(ws)
    out = torch.zeros((B, Hq, 128), dtype=torch.int16, device=DEV)
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=DEV)
    q_all = [w_full.q(s) for s in range(B)]               # one query row per position
    for t in range(steps):
        pos = [n + t for n in start]
        begin = dev(np.array(pos, dtype=np.int32))        # the sequences have grown by t tokens
        k_new = np.concatenate([kv[s][0][pos[s]:pos[s] + 1] for s in range(B)])
        v_new = np.concatenate([kv[s][1][pos[s]:pos[s] + 1] for s in range(B)])
        q = np.concatenate([q_all[s][pos[s]:pos[s] + 1] for s in range(B)])
        mc.mc_kv_append(pool.desc, 0, dev(k_new), dev(v_new), B, B, db.cu_q, begin, db.page_table,
                        db.cu_pages)
        mc.mc_prefix_prefill_attn(pool.desc, 0, dev(q), Hq, B, B, db.cu_q, begin, db.page_table,
                                  db.cu_pages, 0.0, out, lse, ws, ws_bytes)
        for s in range(B):
            oracle.append(opool, pool.shape, 0, k_new[s:s + 1], v_new[s:s + 1], pos[s],
                          w_full.page_tables[s])
        if t % 9 == 0 or t == steps - 1:
            torch.cuda.synchronize()
            for s in range(B):
                ro, rl = oracle.attention(opool, pool.shape, 0, w_full.page_tables[s], q[s:s + 1], Hq,
                                          pos[s], pos[s] + 1)
                assert np.max(np.abs(oracle.decode(bits(out[s:s + 1]), w_full.dtype) - ro)) <= O_TOL, (t, s)
                assert np.max(np.abs(lse[s:s + 1].cpu().numpy() - rl)) <= LSE_TOL, (t, s)
    # a table too short for the tokens to come is reported
    mc.mc_attn_plan_ahead(pool.desc, Hq, B, B, db.cu_q, db.begin, db.page_table, db.cu_pages,
                          steps + 64, ws, ws_bytes)
    with pytest.raises(mc.McError) as e:
        mc.mc_attn_plan_check(ws)
    assert e.value.status == mc.MC_ERR_RANGE


def test_one_plan_with_forks_and_a_prefill_range_up_to_a_tile_edge():
    """mc_attn_plan_ahead over a batch that holds a group of forks (their shared prefix is
    attended together; the group's items keep their KV range while the members' own remainders
    grow), an unrelated decode row and a prefill range: every begin grows step by step until it
    has grown by exactly ahead_tokens, where the first fork's keys end on a 64-key tile edge.
    Every row is checked against the oracle at every step."""
    ahead, Hq, Hkv = 23, 32, 8
    start = [1000, 1300, 1040, 777, 300]                 # lengths before the first step
    qlen = [1, 1, 1, 1, 40]                              # new tokens per step
    assert (start[0] + ahead + 1) % 64 == 0
    final = [n + ahead + q for n, q in zip(start, qlen)]
    w_full = small_workload(725, mi.BF16, Hq, Hkv, final, [0] * 5)
    w_full.share_prefix(1, 0, 960)                       # forks of sequence 0: 60 shared pages
    w_full.share_prefix(2, 0, 960)
    B = 5
    pool = DevPool(w_full)
    opool = oracle.new_pool(pool.shape)
    kv = [w_full.kv(s) for s in range(B)]
    w0 = w_full.with_ranges(np.zeros(B, dtype=np.int64), np.array(start))
    gpu_append(pool, 0, dev(np.concatenate([kv[s][0][:start[s]] for s in range(B)])),
               dev(np.concatenate([kv[s][1][:start[s]] for s in range(B)])), DevBatch(w0))
    for s in range(B):
        oracle.append(opool, pool.shape, 0, kv[s][0][:start[s]], kv[s][1][:start[s]], 0,
                      w_full.page_tables[s])
    w_step = w_full.with_ranges(np.array(start), np.array(start) + np.array(qlen))
    db = DevBatch(w_step)
    tq = int(sum(qlen))
    ws_bytes = mc.mc_attn_workspace_size(B, tq, Hq, Hkv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan_ahead(pool.desc, Hq, B, tq, db.cu_q, db.begin, db.page_table, db.cu_pages, ahead,
                          ws, ws_bytes)
    mc.mc_attn_plan_check(ws)
    hdr = ws[:64].view(torch.int32).cpu().numpy()
    assert hdr[8] > 0, hdr                               # partial rows of a shared-prefix group
    out = torch.zeros((tq, Hq, 128), dtype=torch.int16, device=DEV)
    lse = torch.zeros((tq, Hq), dtype=torch.float32, device=DEV)
    # one query row per position of every sequence
    q_all = [mi.normal_bits(mi.rng_for(725, s, mi.KIND_Q), (final[s], Hq, 128), mi.BF16) for s in range(B)]
    for t in range(ahead + 1):
        pos = [n + t for n in start]
        begin = dev(np.array(pos, dtype=np.int32))
        k_new = np.concatenate([kv[s][0][pos[s]:pos[s] + qlen[s]] for s in range(B)])
        v_new = np.concatenate([kv[s][1][pos[s]:pos[s] + qlen[s]] for s in range(B)])
        q = np.concatenate([q_all[s][pos[s]:pos[s] + qlen[s]] for s in range(B)])
        mc.mc_kv_append(pool.desc, 0, dev(k_new), dev(v_new), B, tq, db.cu_q, begin, db.page_table,
                        db.cu_pages)
        mc.mc_prefix_prefill_attn(pool.desc, 0, dev(q), Hq, B, tq, db.cu_q, begin, db.page_table,
                                  db.cu_pages, 0.0, out, lse, ws, ws_bytes)
        torch.cuda.synchronize()
        lo = 0
        for s in range(B):
            oracle.append(opool, pool.shape, 0, k_new[lo:lo + qlen[s]], v_new[lo:lo + qlen[s]], pos[s],
                          w_full.page_tables[s])
            ro, rl = oracle.attention(opool, pool.shape, 0, w_full.page_tables[s], q[lo:lo + qlen[s]],
                                      Hq, pos[s], pos[s] + qlen[s])
            go = oracle.decode(bits(out[lo:lo + qlen[s]]), mi.BF16)
            assert np.max(np.abs(go - ro)) <= O_TOL, (t, s)
            assert np.max(np.abs(lse[lo:lo + qlen[s]].cpu().numpy() - rl)) <= LSE_TOL, (t, s)
            lo += qlen[s]


def test_a_begin_that_no_longer_fits_the_plan_writes_nothing():
    """The attention call reads begin itself.  A value the plan was not made for - negative, or
    far below the planned one - must neither fault nor read outside the sequence's table: rows of
    a sequence whose begin is negative stay unwritten, the other sequences are unaffected."""
    Hq, Hkv = 32, 8
    start = [1500, 2100, 900]
    w = small_workload(726, mi.BF16, Hq, Hkv, [n + 1 for n in start], start)
    pool, opool = DevPool(w), None
    opool = oracle.new_pool(pool.shape)
    fill_both(w, pool, opool)
    db = DevBatch(w)
    ws_bytes = mc.mc_attn_workspace_size(3, 3, Hq, Hkv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan_ahead(pool.desc, Hq, 3, 3, db.cu_q, db.begin, db.page_table, db.cu_pages, 0, ws,
                          ws_bytes)
    mc.mc_attn_plan_check(ws)
    q = np.concatenate([w.q(s) for s in range(3)])
    out = torch.full((3, Hq, 128), 0x7fc1, dtype=torch.int16, device=DEV)
    lse = torch.full((3, Hq), float("nan"), dtype=torch.float32, device=DEV)
    stale = dev(np.array([-7, 2100, 3], dtype=np.int32))      # negative / as planned / far too small
    mc.mc_prefix_prefill_attn(pool.desc, 0, dev(q), Hq, 3, 3, db.cu_q, stale, db.page_table,
                              db.cu_pages, 0.0, out, lse, ws, ws_bytes)
    torch.cuda.synchronize()
    assert bool((out[0] == 0x7fc1).all()) and bool(torch.isnan(lse[0]).all())   # nothing written
    ro, rl = oracle_rows(w, opool, pool.shape, 0, 1, w.q(1))
    assert np.max(np.abs(oracle.decode(bits(out[1:2]), w.dtype) - ro)) <= O_TOL
    assert np.max(np.abs(lse[1:2].cpu().numpy() - rl)) <= LSE_TOL
    # sequence 2 now stands at 3 tokens: its row attends keys 0..3 of its own pages, as the oracle does
    ro, rl = oracle.attention(opool, pool.shape, 0, w.page_tables[2], w.q(2), Hq, 3, 4)
    assert np.max(np.abs(oracle.decode(bits(out[2:3]), w.dtype) - ro)) <= O_TOL
    assert np.max(np.abs(lse[2:3].cpu().numpy() - rl)) <= LSE_TOL


def test_bad_page_id_in_a_large_batch_is_reported():
    # batches of more than 256 sequences have their page ids checked by a kernel of its own
    rng = mi.rng_for(730)
    lens = [int(x) for x in rng.integers(1, 200, size=300)]
    w = small_workload(731, mi.BF16, 32, 8, lens, [n - 1 for n in lens])
    pool, db = DevPool(w), DevBatch(w)
    ws_bytes = mc.mc_attn_workspace_size(db.batch, db.total_q, 32, 8)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan(pool.desc, 32, db.batch, db.total_q, db.cu_q, db.begin, db.page_table,
                    db.cu_pages, ws, ws_bytes)
    mc.mc_attn_plan_check(ws)                                 # the good tables pass
    bad = db.page_table.clone()
    bad[int(w.cu_pages[217])] = w.num_pages                   # first page of sequence 217
    mc.mc_attn_plan(pool.desc, 32, db.batch, db.total_q, db.cu_q, db.begin, bad, db.cu_pages, ws,
                    ws_bytes)
    with pytest.raises(mc.McError) as e:
        mc.mc_attn_plan_check(ws)
    assert e.value.status == mc.MC_ERR_RANGE
    out = torch.full((db.total_q, 32, 128), 0x7fc1, dtype=torch.int16, device=DEV)
    lse = torch.full((db.total_q, 32), 7.0, dtype=torch.float32, device=DEV)
    q = torch.zeros((db.total_q, 32, 128), dtype=torch.int16, device=DEV)
    mc.mc_prefix_prefill_attn(pool.desc, 0, q, 32, db.batch, db.total_q, db.cu_q, db.begin, bad,
                              db.cu_pages, 0.0, out, lse, ws, ws_bytes)
    torch.cuda.synchronize()
    assert torch.all(out == 0x7fc1) and torch.all(lse == 7.0)     # the failed plan launches nothing useful
