"""The attention entry point that allocates nothing (its workspace is an array inside the
library) against the workspace entry point, through the C ABI, on two calls in a row, the
second on a smaller batch.  Bars: max abs error <= 2e-2 on outputs, LSE within 1e-3."""
import numpy as np
import pytest
import torch

import mc_inputs as mi
import paper_2412_12488_amd as mc
from gpu_harness import DEV, DevBatch, DevPool, bits, dev, gpu_append, gpu_attention

pytestmark = pytest.mark.gpu
O_TOL, LSE_TOL = 2e-2, 1e-3


def _workload(seed, dtype, Hq, Hkv, lens, begins):
    n, b = np.array(lens), np.array(begins)
    num_pages = int(sum(-(-int(t) // 16) for t in n)) + 5
    w = mi.Workload(f"noalloc-{seed}", seed, dtype, 1, Hq, Hkv, num_pages, n, b)
    w.page_tables = mi.scatter_page_tables(mi.rng_for(seed, mi.KIND_TABLE), num_pages, n)
    return w


def _both_ways(w):
    """K/V of every token appended, then attention of the new ranges through the workspace
    entry point and through the one without allocation; both results as float64."""
    import oracle  # decode of 2-byte values only
    pool = DevPool(w)
    whole = w.with_ranges(np.zeros_like(w.n), w.n)
    ks = np.concatenate([w.kv(s)[0] for s in range(w.batch)])
    vs = np.concatenate([w.kv(s)[1] for s in range(w.batch)])
    gpu_append(pool, 0, dev(ks), dev(vs), DevBatch(whole))
    db = DevBatch(w)
    q = dev(np.concatenate([w.q(s) for s in range(w.batch)]))
    ref_o, ref_l = gpu_attention(pool, 0, q, db)
    out = torch.full((db.total_q, w.num_q_heads, 128), 0x7fc1, dtype=torch.int16, device=DEV)
    lse = torch.full((db.total_q, w.num_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    before = torch.cuda.memory_allocated()
    mc.mc_prefix_prefill_attn_noalloc(pool.desc, 0, q, w.num_q_heads, db.batch, db.total_q,
                                      db.cu_q, db.begin, db.page_table, db.cu_pages, 0.0, out, lse)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    dec = lambda t: oracle.decode(bits(t), w.dtype)
    return dec(ref_o), ref_l.cpu().numpy().astype(np.float64), dec(out), \
        lse.cpu().numpy().astype(np.float64)


def _check(w):
    ro, rl, go, gl = _both_ways(w)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    assert float(np.max(np.abs(go - ro))) <= O_TOL
    assert float(np.max(np.abs(gl - rl))) <= LSE_TOL


@pytest.mark.parametrize("dtype,Hq,Hkv", [(mi.BF16, 32, 8), (mi.F16, 8, 8)])
def test_two_calls_in_a_row_the_second_smaller(dtype, Hq, Hkv):
    # prefill ranges next to decode rows over long contexts: the plan cuts KV ranges into
    # chunks, so the work list, the partial rows and the merge all go through the array
    _check(_workload(901, dtype, Hq, Hkv, [1500, 700, 3000, 2200, 64], [1499, 300, 2999, 2100, 0]))
    # smaller batch, shorter contexts: the array still holds the first call's records
    _check(_workload(902, dtype, Hq, Hkv, [300, 90], [299, 40]))


def test_long_ranges_take_the_wide_tiles_through_the_array():
    # a long new range over a long prefix: the planner picks the 256-row q tiles; no KV range is
    # cut, so the array only holds the work list
    _check(_workload(904, mi.BF16, 64, 8, [14113], [10007]))


def test_a_batch_beyond_the_array_is_refused():
    w = _workload(903, mi.BF16, 8, 8, [64], [0])
    pool, db = DevPool(w), DevBatch(w)
    q = dev(w.q(0))
    out = torch.zeros((64, 8, 128), dtype=torch.int16, device=DEV)
    lse = torch.zeros((64, 8), dtype=torch.float32, device=DEV)
    with pytest.raises(mc.McError) as e:   # 2^25 q tiles of work-list records do not fit 8 MiB
        mc.mc_prefix_prefill_attn_noalloc(pool.desc, 0, q, 8, 1, 1 << 30, db.cu_q, db.begin,
                                          db.page_table, db.cu_pages, 0.0, out, lse)
    assert e.value.status == mc.MC_ERR_RANGE
    torch.cuda.synchronize()
    assert not out.any().item()            # nothing was launched
