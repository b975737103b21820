"""Plumbing for the GPU parity tests: device buffers from a Workload, the GPU
path through the C ABI, and the oracle run on the same seeded inputs.  Holds no
arithmetic of the method."""
import numpy as np
import torch

import mc_inputs as mi
import oracle
import paper_2412_12488_amd as mc

DEV = "cuda:0"


def dev(a: np.ndarray) -> torch.Tensor:
    """numpy (uint16 bits or int32) -> device tensor with the same bytes."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(DEV)


def bits(t: torch.Tensor) -> np.ndarray:
    """device int16 tensor -> numpy uint16 bits."""
    return t.cpu().numpy().view(np.uint16)


def layer_variant_dev(base: torch.Tensor, layer: int) -> torch.Tensor:
    """torch twin of mi.layer_variant for int16 device tensors."""
    if layer == 0:
        return base
    out = torch.roll(base, 17 * layer, 0)
    if layer & 1:
        out = out ^ torch.tensor(-32768, dtype=torch.int16, device=base.device)
    return out


class DevBatch:
    """Device-side ragged-batch arrays of a Workload."""

    def __init__(self, w: mi.Workload):
        self.w = w
        self.batch = w.batch
        self.total_q = int(w.cu_q[-1])
        self.cu_q = dev(w.cu_q)
        self.begin = dev(w.b.astype(np.int32))
        self.page_table = dev(w.flat_page_table)
        self.cu_pages = dev(w.cu_pages)
        self.tables = [dev(t) for t in w.page_tables]


class DevPool:
    def __init__(self, w: mi.Workload, num_pages=None, fill=None, num_layers=None):
        self.num_pages = num_pages or w.num_pages
        self.num_layers = num_layers or w.num_layers
        self.elems = self.num_layers * self.num_pages * 2 * w.num_kv_heads * 16 * 128
        if fill is None:
            self.t = torch.zeros(self.elems, dtype=torch.int16, device=DEV)
        else:
            self.t = dev(fill)
            assert self.t.numel() == self.elems
        self.desc = mc.pool_desc(self.t, self.num_layers, self.num_pages, w.num_kv_heads, w.dtype)
        self.shape = oracle.Shape(self.num_layers, self.num_pages, 16, w.num_kv_heads, 128, w.dtype)


def gpu_append(pool: DevPool, layer: int, k: torch.Tensor, v: torch.Tensor, db: DevBatch):
    mc.mc_kv_append(pool.desc, layer, k, v, db.batch, db.total_q, db.cu_q, db.begin,
                    db.page_table, db.cu_pages)


def gpu_attention(pool: DevPool, layer: int, q: torch.Tensor, db: DevBatch, sm_scale=0.0,
                  check_plan=True):
    w = db.w
    ws_bytes = mc.mc_attn_workspace_size(db.batch, db.total_q, w.num_q_heads, w.num_kv_heads)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    mc.mc_attn_plan(pool.desc, w.num_q_heads, db.batch, db.total_q, db.cu_q, db.begin,
                    db.page_table, db.cu_pages, ws, ws_bytes)
    if check_plan:
        mc.mc_attn_plan_check(ws)
    out = torch.full((db.total_q, w.num_q_heads, 128), 0x7fc1, dtype=torch.int16, device=DEV)
    lse = torch.full((db.total_q, w.num_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    mc.mc_prefix_prefill_attn(pool.desc, layer, q, w.num_q_heads, db.batch, db.total_q, db.cu_q,
                              db.begin, db.page_table, db.cu_pages, sm_scale, out, lse, ws,
                              ws_bytes)
    torch.cuda.synchronize()
    return out, lse


def fill_both(w: mi.Workload, pool: DevPool, opool: np.ndarray, layers=(0,), upto_end=True):
    """Put K/V of tokens [0, n) (or [0, b)) of every sequence into the GPU pool through
    mc_kv_append and into the oracle's pool through the oracle's append.  Returns per-layer
    device K/V of the whole batch ([sum n][Hkv][D]) for reuse."""
    lens = w.n if upto_end else w.b
    whole = w.with_ranges(np.zeros_like(lens), lens)
    db = DevBatch(whole)
    for layer in layers:
        ks, vs = [], []
        for s in range(w.batch):
            k, v = w.kv(s, layer)
            k, v = k[: lens[s]], v[: lens[s]]
            if lens[s]:
                oracle.append(opool, pool.shape, layer, k, v, 0, w.page_tables[s])
            ks.append(k)
            vs.append(v)
        if db.total_q:
            gpu_append(pool, layer, dev(np.concatenate(ks)), dev(np.concatenate(vs)), db)
    torch.cuda.synchronize()


def oracle_rows(w: mi.Workload, opool, shape, layer, seq, q_bits, rows=None, heads=None,
                scale=None):
    return oracle.attention(opool, shape, layer, w.page_tables[seq], q_bits, w.num_q_heads,
                            int(w.b[seq]), int(w.n[seq]), scale=scale, sel_rows=rows,
                            sel_heads=heads)
