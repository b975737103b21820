#!/usr/bin/env python3
"""Benchmark of the paged KV-cache hot path on one MI355X.

A step is one pass of the whole path over one batch of the Llama-3-8B-shaped
workload (8 sequences, prompts in [1024, 4096], up to 75 % cached): page
allocation for the new tokens (host), KV append of the new tokens, the plan
(begin_forward), prefix-prefill attention with LSE, then pack of every sequence's
KV into a contiguous buffer and unpack into a second page pool.  All inputs are
resident in HBM before the timed region.  One JSON line goes to stdout.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16/fp16 MFMA, published
HBM_PEAK_GBS = 8000.0         # MI355X HBM3E, published


ATTN_WORKLOADS = ["cfg2", "cfg3-passB", "cfg4", "cfg5-16k", "cfg5-32k", "paper-500-over-500",
                  "paper-500-over-2500", "paper-500-over-4500", "decode-8", "decode-64",
                  "decode-256", "decode-64-plus-prefill", "decode-64-forks", "decode-64-no-forks",
                  "short-64-forks", "short-64-no-forks"]

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this very
# command with the default seed (counters scaled by what a plain 4 GiB copy reads; see
# profiles/bench_cfg2_hbm_traffic.md).  Valid only for the default workload.
MEASURED_TRAFFIC = {"seed": 2000, "attention_bytes": int((380.2 + 79.8) * 2**20),
                    "pack_4GiB_bytes": int((4096.2 + 4096.1) * 2**20)}


def attention_workload(name):
    import numpy as np

    import mc_inputs as mi
    if name == "cfg2":
        return mi.config(2)
    if name == "cfg3-passB":
        return mi.config(3, num_layers=1)
    if name == "cfg4":
        return mi.config(4)
    if name in ("cfg5-16k", "cfg5-32k"):
        w = mi.config(5, num_layers=1)
        keep = 0 if name == "cfg5-16k" else 1
        b = np.where(np.arange(2) == keep, w.b, 0)
        n = np.where(np.arange(2) == keep, w.n, 0)
        return w.with_ranges(b, n, name)
    if name.startswith("paper-500-over-"):
        return mi.paper_point(int(name.rsplit("-", 1)[1]))
    if name in ("decode-64-forks", "decode-64-no-forks"):
        # 64 decode steps of sequences that continue one 2048-token prompt by 64..1024 tokens of
        # their own: as forks (page tables share the prompt's 128 pages, Sec. 3.5 fork_sequence)
        # or as unrelated sequences of the same lengths
        rng = mi.rng_for(4243)
        n = 2048 + rng.integers(64, 1025, size=64)
        w = mi.Workload(name, 4243, mi.BF16, 1, 32, 8, 65536, n, n - 1)
        w.page_tables = mi.scatter_page_tables(mi.rng_for(4243, mi.KIND_TABLE), 65536, n)
        if name == "decode-64-forks":
            for s in range(1, 64):
                w.share_prefix(s, 0, 2048)
        return w
    if name in ("short-64-forks", "short-64-no-forks"):
        # 64 sequences that continue one 2048-token prompt by 0..512 cached tokens of their own
        # and bring 5..24 new tokens each (speculative or chunked continuation of forked
        # requests): as forks of the prompt, or as unrelated sequences of the same lengths
        rng = mi.rng_for(4244)
        b = 2048 + rng.integers(0, 513, size=64)
        n = b + rng.integers(5, 25, size=64)
        w = mi.Workload(name, 4244, mi.BF16, 1, 32, 8, 65536, n, b)
        w.page_tables = mi.scatter_page_tables(mi.rng_for(4244, mi.KIND_TABLE), 65536, n)
        if name == "short-64-forks":
            for s in range(1, 64):
                w.share_prefix(s, 0, 2048)
        return w
    if name.startswith("decode-"):
        # one new token per sequence over contexts ~ U[1024, 4096] (Llama-3-8B shapes), alone or
        # in one ragged batch with a 2048-token prefill range over 1024 cached tokens
        batch = int(name.split("-")[1])
        rng = mi.rng_for(4242, batch)
        n = rng.integers(1024, 4097, size=batch)
        b = n - 1
        if name.endswith("-plus-prefill"):
            n, b = np.append(n, 3072), np.append(b, 1024)
        w = mi.Workload(name, 4242, mi.BF16, 1, 32, 8, 65536, n, b)
        w.page_tables = mi.scatter_page_tables(mi.rng_for(4242, mi.KIND_TABLE), 65536, n)
        return w
    raise SystemExit(f"unknown workload {name}; choose from {ATTN_WORKLOADS}")


def launch_stats(fn, iters, warm=2):
    """Per-call milliseconds of fn (HIP events between consecutive calls on the current
    stream): mean, median and minimum over iters calls after warm untimed ones."""
    import numpy as np
    import torch
    for _ in range(warm):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    ev[0].record()
    for i in range(iters):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(iters)])
    return {"mean": float(t.mean()), "median": float(np.median(t)), "min": float(t.min())}


def oracle_sample_check(w, pool_bits, q_bits, out_t, lse_t, triples, seed=17):
    """A bounded sample of (sequence, row, q head) triples of an attention result against the
    CPU oracle (fp64), with the oracle's time for the sample (mostly the gather of each
    sequence's K/V through its page table).  pool_bits / q_bits: host uint16 arrays of what the
    GPU read."""
    import time

    import numpy as np

    import mc_inputs as mi
    import oracle
    shape = oracle.Shape(1, w.num_pages, 16, w.num_kv_heads, 128, w.dtype)
    out_b = out_t.cpu().numpy().view(np.uint16)
    lse_h = lse_t.cpu().numpy().astype(np.float64)
    G = w.num_q_heads // w.num_kv_heads
    live = [s for s in range(w.batch) if w.n[s] > w.b[s]]
    err_o = err_l = 0.0
    t_or, fl_sample, n_done = 0.0, 0, 0
    for s in live:
        q_len, b, lo = int(w.n[s] - w.b[s]), int(w.b[s]), int(w.cu_q[s])
        rows, heads = mi.sample_rows(mi.rng_for(seed, s), q_len, b, w.num_q_heads,
                                     max(w.num_kv_heads, triples // len(live)),
                                     tile_tokens=128 // G, num_kv_heads=w.num_kv_heads)
        qs = q_bits[lo:lo + q_len]
        c0 = time.perf_counter()
        ro, rl = oracle.attention(pool_bits, shape, 0, w.page_tables[s], qs, w.num_q_heads, b,
                                  int(w.n[s]), sel_rows=rows, sel_heads=heads)
        t_or += time.perf_counter() - c0
        go = oracle.decode(out_b[lo:lo + q_len][rows, heads], w.dtype)
        err_o = max(err_o, float(np.max(np.abs(go - ro))))
        err_l = max(err_l, float(np.max(np.abs(lse_h[lo:lo + q_len][rows, heads] - rl))))
        fl_sample += int(np.sum(4 * 128 * (b + rows.astype(np.int64) + 1)))
        n_done += int(rows.size)
    return {"triples": n_done, "max_abs_err_O": round(err_o, 6), "max_abs_err_LSE": round(err_l, 8),
            "oracle_s": round(t_or, 2), "oracle_cores": len(os.sched_getaffinity(0)),
            "sample_flops": fl_sample}


def attention_only(name, iters, values="normal", oracle_triples=0, mfma_ceiling=None):
    """Attention kernel alone on resident Q/K/V: one dict.  For rocprofv3 runs and the
    per-workload table.  values: "normal" = N(0,1) like the workload; "zero" = all zeros (same
    instructions, the least operand switching: shows how far the data's power draw holds the
    clock down).  oracle_triples > 0: that many sampled outputs are checked against the CPU
    oracle after the timing.  mfma_ceiling: measured MFMA-alone rate (TFLOP/s) to relate to."""
    import numpy as np
    import torch

    import paper_2412_12488_amd as mc
    dev = "cuda:0"
    w = attention_workload(name)
    Hq, Hkv = w.num_q_heads, w.num_kv_heads
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    gen = torch.randn if values == "normal" else torch.zeros
    pool = gen(w.num_pages * 2 * Hkv * 16 * 128, dtype=torch.bfloat16, device=dev)
    desc = mc.pool_desc(pool, 1, w.num_pages, Hkv, w.dtype)
    tq = int(w.cu_q[-1])
    q = gen(tq * Hq * 128, dtype=torch.bfloat16, device=dev)
    cu_q, begin = up(w.cu_q), up(w.b.astype(np.int32))
    table, cu_pages = up(w.flat_page_table), up(w.cu_pages)
    wsb = mc.mc_attn_workspace_size(w.batch, tq, Hq, Hkv)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    out = torch.empty((tq, Hq, 128), dtype=torch.int16, device=dev)
    lse = torch.empty((tq, Hq), dtype=torch.float32, device=dev)
    mc.mc_attn_plan(desc, Hq, w.batch, tq, cu_q, begin, table, cu_pages, ws, wsb)
    mc.mc_attn_plan_check(ws)
    run = lambda: mc.mc_prefix_prefill_attn(desc, 0, q, Hq, w.batch, tq, cu_q, begin, table, cu_pages,
                                            0.0, out, lse, ws, wsb)
    st = launch_stats(run, iters)
    ms = st["mean"]
    fl = w.useful_flops()
    alg_bytes = 2 * tq * Hq * 256 + tq * Hq * 4 + int(np.sum(w.n)) * w.token_bytes
    res = {"workload": w.name, "values": values, "new_tokens": tq,
           "kv_tokens": int(np.sum(w.n)),
           "algorithmic_GBps": round(alg_bytes / ms / 1e6, 1),
           "useful_flops": fl, "ms": round(ms, 4), "ms_median": round(st["median"], 4),
           "ms_min": round(st["min"], 4),
           "TFLOPs": round(fl / ms / 1e9, 1),
           "frac_of_mfma_peak": round(fl / ms / 1e9 / MFMA_PEAK_TFLOPS, 4)}
    if mfma_ceiling:
        res["frac_of_measured_mfma_rate"] = round(fl / ms / 1e9 / mfma_ceiling, 4)
    if oracle_triples:
        res["oracle_sample"] = oracle_sample_check(
            w, pool.view(torch.int16).cpu().numpy().view(np.uint16),
            q.view(torch.int16).cpu().numpy().view(np.uint16).reshape(tq, Hq, 128), out, lse,
            oracle_triples)
    del pool, q, out, lse, ws
    torch.cuda.empty_cache()
    return res


def layer_overlap(w, layers, iters=5):
    """`layers` layers of the workload, append + attention per layer on the main stream, each
    layer's KV shipped to a second pool (pack + unpack) either on the same stream after the
    layer's attention, or on a side stream beside the next layer's work (paper Sec. 3.6: a
    computation stream and a communication stream).  Both streams have the default priority.
    Returns milliseconds for the whole pass and per attention launch, both ways."""
    import numpy as np
    import torch

    import mc_inputs as mi
    import paper_2412_12488_amd as mc
    dev = "cuda:0"
    B, Hq, Hkv = w.batch, w.num_q_heads, w.num_kv_heads
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    tq, n_tok = int(w.cu_q[-1]), int(np.sum(w.n))
    # pages of the whole batch, scattered in a pool of 8 x that many pages per layer
    pages = 8 * int(sum(-(-int(t) // 16) for t in w.n))
    tab_a = mi.scatter_page_tables(mi.rng_for(w.seed, 301), pages, w.n)
    tab_b = mi.scatter_page_tables(mi.rng_for(w.seed, 302), pages, w.n)
    elems = layers * pages * 2 * Hkv * 16 * 128
    pool_a = torch.randn(elems, dtype=torch.bfloat16, device=dev)
    pool_b = torch.empty(elems, dtype=torch.bfloat16, device=dev)
    da = mc.pool_desc(pool_a, layers, pages, Hkv, w.dtype)
    db = mc.pool_desc(pool_b, layers, pages, Hkv, w.dtype)
    q = torch.randn(tq * Hq * 128, dtype=torch.bfloat16, device=dev)
    k = torch.randn(tq * Hkv * 128, dtype=torch.bfloat16, device=dev)
    v = torch.randn(tq * Hkv * 128, dtype=torch.bfloat16, device=dev)
    cu_q, begin = up(w.cu_q), up(w.b.astype(np.int32))
    cu_pages = up(w.cu_pages)
    table_a, table_b = up(np.concatenate(tab_a).astype(np.int32)), up(np.concatenate(tab_b).astype(np.int32))
    s0, s1 = up(np.zeros(B, np.int32)), up(w.n.astype(np.int32))
    sizes = np.array([2 * int(t) * Hkv * 128 * 2 for t in w.n], dtype=np.int64)      # bytes
    off = up(np.concatenate([[0], np.cumsum(sizes)[:-1]]))
    sends = [torch.empty(int(sizes.sum()) // 2, dtype=torch.int16, device=dev) for _ in range(layers)]
    max_pages = int(max(-(-int(t) // 16) for t in w.n))
    wsb = mc.mc_attn_workspace_size(B, tq, Hq, Hkv)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    out = torch.empty((tq, Hq, 128), dtype=torch.int16, device=dev)
    lse = torch.empty((tq, Hq), dtype=torch.float32, device=dev)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    mc.mc_attn_plan(da, Hq, B, tq, cu_q, begin, table_a, cu_pages, ws, wsb)   # once for all layers

    def one_pass(overlap, attn_ev):
        xfer = side if overlap else main
        for layer in range(layers):
            mc.mc_kv_append(da, layer, k, v, B, tq, cu_q, begin, table_a, cu_pages, stream=main)
            appended = torch.cuda.Event()
            appended.record(main)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            mc.mc_prefix_prefill_attn(da, layer, q, Hq, B, tq, cu_q, begin, table_a, cu_pages, 0.0,
                                      out, lse, ws, wsb, stream=main)
            e1.record(main)
            attn_ev.append((e0, e1))
            if overlap:                 # the layer's KV is in the pages: it may leave
                side.wait_event(appended)
            mc.mc_kv_pack_batch(da, layer, layer + 1, B, table_a, cu_pages, s0, s1, off, max_pages,
                                sends[layer], stream=xfer)
            mc.mc_kv_unpack_batch(db, layer, layer + 1, B, table_b, cu_pages, s0, s1, off,
                                  max_pages, sends[layer], stream=xfer)
        if overlap:
            main.wait_stream(side)

    res = {}
    for overlap in (False, True):
        totals, attn = [], []
        for it in range(iters + 1):
            ev, t0, t1 = [], torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0.record(main)
            one_pass(overlap, ev)
            t1.record(main)
            torch.cuda.synchronize()
            if it:                                       # the first pass warms up
                totals.append(t0.elapsed_time(t1))
                attn += [a.elapsed_time(b) for a, b in ev]
        key = "two_streams" if overlap else "one_stream"
        res[key] = {"pass_ms_median": round(float(np.median(totals)), 4),
                    "pass_ms_min": round(float(np.min(totals)), 4),
                    "attention_ms_median": round(float(np.median(attn)), 4),
                    "attention_ms_min": round(float(np.min(attn)), 4)}
    res["layers"] = layers
    res["payload_MiB_per_layer"] = round(n_tok * w.token_bytes / 2**20, 1)
    res["pass_gain"] = round(res["one_stream"]["pass_ms_median"] / res["two_streams"]["pass_ms_median"], 3)
    res["attention_slowdown_beside_transfer"] = round(
        res["two_streams"]["attention_ms_median"] / res["one_stream"]["attention_ms_median"], 3)
    del pool_a, pool_b, sends, q, k, v, ws, out, lse
    torch.cuda.empty_cache()
    return res


def decode_step_latency(name, iters=50):
    """One decode step = append + plan + attention (+ merge) of a decode batch, launched call by
    call and replayed from a HIP graph (the calls allocate nothing and never synchronise, so the
    step can be captured): microseconds per step, both ways."""
    import numpy as np
    import torch

    import paper_2412_12488_amd as mc
    dev = "cuda:0"
    w = attention_workload(name)
    Hq, Hkv = w.num_q_heads, w.num_kv_heads
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    pool = torch.randn(w.num_pages * 2 * Hkv * 16 * 128, dtype=torch.bfloat16, device=dev)
    desc = mc.pool_desc(pool, 1, w.num_pages, Hkv, w.dtype)
    tq = int(w.cu_q[-1])
    q = torch.randn(tq * Hq * 128, dtype=torch.bfloat16, device=dev)
    k = torch.randn(tq * Hkv * 128, dtype=torch.bfloat16, device=dev)
    v = torch.randn(tq * Hkv * 128, dtype=torch.bfloat16, device=dev)
    cu_q, begin = up(w.cu_q), up(w.b.astype(np.int32))
    table, cu_pages = up(w.flat_page_table), up(w.cu_pages)
    wsb = mc.mc_attn_workspace_size(w.batch, tq, Hq, Hkv)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    out = torch.empty((tq, Hq, 128), dtype=torch.int16, device=dev)
    lse = torch.empty((tq, Hq), dtype=torch.float32, device=dev)

    def step():
        mc.mc_kv_append(desc, 0, k, v, w.batch, tq, cu_q, begin, table, cu_pages)
        mc.mc_attn_plan(desc, Hq, w.batch, tq, cu_q, begin, table, cu_pages, ws, wsb)
        mc.mc_prefix_prefill_attn(desc, 0, q, Hq, w.batch, tq, cu_q, begin, table, cu_pages, 0.0,
                                  out, lse, ws, wsb)

    def timed(fn):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3

    eager = timed(step)
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    replay = timed(graph.replay)

    # the same step when the plan was made once for many steps ahead (mc_attn_plan_ahead)
    mc.mc_attn_plan_ahead(desc, Hq, w.batch, tq, cu_q, begin, table, cu_pages, 0, ws, wsb)

    def step_planned():
        mc.mc_kv_append(desc, 0, k, v, w.batch, tq, cu_q, begin, table, cu_pages)
        mc.mc_prefix_prefill_attn(desc, 0, q, Hq, w.batch, tq, cu_q, begin, table, cu_pages, 0.0,
                                  out, lse, ws, wsb)
    planned = timed(step_planned)
    del pool, q, k, v, out, lse, ws, graph
    torch.cuda.empty_cache()
    return {"eager_us": round(eager, 1), "graph_us": round(replay, 1),
            "plan_reused_us": round(planned, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--seed", type=int, default=2000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-copy-sweep", action="store_true")
    ap.add_argument("--overlap", action="store_true",
                    help="plan and KV transfer on a second stream, beside append and attention "
                         "(default: the step's kernels run one after the other on one stream, so "
                         "that each kernel's duration is its own)")
    ap.add_argument("--attention-only", metavar="WORKLOAD", default=None,
                    help="time only the attention kernel on one workload and exit (for profiling): "
                         + ", ".join(ATTN_WORKLOADS))
    ap.add_argument("--decode-step", metavar="WORKLOAD", default=None,
                    help="time only one decode step (append + plan + attention + merge), launched "
                         "call by call, from a HIP graph and with a plan made once, and exit")
    ap.add_argument("--values", choices=["normal", "zero"], default="normal",
                    help="with --attention-only: Q/K/V values, N(0,1) or all zeros")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path has no cross-GPU step "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import bench_probe
    import mc_inputs as mi
    import paper_2412_12488_amd as mc

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    if args.attention_only:
        print(json.dumps(attention_only(args.attention_only, max(1, min(args.steps, 20)),
                                        args.values)))
        return
    if args.decode_step:
        print(json.dumps({args.decode_step: decode_step_latency(args.decode_step,
                                                                max(1, min(args.steps, 50)))}))
        return

    def up(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)

    w = mi.config(2, seed=args.seed)
    B, Hq, Hkv, D = w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim
    total_q = int(w.cu_q[-1])
    flops = w.useful_flops()

    # ---- resident inputs -------------------------------------------------------
    pool_elems = w.num_pages * 2 * Hkv * 16 * D
    pool_a = torch.zeros(pool_elems, dtype=torch.int16, device=dev)
    pool_b = torch.zeros(pool_elems, dtype=torch.int16, device=dev)
    desc_a = mc.pool_desc(pool_a, 1, w.num_pages, Hkv, w.dtype)
    desc_b = mc.pool_desc(pool_b, 1, w.num_pages, Hkv, w.dtype)
    kv = [w.kv(s) for s in range(B)]
    q_new = up(np.concatenate([w.q(s) for s in range(B)]))
    k_new = up(np.concatenate([kv[s][0][w.b[s]:] for s in range(B)]))
    v_new = up(np.concatenate([kv[s][1][w.b[s]:] for s in range(B)]))
    cu_q, begin = up(w.cu_q), up(w.b.astype(np.int32))
    table, cu_pages = up(w.flat_page_table), up(w.cu_pages)
    tables_a = [up(t) for t in w.page_tables]
    trng = mi.rng_for(args.seed, 77)
    tables_b_np = mi.scatter_page_tables(trng, w.num_pages, w.n)
    tables_b = [up(t) for t in tables_b_np]
    # one transfer buffer for the batch: sequence s at byte offset send_off[s]
    send_elems = [2 * int(w.n[s]) * Hkv * D for s in range(B)]
    send_off_np = np.concatenate([[0], np.cumsum(send_elems)[:-1]]).astype(np.int64) * 2
    send_all = torch.empty(int(sum(send_elems)), dtype=torch.int16, device=dev)
    send = [send_all[int(o) // 2: int(o) // 2 + e] for o, e in zip(send_off_np, send_elems)]
    send_off = torch.from_numpy(send_off_np).to(dev)
    r_s0 = up(np.zeros(B, dtype=np.int32))
    r_s1 = up(w.n.astype(np.int32))
    table_b, cu_pages_b = up(np.concatenate(tables_b_np).astype(np.int32)), cu_pages
    max_range_pages = int(max(-(-int(x) // 16) for x in w.n))
    # the cached prefixes [0, b) are already in the cache when a step starts
    wp = w.with_ranges(np.zeros_like(w.b), w.b)
    if int(wp.cu_q[-1]):
        mc.mc_kv_append(desc_a, 0, up(np.concatenate([kv[s][0][: w.b[s]] for s in range(B)])),
                        up(np.concatenate([kv[s][1][: w.b[s]] for s in range(B)])), B,
                        int(wp.cu_q[-1]), up(wp.cu_q), up(wp.b.astype(np.int32)), table, cu_pages)
    ws_bytes = mc.mc_attn_workspace_size(B, total_q, Hq, Hkv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out = torch.empty((total_q, Hq, D), dtype=torch.int16, device=dev)
    lse = torch.empty((total_q, Hq), dtype=torch.float32, device=dev)
    alloc = mc.mc_kv_allocator_create(w.num_pages)
    new_pages = [-(-int(w.n[s]) // 16) - int(w.b[s]) // 16 for s in range(B)]
    torch.cuda.synchronize()

    attn_events = []

    # Streams (all at the default priority).  By default every kernel of the step runs on one
    # stream, one after the other, so that each kernel's duration is its own.  With --overlap the
    # plan (begin_forward needs nothing from the step's kernels) and the transfer run on a second
    # stream, the plan beside the append and the transfer beside the attention (Sec. 3.6 of the
    # paper).  (The plan alone on a second stream was measured too: the two event waits it needs
    # cost what the 20 us of overlap save, 0.376 against 0.373 ms per step.)
    main_s = torch.cuda.current_stream()
    side_s = torch.cuda.Stream() if args.overlap else main_s
    plan_s = side_s
    xfer_s = side_s
    ev = {k: torch.cuda.Event() for k in ("append", "plan", "attn", "xfer")}

    def step(record):
        # a1: page reservation for the new tokens (host free list; ids from the seeded tables
        # are the ones the kernels use, so the step is repeatable)
        got = [mc.mc_kv_alloc_pages(alloc, n) for n in new_pages]
        for g in reversed(got):
            mc.mc_kv_free_pages(alloc, g[::-1])
        if xfer_s is not main_s:
            main_s.wait_event(ev["xfer"])     # the last step's pack has read the pages appended now
        if plan_s is not main_s:
            plan_s.wait_event(ev["attn"])     # the last step's attention has read the work list
        # begin_forward: plan the batch (second stream), a2: append the new tokens' K/V (main)
        mc.mc_attn_plan(desc_a, Hq, B, total_q, cu_q, begin, table, cu_pages, ws, ws_bytes,
                        stream=plan_s)
        mc.mc_kv_append(desc_a, 0, k_new, v_new, B, total_q, cu_q, begin, table, cu_pages,
                        stream=main_s)
        if plan_s is not main_s:
            ev["plan"].record(plan_s)
            main_s.wait_event(ev["plan"])
        if xfer_s is not main_s:
            ev["append"].record(main_s)
            xfer_s.wait_event(ev["append"])
        # a3: attention of the new range over cache + itself
        if record:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main_s)
        mc.mc_prefix_prefill_attn(desc_a, 0, q_new, Hq, B, total_q, cu_q, begin, table, cu_pages,
                                  0.0, out, lse, ws, ws_bytes, stream=main_s)
        if record:
            e1.record(main_s)
            attn_events.append((e0, e1))
        if plan_s is not main_s:
            ev["attn"].record(main_s)
        # a4 + a5: ship every sequence's KV [0, n) to the second pool (one launch each way)
        mc.mc_kv_pack_batch(desc_a, 0, 1, B, table, cu_pages, r_s0, r_s1, send_off,
                            max_range_pages, send_all, stream=xfer_s)
        mc.mc_kv_unpack_batch(desc_b, 0, 1, B, table_b, cu_pages_b, r_s0, r_s1, send_off,
                              max_range_pages, send_all, stream=xfer_s)
        if xfer_s is not main_s:
            ev["xfer"].record(xfer_s)

    for _ in range(args.warmup):
        step(False)
    mc.mc_attn_plan_check(ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    attn_times = np.array([a.elapsed_time(b) for a, b in attn_events])
    attn_ms = float(attn_times.mean())
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12
    value = flops / (ms_per_step * 1e-3) / 1e12

    def timed(fn, iters=20, warm=3):
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    # ---- MFMA issue rate of this GPU, alone, on constant operands and on operands drawn like
    #      the workload's (the matrix pipes' power, and with it the clock, follows the data) ----
    def mfma_rate(operands):
        sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
        fl = [0]

        def go():
            fl[0] = bench_probe.mfma_probe(w.dtype, operands, 512, 1000, sink,
                                           torch.cuda.current_stream().cuda_stream)
        ms = timed(go, iters=5, warm=2)
        return round(fl[0] / ms / 1e9, 1)

    n_op = bench_probe.operand_bytes() // 2
    ops_const = torch.full((n_op,), 1.0, dtype=torch.bfloat16, device=dev)
    ops_normal = up(mi.normal_bits(mi.rng_for(args.seed, 91), n_op, w.dtype))
    mfma_measured = {"constant_operands_TFLOPs": mfma_rate(ops_const),
                     "normal_operands_TFLOPs": mfma_rate(ops_normal)}
    del ops_const, ops_normal

    # ---- the attention call alone on the other configs (each with a sample of its outputs
    #      checked against the CPU oracle), on the paper's Table-2 shapes and on decode steps (one
    #      new token per sequence, alone and fused with a prefill range): the planner cuts the
    #      KV ranges of the small launches into chunks; decode is bound by HBM, so its figure is
    #      algorithmic GB/s ----
    other, overlap = {}, None
    if not args.no_copy_sweep:
        ceiling = mfma_measured["normal_operands_TFLOPs"]
        for name in ("cfg3-passB", "cfg4", "cfg5-16k", "cfg5-32k"):
            r = attention_only(name, 10, oracle_triples=0 if args.no_cpu_baseline else 1024,
                               mfma_ceiling=ceiling)
            other[name] = {k: r[k] for k in ("ms", "ms_median", "ms_min", "TFLOPs",
                                             "frac_of_mfma_peak", "frac_of_measured_mfma_rate",
                                             "useful_flops") if k in r}
            if "oracle_sample" in r:
                other[name]["oracle_sample"] = r["oracle_sample"]
        for name in ("paper-500-over-500", "paper-500-over-2500", "paper-500-over-4500",
                     "decode-64", "decode-256", "decode-64-plus-prefill", "decode-64-no-forks",
                     "decode-64-forks", "short-64-no-forks", "short-64-forks"):
            r = attention_only(name, 10)
            other[name] = {"ms": r["ms"], "ms_median": r["ms_median"], "ms_min": r["ms_min"],
                           "TFLOPs": r["TFLOPs"], "algorithmic_GBps": r["algorithmic_GBps"]}
        # a whole decode step (append + plan + attention + merge), call by call and as a graph
        other["decode_step_us"] = {n: decode_step_latency(n) for n in ("decode-8", "decode-64")}
        # four layers, each layer's KV shipped to a second pool after or beside the next layer
        overlap = layer_overlap(w, 4)

    # ---- copies, each alone: this workload, then the long-context transfer size ----
    copy = {}
    kv_bytes = int(np.sum(w.n)) * w.token_bytes
    new_bytes = total_q * w.token_bytes
    ms = timed(lambda: mc.mc_kv_append(desc_a, 0, k_new, v_new, B, total_q, cu_q, begin, table,
                                       cu_pages))
    copy["append_GBps"] = round(2 * new_bytes / ms / 1e6, 1)
    # mark_send: the new range also goes to a transfer buffer, in the append's pass (3 x payload
    # moved) or by a pack of the new range after the append (4 x payload moved)
    new_off = torch.from_numpy((np.concatenate([[0], np.cumsum(w.n - w.b)[:-1]]).astype(np.int64)
                                * w.token_bytes)).to(dev)
    new_buf = torch.empty(max(total_q, 1) * 2 * Hkv * D, dtype=torch.int16, device=dev)
    d_b, d_n = up(w.b.astype(np.int32)), up(w.n.astype(np.int32))
    new_pages_max = int(max(-(-int(n) // 16) - int(b) // 16 for n, b in zip(w.n, w.b)))
    ms_fused = timed(lambda: mc.mc_kv_append_send(desc_a, 0, k_new, v_new, B, total_q, cu_q, begin,
                                                  table, cu_pages, 0, d_b, d_n, new_off, new_buf))

    def append_then_pack():
        mc.mc_kv_append(desc_a, 0, k_new, v_new, B, total_q, cu_q, begin, table, cu_pages)
        mc.mc_kv_pack_batch(desc_a, 0, 1, B, table, cu_pages, d_b, d_n, new_off, new_pages_max,
                            new_buf)
    ms_two = timed(append_then_pack)
    copy["append_send_us"] = round(ms_fused * 1e3, 1)
    copy["append_then_pack_us"] = round(ms_two * 1e3, 1)
    copy["append_send_GBps"] = round(3 * new_bytes / ms_fused / 1e6, 1)

    def pack_all():
        for s in range(B):
            mc.mc_kv_pack_range(desc_a, 0, 1, tables_a[s], len(w.page_tables[s]), 0, int(w.n[s]),
                                send[s])

    def unpack_all():
        for s in range(B):
            mc.mc_kv_unpack_range(desc_b, 0, 1, tables_b[s], len(tables_b_np[s]), 0, int(w.n[s]),
                                  send[s])
    copy["pack_GBps"] = round(2 * kv_bytes / timed(pack_all) / 1e6, 1)
    copy["unpack_GBps"] = round(2 * kv_bytes / timed(unpack_all) / 1e6, 1)
    copy["pack_batch_GBps"] = round(2 * kv_bytes / timed(lambda: mc.mc_kv_pack_batch(
        desc_a, 0, 1, B, table, cu_pages, r_s0, r_s1, send_off, max_range_pages, send_all)) / 1e6, 1)
    copy["unpack_batch_GBps"] = round(2 * kv_bytes / timed(lambda: mc.mc_kv_unpack_batch(
        desc_b, 0, 1, B, table_b, cu_pages_b, r_s0, r_s1, send_off, max_range_pages,
        send_all)) / 1e6, 1)
    copy["payload_MiB"] = round(kv_bytes / 2**20, 1)
    # the same three copies with the pages, the new K/V and the transfer buffer changing from
    # launch to launch (six sets, about 0.9 GiB touched per round): nothing a launch reads or
    # writes can still sit in the 256 MiB Infinity Cache from the launch before
    R = 6
    rot_tables = [up(np.concatenate(mi.scatter_page_tables(mi.rng_for(args.seed, 400 + r),
                                                           w.num_pages, w.n)).astype(np.int32))
                  for r in range(R)]
    rot_send = [torch.empty_like(send_all) for _ in range(R)]
    rot_k = [torch.empty_like(k_new).copy_(k_new) for _ in range(R)]
    rot_v = [torch.empty_like(v_new).copy_(v_new) for _ in range(R)]
    turn = [0]

    def rotated(fn):
        def go():
            r = turn[0] = (turn[0] + 1) % R
            fn(r)
        return timed(go, iters=4 * R, warm=R)
    copy["rotated"] = {
        "sets": R,
        "append_GBps": round(2 * new_bytes / rotated(lambda r: mc.mc_kv_append(
            desc_a, 0, rot_k[r], rot_v[r], B, total_q, cu_q, begin, rot_tables[r], cu_pages)) / 1e6, 1),
        "pack_batch_GBps": round(2 * kv_bytes / rotated(lambda r: mc.mc_kv_pack_batch(
            desc_a, 0, 1, B, rot_tables[r], cu_pages, r_s0, r_s1, send_off, max_range_pages,
            rot_send[r])) / 1e6, 1),
        "unpack_batch_GBps": round(2 * kv_bytes / rotated(lambda r: mc.mc_kv_unpack_batch(
            desc_b, 0, 1, B, rot_tables[r], cu_pages_b, r_s0, r_s1, send_off, max_range_pages,
            rot_send[r])) / 1e6, 1)}
    del rot_send, rot_k, rot_v
    # one layer of a 1000 / 3000 / 5000-token sequence out of one pool and into another (the
    # paper's Table 2 transfers, there with the wire): microseconds for pack + unpack
    t2 = {}
    for tokens in (1000, 3000, 5000):
        pages = up(mi.rng_for(args.seed, tokens).permutation(w.num_pages)[: -(-tokens // 16)]
                   .astype(np.int32))
        buf = send_all[: 2 * tokens * Hkv * D]

        def there_and_back():
            mc.mc_kv_pack_range(desc_a, 0, 1, pages, int(pages.numel()), 0, tokens, buf)
            mc.mc_kv_unpack_range(desc_b, 0, 1, pages, int(pages.numel()), 0, tokens, buf)
        t2[str(tokens)] = round(timed(there_and_back) * 1e3, 1)
    copy["one_layer_pack_plus_unpack_us"] = t2
    if not args.no_copy_sweep:
        # 32768 tokens x 32 layers = 4 GiB of KV between two pools (long-context transfer)
        del pool_a, pool_b, send, send_all
        torch.cuda.empty_cache()
        L, T = 32, 32768
        npg = T // 16
        big = L * npg * 2 * Hkv * 16 * D
        big_a = torch.empty(big, dtype=torch.int16, device=dev)
        big_b = torch.empty(big, dtype=torch.int16, device=dev)
        big_a.view(torch.int32).random_()
        big_s = torch.empty(big, dtype=torch.int16, device=dev)
        da = mc.pool_desc(big_a, L, npg, Hkv, w.dtype)
        dbb = mc.pool_desc(big_b, L, npg, Hkv, w.dtype)
        ta = up(mi.rng_for(args.seed, 78).permutation(npg).astype(np.int32))
        tb = up(mi.rng_for(args.seed, 79).permutation(npg).astype(np.int32))
        payload = L * T * w.token_bytes
        st_p = launch_stats(lambda: mc.mc_kv_pack_range(da, 0, L, ta, npg, 0, T, big_s), 10, 3)
        st_u = launch_stats(lambda: mc.mc_kv_unpack_range(dbb, 0, L, tb, npg, 0, T, big_s), 10, 3)
        ms_p, ms_u = st_p["mean"], st_u["mean"]
        ms_c = timed(lambda: big_b.copy_(big_a), iters=10)
        copy["long_context"] = {
            "payload_GiB": payload / 2**30,
            "pack_GBps": round(2 * payload / ms_p / 1e6, 1),
            "unpack_GBps": round(2 * payload / ms_u / 1e6, 1),
            "pack_frac_of_hbm_peak": round(2 * payload / ms_p / 1e6 / HBM_PEAK_GBS, 3),
            "unpack_frac_of_hbm_peak": round(2 * payload / ms_u / 1e6 / HBM_PEAK_GBS, 3),
            "pack_ms": {k: round(v, 4) for k, v in st_p.items()},
            "unpack_ms": {k: round(v, 4) for k, v in st_u.items()},
            "plain_copy_GBps": round(2 * payload / ms_c / 1e6, 1),
        }
        del big_a, big_b, big_s

    # ---- CPU oracle on this machine's host cores: the attention of the whole workload on all
    #      cores (also the reference for the error of the last step's output), a sample of it
    #      on one core, and the copies ----
    cpu, parity = None, None
    if not args.no_cpu_baseline:
        import ctypes

        import oracle
        shape = oracle.Shape(1, w.num_pages, 16, Hkv, D, w.dtype)
        opool = oracle.new_pool(shape)
        c0 = time.perf_counter()
        for s in range(B):
            oracle.append(opool, shape, 0, kv[s][0], kv[s][1], 0, w.page_tables[s])
        t_append = time.perf_counter() - c0
        cores = len(os.sched_getaffinity(0))
        omp = int(os.environ.get("OMP_NUM_THREADS", cores))
        t_cpu, err_o, err_l = 0.0, 0.0, 0.0
        out_h, lse_h = out.cpu().numpy().view(np.uint16), lse.cpu().numpy().astype(np.float64)
        for s in range(B):
            qs = w.q(s)
            c0 = time.perf_counter()
            ro, rl = oracle.attention(opool, shape, 0, w.page_tables[s], qs, Hq, int(w.b[s]),
                                      int(w.n[s]))
            t_cpu += time.perf_counter() - c0
            lo, hi = int(w.cu_q[s]), int(w.cu_q[s + 1])
            err_o = max(err_o, float(np.max(np.abs(oracle.decode(out_h[lo:hi], w.dtype) - ro))))
            err_l = max(err_l, float(np.max(np.abs(lse_h[lo:hi] - rl))))
        parity = {"rows": "every row and q head of the timed workload",
                  "max_abs_err_O": round(err_o, 6), "max_abs_err_LSE": round(err_l, 8)}
        # one core: 4096 sampled (row, head) pairs of the longest sequence
        gomp = ctypes.CDLL("libgomp.so.1")
        s_long = int(np.argmax(w.n))
        rows, heads = mi.sample_rows(mi.rng_for(args.seed, 93), int(w.n[s_long] - w.b[s_long]),
                                     int(w.b[s_long]), Hq, 4096, 32, num_kv_heads=Hkv)
        fl_one = int(np.sum(4 * D * (int(w.b[s_long]) + rows.astype(np.int64) + 1)))
        gomp.omp_set_num_threads(1)
        c0 = time.perf_counter()
        oracle.attention(opool, shape, 0, w.page_tables[s_long], w.q(s_long), Hq, int(w.b[s_long]),
                         int(w.n[s_long]), sel_rows=rows, sel_heads=heads)
        t_one = time.perf_counter() - c0
        gomp.omp_set_num_threads(min(cores, omp))
        # copies: pack of every sequence out of the pool, unpack into a second one
        opool_b = oracle.new_pool(shape)
        c0 = time.perf_counter()
        bufs = [oracle.pack(opool, shape, 0, 1, w.page_tables[s], 0, int(w.n[s])) for s in range(B)]
        t_pack = time.perf_counter() - c0
        c0 = time.perf_counter()
        for s in range(B):
            oracle.unpack(opool_b, shape, 0, 1, tables_b_np[s], 0, int(w.n[s]), bufs[s])
        t_unpack = time.perf_counter() - c0
        cpu = {"value": round(flops / t_cpu / 1e12, 6), "unit": "TFLOP/s",
               "cores": min(cores, omp), "kind": "oracle",
               "sample": f"attention of the whole workload (all {total_q} new rows x {Hq} heads, "
                         f"{B} sequences), fp64 C/OpenMP oracle, {t_cpu:.1f} s",
               "one_core": {"value": round(fl_one / t_one / 1e12, 6), "unit": "TFLOP/s",
                            "sample": f"{rows.size} sampled (row, head) pairs of the longest "
                                      f"sequence, {t_one:.1f} s",
                            "whole_workload_s_extrapolated": round(t_one * flops / fl_one, 1)},
               "copies_GBps": {"append": round(2 * kv_bytes / t_append / 1e9, 2),
                               "pack": round(2 * kv_bytes / t_pack / 1e9, 2),
                               "unpack": round(2 * kv_bytes / t_unpack / 1e9, 2),
                               "note": "whole workload, one thread (per-token memcpy loops)"}}

    # what the oracle would need for each other config at the rate it reached on this one
    if cpu and other:
        for name, r in other.items():
            if isinstance(r, dict) and "useful_flops" in r:
                r["oracle_whole_workload_s_extrapolated"] = {
                    f"{cpu['cores']}_cores": round(r["useful_flops"] / (cpu["value"] * 1e12), 1),
                    "one_core": round(r["useful_flops"] / (cpu["one_core"]["value"] * 1e12), 1),
                    "basis": "extrapolated from the oracle's measured rate on the timed workload"}

    result = {
        "metric": "prefix-prefill attention TFLOP/s (% MFMA peak); KV pack/unpack GB/s (% HBM)",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-3-8B layer, bf16, 32 q heads / 8 kv heads, "
                               "head_dim 128, page 16, batch 8, prompts U[1024,4096], cached "
                               "fraction U[0,0.75], pages scattered in a 65536-page pool",
                   "seed": args.seed, "total_new_tokens": total_q,
                   "total_tokens": int(np.sum(w.n)),
                   "useful_attention_flops_per_step": flops,
                   "step": "alloc + append + plan + attention + pack_batch + unpack_batch",
                   "streams": 2 if args.overlap else 1},
        "roofline": {"kernel": "attn_kernel<bf16, G=4>", "bound": "mfma",
                     "achieved": round(attn_tflops, 2), "peak": MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(attn_tflops / MFMA_PEAK_TFLOPS, 4),
                     "mfma_alone_measured": mfma_measured,
                     "traffic": MEASURED_TRAFFIC["attention_bytes"]
                     if args.seed == MEASURED_TRAFFIC["seed"] else None,
                     "algorithmic_bytes": 2 * total_q * Hq * D * 2 + total_q * Hq * 4
                     + int(np.sum(w.n)) * w.token_bytes,
                     "traffic_source": "rocprofv3 FETCH_SIZE + WRITE_SIZE of this command with seed "
                                       "2000 (profiles/bench_cfg2_hbm_traffic.md), not measured "
                                       "in this run",
                     "avg_launch_ms": round(attn_ms, 4),
                     "median_launch_ms": round(float(np.median(attn_times)), 4),
                     "min_launch_ms": round(float(attn_times.min()), 4),
                     "frac_of_measured_mfma_rate": round(
                         attn_tflops / mfma_measured["normal_operands_TFLOPs"], 4),
                     "target_frac": 0.5, "target_met": bool(attn_tflops / MFMA_PEAK_TFLOPS >= 0.5)},
        "roofline_copy": None if args.no_copy_sweep else {
            "kernel": "range_copy_kernel<pack>, 32 layers x 32768 tokens", "bound": "hbm",
            "achieved": copy["long_context"]["pack_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": copy["long_context"]["pack_frac_of_hbm_peak"],
            "traffic": MEASURED_TRAFFIC["pack_4GiB_bytes"],
            "traffic_source": "rocprofv3 FETCH_SIZE + WRITE_SIZE (profiles/), not measured in "
                              "this run",
            "algorithmic_bytes": 2 * int(copy["long_context"]["payload_GiB"] * 2**30),
            "target_frac": 0.7,
            "target_met_pack": bool(copy["long_context"]["pack_frac_of_hbm_peak"] >= 0.7),
            "target_met_unpack": bool(copy["long_context"]["unpack_frac_of_hbm_peak"] >= 0.7)},
        "copy": copy,
        "attention_other_workloads": other or None,
        "layer_overlap": overlap,
        "parity_in_this_run": parity,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
