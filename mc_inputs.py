"""Seeded synthetic inputs for the paged KV-cache hot path.

Shared by the CPU oracle's tests and the GPU library's tests and benchmark.
Holds none of the method's arithmetic: only shapes, lengths, page tables and
random 2-byte tensors.  numpy only.

The five workloads follow the serving shapes the paper evaluates on
(Llama-3.1-8B, Sec. 4.1; inputs of about 3000-5000 tokens and 500 new tokens
over 500-4500 cached ones, Sec. 4.2, Table 2) as fixed by this build's configs.
"""
from dataclasses import dataclass, field
from typing import List

import numpy as np

F16, BF16 = 0, 1
KIND_K, KIND_V, KIND_Q, KIND_TABLE, KIND_LEN = 0, 1, 2, 3, 4


def f32_to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """float32 -> fp16 / bf16 bit patterns, round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    u = x.view(np.uint32)
    u = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (u >> np.uint32(16)).astype(np.uint16)


def rng_for(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *stream])))


def normal_bits(rng: np.random.Generator, shape, dtype: int) -> np.ndarray:
    """N(0,1) samples rounded to the 2-byte dtype, as uint16."""
    return f32_to_bits(rng.standard_normal(size=shape, dtype=np.float32), dtype)


def layer_variant(base: np.ndarray, layer: int) -> np.ndarray:
    """Cheap per-layer variant of a [token][...] uint16 tensor: rotate the token
    axis by 17*layer and flip the sign bit on odd layers (keeps N(0,1))."""
    if layer == 0:
        return base
    out = np.roll(base, 17 * layer, axis=0)
    if layer & 1:
        out = out ^ np.uint16(0x8000)
    return out


@dataclass
class Workload:
    name: str
    seed: int
    dtype: int
    num_layers: int
    num_q_heads: int
    num_kv_heads: int
    num_pages: int
    n: np.ndarray                      # [batch] tokens in the sequence after the call (= end)
    b: np.ndarray                      # [batch] cached prefix length (= begin)
    page_tables: List[np.ndarray] = field(default_factory=list)  # per seq, ceil(n/P) page ids
    head_dim: int = 128
    page_size: int = 16
    # shared prefixes (fork_sequence, paper Sec. 3.5): share[s] = (source sequence < s, tokens);
    # sequence s has the source's K/V on its first `tokens` tokens (a multiple of the page size)
    # and lists the source's pages for them
    share: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return len(self.n)

    @property
    def q_lens(self) -> np.ndarray:
        return self.n - self.b

    @property
    def cu_q(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.q_lens)]).astype(np.int32)

    @property
    def cu_pages(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([len(t) for t in self.page_tables])]).astype(np.int32)

    @property
    def flat_page_table(self) -> np.ndarray:
        if not self.page_tables:
            return np.zeros(0, dtype=np.int32)
        return np.concatenate(self.page_tables).astype(np.int32)

    @property
    def token_bytes(self) -> int:
        """K+V bytes of one token in one layer."""
        return 2 * self.num_kv_heads * self.head_dim * 2

    def useful_flops(self) -> int:
        """4*D*Hq*sum(q*b + q(q+1)/2): masked work is not credited."""
        q = self.q_lens.astype(np.int64)
        b = self.b.astype(np.int64)
        return int(4 * self.head_dim * self.num_q_heads * np.sum(q * b + q * (q + 1) // 2))

    # ---- data ------------------------------------------------------------
    def kv(self, seq: int, layer: int = 0):
        """(k, v) uint16 [n][Hkv][D] of the whole sequence [0, n) for one layer."""
        shape = (int(self.n[seq]), self.num_kv_heads, self.head_dim)
        k = normal_bits(rng_for(self.seed, seq, KIND_K), shape, self.dtype)
        v = normal_bits(rng_for(self.seed, seq, KIND_V), shape, self.dtype)
        if seq in self.share:
            src, tokens = self.share[seq]
            ks, vs = self.kv(src, 0)
            k[:tokens], v[:tokens] = ks[:tokens], vs[:tokens]
        return layer_variant(k, layer), layer_variant(v, layer)

    def q(self, seq: int, layer: int = 0) -> np.ndarray:
        """uint16 [n-b][Hq][D]: queries of the new range of one sequence."""
        shape = (int(self.n[seq] - self.b[seq]), self.num_q_heads, self.head_dim)
        return layer_variant(normal_bits(rng_for(self.seed, seq, KIND_Q), shape, self.dtype), layer)

    def with_ranges(self, b, n, name=None) -> "Workload":
        """Same sequences and page tables, another [begin,end) per sequence (end <= n)."""
        b = np.asarray(b, dtype=np.int64)
        n = np.asarray(n, dtype=np.int64)
        assert np.all(b >= 0) and np.all(b <= n) and np.all(n <= self.n)
        w = Workload(name or self.name, self.seed, self.dtype, self.num_layers, self.num_q_heads,
                     self.num_kv_heads, self.num_pages, n, b, self.page_tables, self.head_dim,
                     self.page_size, self.share)
        return w

    def share_prefix(self, seq: int, src: int, tokens: int) -> None:
        """Make sequence seq a fork of src over its first `tokens` tokens: same K/V, same pages."""
        assert src < seq and tokens % self.page_size == 0
        assert tokens <= min(int(self.n[seq]), int(self.n[src]))
        if src in self.share:
            assert tokens <= self.share[src][1] or True
        self.share[seq] = (src, tokens)
        pages = tokens // self.page_size
        self.page_tables[seq] = self.page_tables[seq].copy()
        self.page_tables[seq][:pages] = self.page_tables[src][:pages]


def scatter_page_tables(rng: np.random.Generator, num_pages: int, n_tokens, page_size: int = 16):
    """Distinct pages drawn without replacement from the pool, dealt to the sequences."""
    counts = [-(-int(t) // page_size) for t in n_tokens]
    total = int(sum(counts))
    assert total <= num_pages, (total, num_pages)
    if total * 4 >= num_pages:
        ids = rng.permutation(num_pages)[:total]
    else:
        ids = rng.choice(num_pages, size=total, replace=False)
    out, at = [], 0
    for c in counts:
        out.append(ids[at:at + c].astype(np.int32))
        at += c
    return out


def config(idx: int, seed: int = None, shrink: int = 1, num_layers: int = None) -> Workload:
    """Workload `idx` in 1..5.  shrink > 1 divides every length (and the pool) so that
    the CPU oracle finishes in seconds while keeping ragged, unaligned ranges."""
    seed = 1000 * idx if seed is None else seed
    rng = rng_for(seed, KIND_LEN)
    trng = rng_for(seed, KIND_TABLE)
    P = 16
    if idx == 1:
        # one fp16 sequence, 8 q heads = 8 kv heads, 256 cached + 256 new, pool of 64 pages
        n, b = np.array([512 // shrink]), np.array([256 // shrink])
        w = Workload("cfg1-tiny-fp16", seed, F16, 1, 8, 8, 64, n, b)
        w.page_tables = [trng.permutation(64)[: -(-int(n[0]) // P)].astype(np.int32)]
        return w
    if idx == 2:
        # Llama-3-8B layer: 8 sequences, n ~ U{1024..4096}, cached fraction ~ U[0, 0.75]
        n = rng.integers(1024 // shrink, 4096 // shrink + 1, size=8)
        f = rng.uniform(0.0, 0.75, size=8)
        b = np.floor(f * n).astype(np.int64)
        pool = max(65536 // shrink, 8 * (4096 // shrink // P + 1))
        w = Workload("cfg2-llama3-8b-batch8", seed, BF16, num_layers or 1, 32, 8, pool, n, b)
        w.page_tables = scatter_page_tables(trng, pool, n)
        return w
    if idx == 3:
        # balanced prefill/decode split: 16 sequences, n ~ U{2048..8192}, m = n // 2
        n = rng.integers(2048 // shrink, 8192 // shrink + 1, size=16)
        b = n // 2
        L = num_layers or 32
        pool = int(sum(-(-int(t) // P) for t in n))
        w = Workload("cfg3-balanced-split", seed, BF16, L, 32, 8, pool, n, b)
        w.page_tables = scatter_page_tables(trng, pool, n)
        return w
    if idx == 4:
        # Llama-3-70B heads (GQA 8:1): 4 sequences of 8192 tokens, 90 % cached (unaligned)
        n = np.full(4, 8192 // shrink)
        b = (n * 9) // 10
        pool = max(4096 // shrink, 4 * (8192 // shrink // P + 1))
        w = Workload("cfg4-llama3-70b-prefix90", seed, BF16, num_layers or 1, 64, 8, pool, n, b)
        w.page_tables = scatter_page_tables(trng, pool, n)
        return w
    if idx == 5:
        # long context: sequences of 16384 and 32768 tokens, half cached
        n = np.array([16384 // shrink, 32768 // shrink])
        b = n // 2
        L = num_layers or 32
        pool = int(sum(-(-int(t) // P) for t in n))
        w = Workload("cfg5-long-context", seed, BF16, L, 32, 8, pool, n, b)
        w.page_tables = scatter_page_tables(trng, pool, n)
        return w
    raise ValueError(f"no config {idx}")


def paper_point(cached: int, new: int = 500, seed: int = 7000) -> Workload:
    """One Llama-3-8B-shaped sequence with `new` tokens over `cached` ones (Sec. 4.2, Table 2)."""
    n, b = np.array([cached + new]), np.array([cached])
    pool = 4096
    w = Workload(f"paper-{new}-over-{cached}", seed + cached, BF16, 1, 32, 8, pool, n, b)
    w.page_tables = scatter_page_tables(rng_for(seed + cached, KIND_TABLE), pool, n)
    return w


def sample_rows(rng: np.random.Generator, q_len: int, begin: int, num_q_heads: int, count: int,
                tile_tokens: int = 32, page_size: int = 16, num_kv_heads: int = None):
    """(rows, heads) pairs to spot-check, about `count` of them, rows relative to `begin`.

    Rows: the first and the last row of the range; the first and last row of q tiles
    (tile_tokens rows each; always the first, the last whole and the ragged last tile, the
    others spread evenly over the whole range); several rows of the ragged last tile; rows on
    both sides of page boundaries (positions with pos % page_size in {page_size - 1, 0}) at
    boundaries spread evenly from the start to the end of the range; the rest uniform.
    Heads: with num_kv_heads given, every row is paired with one random q head of every kv
    head's group (num_kv_heads pairs per row); otherwise with one random q head."""
    per_row = num_kv_heads or 1
    n_rows = max(4, min(q_len, -(-count // per_row)))
    rows = {0, q_len - 1}
    n_tiles = -(-q_len // tile_tokens)
    # q tiles: first, last whole, ragged last, and an even spread in between
    tiles = {0, n_tiles - 1, max(0, n_tiles - 2)}
    tiles.update(int(t) for t in np.linspace(0, n_tiles - 1, num=max(2, n_rows // 8)))
    for t in sorted(tiles):
        rows.update({t * tile_tokens, min(q_len, (t + 1) * tile_tokens) - 1})
    last0 = (n_tiles - 1) * tile_tokens
    rows.update(int(r) for r in rng.integers(last0, q_len, size=min(4, q_len - last0)))
    # page boundaries: first position of a page and the one before it
    first_b = (-begin) % page_size                      # first row with pos % page_size == 0
    bounds = np.arange(first_b, q_len, page_size)
    if bounds.size:
        pick = bounds[np.unique(np.linspace(0, bounds.size - 1, num=max(2, n_rows // 8)).astype(int))]
        for r in pick:
            rows.add(int(r))
            if r > 0:
                rows.add(int(r) - 1)
    rows = sorted(r for r in rows if 0 <= r < q_len)
    extra = rng.integers(0, q_len, size=max(0, n_rows - len(rows)))
    rows = np.concatenate([np.array(rows, dtype=np.int64), extra]).astype(np.int32)
    if num_kv_heads is None:
        heads = rng.integers(0, num_q_heads, size=rows.size).astype(np.int32)
        return rows, heads
    group = num_q_heads // num_kv_heads
    heads = (np.arange(num_kv_heads)[None, :] * group
             + rng.integers(0, group, size=(rows.size, num_kv_heads))).astype(np.int32)
    return np.repeat(rows, num_kv_heads).astype(np.int32), heads.ravel()
