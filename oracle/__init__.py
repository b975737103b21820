"""CPU oracle (fp64, plain C) for the paged KV-cache hot path.

TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the GPU library never does, and this
package imports nothing from the GPU library.

All tensors are numpy arrays.  2-byte data (fp16 / bf16) travels as raw uint16
bit patterns; `dtype` is 0 for IEEE binary16 and 1 for bfloat16.

Layouts (a reading of this build; the paper fixes none of them):
  pool    [layer][page][2 (K,V)][kv_head][slot][head_dim]
  q       [token][q_head][head_dim]            k_new/v_new [token][kv_head][head_dim]
  sendbuf [layer][2][token][kv_head][head_dim]
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F16, BF16 = 0, 1


class Shape(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("num_pages", C.c_int32), ("page_size", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32)]

    def pool_elems(self) -> int:
        return (self.num_layers * self.num_pages * 2 * self.num_kv_heads * self.page_size
                * self.head_dim)

    def pool_dims(self):
        return (self.num_layers, self.num_pages, 2, self.num_kv_heads, self.page_size,
                self.head_dim)


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = C.CDLL(path)
        vp, i32, i64, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        sp = C.POINTER(Shape)
        L.orc_decode_array.argtypes = [vp, i64, i32, vp]
        L.orc_decode_array.restype = None
        L.orc_gather_kv.argtypes = [vp, sp, i32, vp, i32, vp, vp]
        L.orc_attention_rows.argtypes = [vp, sp, i32, vp, vp, i32, i32, i32, f64, i64, vp, vp,
                                         vp, vp]
        L.orc_lse_merge.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp]
        L.orc_lse_merge.restype = None
        L.orc_append.argtypes = [vp, sp, i32, vp, vp, i32, i32, vp]
        L.orc_pack.argtypes = [vp, sp, i32, i32, vp, i32, i32, vp]
        L.orc_unpack.argtypes = [vp, sp, i32, i32, vp, i32, i32, vp]
        L.orc_alloc_create.argtypes = [i32]
        L.orc_alloc_create.restype = vp
        L.orc_alloc_destroy.argtypes = [vp]
        L.orc_alloc_destroy.restype = None
        L.orc_alloc_num_free.argtypes = [vp]
        L.orc_alloc_take.argtypes = [vp, i32, vp]
        L.orc_alloc_give.argtypes = [vp, i32, vp]
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def decode(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact 2-byte -> fp64 conversion."""
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    lib().orc_decode_array(_p(bits), bits.size, dtype, _p(out))
    return out


def new_pool(shape: Shape) -> np.ndarray:
    """Zero pool; pages that are never touched cost no host memory."""
    return np.zeros(shape.pool_elems(), dtype=np.uint16)


def attention(pool, shape: Shape, layer: int, pages, q, num_q_heads: int, begin: int, end: int,
              scale=None, sel_rows=None, sel_heads=None):
    """Attention of tokens [begin,end) of one sequence over its paged KV [0,end).

    With sel_rows/sel_heads None: returns (O [q_len][Hq][D], LSE [q_len][Hq]) as fp64.
    Otherwise computes only the listed (row relative to begin, head) pairs and
    returns (O [n_sel][D], LSE [n_sel]).
    """
    pool, q, pages = _u16(pool), _u16(q), _i32(pages)
    D = shape.head_dim
    q_len = end - begin
    assert q.size == q_len * num_q_heads * D
    need_pages = -(-end // shape.page_size)
    assert pages.size >= need_pages, (pages.size, need_pages)
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    full = sel_rows is None
    if full:
        rr, hh = np.meshgrid(np.arange(q_len, dtype=np.int32),
                             np.arange(num_q_heads, dtype=np.int32), indexing="ij")
        sel_rows, sel_heads = rr.ravel(), hh.ravel()
    sel_rows, sel_heads = _i32(sel_rows), _i32(sel_heads)
    n = sel_rows.size
    assert sel_heads.size == n
    if n:
        assert 0 <= sel_rows.min() and sel_rows.max() < q_len
        assert 0 <= sel_heads.min() and sel_heads.max() < num_q_heads
    out = np.zeros((n, D), dtype=np.float64)
    lse = np.zeros(n, dtype=np.float64)
    rc = lib().orc_attention_rows(_p(pool), C.byref(shape), layer, _p(pages), _p(q), num_q_heads,
                                  begin, end, float(scale), n, _p(sel_rows), _p(sel_heads),
                                  _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle attention failed rc={rc}")
    if full:
        return out.reshape(q_len, num_q_heads, D), lse.reshape(q_len, num_q_heads)
    return out, lse


def lse_merge(o1, l1, o2, l2):
    """Exact merge of two softmax partials over disjoint key sets (natural-log LSE)."""
    o1 = np.ascontiguousarray(o1, dtype=np.float64)
    o2 = np.ascontiguousarray(o2, dtype=np.float64)
    l1 = np.ascontiguousarray(l1, dtype=np.float64)
    l2 = np.ascontiguousarray(l2, dtype=np.float64)
    D = o1.shape[-1]
    n = l1.size
    assert o1.shape == o2.shape and l1.shape == l2.shape and o1.size == n * D
    o = np.empty_like(o1)
    l = np.empty_like(l1)
    lib().orc_lse_merge(_p(o1), _p(l1), _p(o2), _p(l2), n, D, _p(o), _p(l))
    return o, l


def append(pool, shape: Shape, layer: int, k_new, v_new, begin: int, pages) -> None:
    """In place: write K/V of tokens [begin, begin+len) into their (page, slot) entries."""
    assert pool.dtype == np.uint16 and pool.flags.c_contiguous and pool.flags.writeable
    k_new, v_new, pages = _u16(k_new), _u16(v_new), _i32(pages)
    row = shape.num_kv_heads * shape.head_dim
    q_len = k_new.size // row
    assert k_new.size == q_len * row and v_new.size == k_new.size
    assert pages.size >= -(-(begin + q_len) // shape.page_size)
    rc = lib().orc_append(_p(pool), C.byref(shape), layer, _p(k_new), _p(v_new), q_len, begin,
                          _p(pages))
    if rc:
        raise ValueError(f"oracle append failed rc={rc}")


def pack(pool, shape: Shape, layer_begin: int, layer_end: int, pages, s0: int, s1: int):
    """Returns sendbuf [layers][2][s1-s0][Hkv][D] (uint16) gathered from the pages."""
    pool, pages = _u16(pool), _i32(pages)
    assert 0 <= s0 <= s1 and pages.size >= -(-s1 // shape.page_size)
    nl = layer_end - layer_begin
    buf = np.zeros((nl, 2, s1 - s0, shape.num_kv_heads, shape.head_dim), dtype=np.uint16)
    rc = lib().orc_pack(_p(pool), C.byref(shape), layer_begin, layer_end, _p(pages), s0, s1,
                        _p(buf))
    if rc:
        raise ValueError(f"oracle pack failed rc={rc}")
    return buf


def unpack(pool, shape: Shape, layer_begin: int, layer_end: int, pages, s0: int, s1: int,
           buf) -> None:
    """In place: scatter sendbuf into the (page, slot) entries of tokens [s0,s1)."""
    assert pool.dtype == np.uint16 and pool.flags.c_contiguous and pool.flags.writeable
    buf, pages = _u16(buf), _i32(pages)
    nl = layer_end - layer_begin
    assert buf.size == nl * 2 * (s1 - s0) * shape.num_kv_heads * shape.head_dim
    assert 0 <= s0 <= s1 and pages.size >= -(-s1 // shape.page_size)
    rc = lib().orc_unpack(_p(pool), C.byref(shape), layer_begin, layer_end, _p(pages), s0, s1,
                          _p(buf))
    if rc:
        raise ValueError(f"oracle unpack failed rc={rc}")


class Allocator:
    """LIFO free list; first allocations hand out 0, 1, 2, ...; all-or-nothing."""

    def __init__(self, num_pages: int):
        self._h = lib().orc_alloc_create(num_pages)
        if not self._h:
            raise ValueError("bad num_pages")

    def close(self):
        if self._h:
            lib().orc_alloc_destroy(self._h)
            self._h = None

    __del__ = close

    @property
    def num_free(self) -> int:
        return lib().orc_alloc_num_free(self._h)

    def take(self, n: int):
        """Returns a list of n pages, or None when fewer than n are free."""
        out = np.empty(max(n, 1), dtype=np.int32)
        rc = lib().orc_alloc_take(self._h, n, _p(out))
        if rc == 2:
            return None
        if rc:
            raise ValueError("bad argument")
        return out[:n].tolist()

    def give(self, pages) -> bool:
        pages = _i32(pages)
        return lib().orc_alloc_give(self._h, pages.size, _p(pages)) == 0


# ---- host arithmetic of remote_send (paper Sec. 3.5, the two prefix-matching cases) ----
def send_plan(sender_match: int, receiver_match: int, begin: int, end: int) -> dict:
    """Token by token.  Token t of the prompt is on the sender if t < sender_match and on the
    receiver if t < receiver_match.  The receiver needs t if begin <= t < end and it does not
    have it.  A needed token the sender has is copied; if any needed token is not on the sender,
    the sender computes every token below `end` that it lacks (attention needs the whole
    context) and sends the needed ones among them.  Returns the three token sets as sorted
    lists under "copy", "prefill", "send"."""
    needed = [t for t in range(begin, end) if not t < receiver_match]
    copy = [t for t in needed if t < sender_match]
    must_compute = any(not t < sender_match for t in needed)
    prefill = [t for t in range(end) if not t < sender_match] if must_compute else []
    send = [t for t in needed if t in set(prefill)]
    return {"copy": copy, "prefill": prefill, "send": send}


def addr_runs(pages) -> list:
    """Run-length form of a page list: maximal runs of consecutive ids as (first, count)."""
    runs = []
    for p in pages:
        if runs and runs[-1][0] + runs[-1][1] == p:
            runs[-1] = (runs[-1][0], runs[-1][1] + 1)
        else:
            runs.append((int(p), 1))
    return runs


# ---- context cache index behind prep_recv (paper Sec. 3.1, Sec. 3.2) ----
class PrefixIndex:
    """Which page holds the KV of which 16-token block of which token prefix, by brute force:
    a dictionary from the whole token prefix up to and including a block to that block's page.
    A block recorded earlier keeps its page."""

    def __init__(self, page_size: int = 16):
        self.page_size = page_size
        self.page_of_prefix = {}

    def insert(self, tokens, pages):
        P = self.page_size
        for k in range(len(tokens) // P):
            self.page_of_prefix.setdefault(tuple(tokens[: (k + 1) * P]), int(pages[k]))

    def match(self, tokens):
        """(match_len, pages): the longest run of whole pages from the start that are recorded."""
        P, pages = self.page_size, []
        for k in range(len(tokens) // P):
            key = tuple(tokens[: (k + 1) * P])
            if key not in self.page_of_prefix:
                break
            pages.append(self.page_of_prefix[key])
        return len(pages) * P, pages


def prep_recv(index: PrefixIndex, alloc: Allocator, prompt, end: int):
    """prep_recv(prompt, end): matched pages of prompt[0, end) followed by freshly allocated
    ones for the rest; (pages, match_len), or None when the allocator cannot supply them."""
    match_len, pages = index.match(list(prompt[:end]))
    need = -(-end // index.page_size) - len(pages)
    fresh = alloc.take(need)
    if fresh is None:
        return None
    return pages + fresh, match_len


# ---- fork_sequence (paper Sec. 3.5) ----
def fork_sequence(alloc: Allocator, parent_pages, n_tokens: int, page_size: int = 16):
    """The child's page list for the parent's first n_tokens tokens: whole pages shared, a fresh
    page for a partly filled last one; plus the copy to make as (src page, dst page, slots), or
    (-1, -1, 0).  None when the allocator has no page left."""
    whole, rest = divmod(n_tokens, page_size)
    child = [int(p) for p in parent_pages[:whole]]
    if rest == 0:
        return child, (-1, -1, 0)
    fresh = alloc.take(1)
    if fresh is None:
        return None
    return child + fresh, (int(parent_pages[whole]), fresh[0], rest)


def copy_page(pool, shape: Shape, layer_begin: int, layer_end: int, src: int, dst: int,
              slots: int) -> None:
    """In place: slots [0, slots) of page src to page dst, K and V, every head, given layers."""
    view = pool.reshape(shape.pool_dims())      # [layer][page][K|V][head][slot][d]
    view[layer_begin:layer_end, dst, :, :, :slots, :] = view[layer_begin:layer_end, src, :, :, :slots, :]
