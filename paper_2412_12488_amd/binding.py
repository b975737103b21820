"""ctypes binding of libmc_kv.so: the same names as include/mc_kv.h, argument
marshalling only.  Device buffers are torch tensors (or raw integer addresses);
every step of the path runs in the library's HIP kernels.  There is no fallback:
if the library is missing or a call fails, this raises."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmc_kv.so")

MC_OK, MC_ERR_INVALID, MC_ERR_NO_PAGES, MC_ERR_RANGE, MC_ERR_ALIAS, MC_ERR_UNSUPPORTED, \
    MC_ERR_HIP = range(7)
MC_F16, MC_BF16 = 0, 1

EXPORTS = [
    "mc_status_string", "mc_abi_version",
    "mc_kv_allocator_create", "mc_kv_allocator_destroy", "mc_kv_alloc_pages", "mc_kv_free_pages",
    "mc_kv_allocator_num_free", "mc_kv_check_page_table",
    "mc_kv_copy_check", "mc_kv_append", "mc_kv_append_send", "mc_attn_workspace_size", "mc_attn_plan", "mc_attn_plan_ahead", "mc_attn_plan_check",
    "mc_prefix_prefill_attn", "mc_prefix_prefill_attn_noalloc", "mc_kv_pack_range", "mc_kv_unpack_range",
    "mc_kv_pack_batch", "mc_kv_unpack_batch",
    "mc_plan_remote_send", "mc_addr_compress", "mc_addr_expand",
    "mc_prefix_index_create", "mc_prefix_index_destroy", "mc_prefix_index_insert",
    "mc_prefix_index_match", "mc_prep_recv", "mc_kv_fork_sequence", "mc_kv_copy_page",
]


class McError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


class mc_send_plan(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("copy_begin", "copy_end", "prefill_begin", "prefill_end",
                                         "send_begin", "send_end")]


class mc_pool_desc(C.Structure):
    _fields_ = [("base", C.c_void_p), ("num_layers", C.c_int32), ("num_pages", C.c_int32),
                ("page_size", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("skipped", C.c_void_p)]


_lib = None


def lib():
    """Load the built library; build it only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    pd = C.POINTER(mc_pool_desc)
    L.mc_status_string.argtypes = [i32]
    L.mc_status_string.restype = C.c_char_p
    L.mc_abi_version.argtypes = []
    L.mc_kv_allocator_create.argtypes = [i32, C.POINTER(vp)]
    L.mc_kv_allocator_destroy.argtypes = [vp]
    L.mc_kv_alloc_pages.argtypes = [vp, i32, C.POINTER(i32)]
    L.mc_kv_free_pages.argtypes = [vp, i32, C.POINTER(i32)]
    L.mc_kv_allocator_num_free.argtypes = [vp, C.POINTER(i32)]
    L.mc_kv_check_page_table.argtypes = [C.POINTER(i32), i64, i32]
    L.mc_kv_copy_check.argtypes = [pd, C.POINTER(i32), vp]
    L.mc_kv_append.argtypes = [pd, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp]
    L.mc_kv_append_send.argtypes = [pd, i32, vp, vp, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp,
                                    vp]
    L.mc_attn_workspace_size.argtypes = [i32, i32, i32, i32]
    L.mc_attn_workspace_size.restype = sz
    L.mc_attn_plan.argtypes = [pd, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.mc_attn_plan_ahead.argtypes = [pd, i32, i32, i32, vp, vp, vp, vp, i32, vp, sz, vp]
    L.mc_attn_plan_check.argtypes = [vp, vp]
    L.mc_prefix_prefill_attn.argtypes = [pd, i32, vp, i32, i32, i32, vp, vp, vp, vp, C.c_float,
                                         vp, vp, vp, sz, vp]
    L.mc_prefix_prefill_attn_noalloc.argtypes = [pd, i32, vp, i32, i32, i32, vp, vp, vp, vp,
                                                 C.c_float, vp, vp, vp]
    L.mc_kv_pack_range.argtypes = [pd, i32, i32, vp, i32, i32, i32, vp, vp]
    L.mc_kv_unpack_range.argtypes = [pd, i32, i32, vp, i32, i32, i32, vp, vp]
    L.mc_kv_pack_batch.argtypes = [pd, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp]
    L.mc_kv_unpack_batch.argtypes = [pd, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp]
    L.mc_plan_remote_send.argtypes = [i32, i32, i32, i32, C.POINTER(mc_send_plan)]
    L.mc_addr_compress.argtypes = [C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i32)]
    L.mc_addr_expand.argtypes = [C.POINTER(i32), i32, C.POINTER(i32), i32, C.POINTER(i32)]
    L.mc_prefix_index_create.argtypes = [C.POINTER(vp)]
    L.mc_prefix_index_destroy.argtypes = [vp]
    L.mc_prefix_index_insert.argtypes = [vp, C.POINTER(i32), i32, C.POINTER(i32)]
    L.mc_prefix_index_match.argtypes = [vp, C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i32)]
    L.mc_prep_recv.argtypes = [vp, vp, C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i32)]
    L.mc_kv_fork_sequence.argtypes = [vp, C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i32),
                                      C.POINTER(i32), C.POINTER(i32)]
    L.mc_kv_copy_page.argtypes = [pd, i32, i32, i32, i32, i32, vp]
    _lib = L
    return L


def _ptr(x):
    """Device (or host) address of a tensor, an int address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str):
    if status != MC_OK:
        raise McError(status, where)


def _i32_array(values):
    arr = (C.c_int32 * max(len(values), 1))(*[int(v) for v in values])
    return arr


def status_string(status: int) -> str:
    return lib().mc_status_string(int(status)).decode()


mc_status_string = status_string


def mc_abi_version() -> int:
    return lib().mc_abi_version()


def pool_desc(base, num_layers, num_pages, num_kv_heads, dtype, page_size=16, head_dim=128,
              skipped=None):
    """skipped: optional device int32 counter (zeroed by the caller) for mc_kv_copy_check."""
    return mc_pool_desc(_ptr(base), num_layers, num_pages, page_size, num_kv_heads, head_dim, dtype,
                        _ptr(skipped))


# ---- allocator (host) ---------------------------------------------------------
def mc_kv_allocator_create(num_pages: int):
    h = C.c_void_p()
    _check(lib().mc_kv_allocator_create(num_pages, C.byref(h)), "mc_kv_allocator_create")
    return h


def mc_kv_allocator_destroy(alloc):
    _check(lib().mc_kv_allocator_destroy(alloc), "mc_kv_allocator_destroy")


def mc_kv_alloc_pages(alloc, n: int):
    out = (C.c_int32 * max(n, 1))()
    _check(lib().mc_kv_alloc_pages(alloc, n, out), "mc_kv_alloc_pages")
    return list(out[:n])


def mc_kv_free_pages(alloc, pages):
    _check(lib().mc_kv_free_pages(alloc, len(pages), _i32_array(pages)), "mc_kv_free_pages")


def mc_kv_allocator_num_free(alloc) -> int:
    n = C.c_int32()
    _check(lib().mc_kv_allocator_num_free(alloc, C.byref(n)), "mc_kv_allocator_num_free")
    return n.value


def mc_kv_check_page_table(pages, num_pages: int) -> int:
    """Returns the status code (MC_OK / MC_ERR_RANGE / MC_ERR_ALIAS) instead of raising."""
    return lib().mc_kv_check_page_table(_i32_array(pages), len(pages), num_pages)


# ---- device calls -------------------------------------------------------------
def mc_kv_copy_check(pool: mc_pool_desc, stream=None) -> int:
    """Status code (MC_OK / MC_ERR_RANGE / ...) and the count, as (status, skipped); does not
    raise on MC_ERR_RANGE, since the count is the point."""
    n = C.c_int32(0)
    st = lib().mc_kv_copy_check(C.byref(pool), C.byref(n), _stream(stream))
    if st not in (MC_OK, MC_ERR_RANGE):
        raise McError(st, "mc_kv_copy_check")
    return st, n.value


def mc_kv_append(pool: mc_pool_desc, layer, k_new, v_new, batch, total_q, cu_q, begin,
                 page_table, cu_pages, stream=None):
    _check(lib().mc_kv_append(C.byref(pool), layer, _ptr(k_new), _ptr(v_new), batch, total_q,
                              _ptr(cu_q), _ptr(begin), _ptr(page_table), _ptr(cu_pages),
                              _stream(stream)), "mc_kv_append")


def mc_kv_append_send(pool: mc_pool_desc, layer, k_new, v_new, batch, total_q, cu_q, begin,
                      page_table, cu_pages, send_layer_begin, s0, s1, buf_offset, sendbuf,
                      stream=None):
    _check(lib().mc_kv_append_send(C.byref(pool), layer, _ptr(k_new), _ptr(v_new), batch, total_q,
                                   _ptr(cu_q), _ptr(begin), _ptr(page_table), _ptr(cu_pages),
                                   send_layer_begin, _ptr(s0), _ptr(s1), _ptr(buf_offset),
                                   _ptr(sendbuf), _stream(stream)), "mc_kv_append_send")


def mc_attn_workspace_size(batch, total_q, num_q_heads, num_kv_heads) -> int:
    return lib().mc_attn_workspace_size(batch, total_q, num_q_heads, num_kv_heads)


def mc_attn_plan(pool: mc_pool_desc, num_q_heads, batch, total_q, cu_q, begin, page_table,
                 cu_pages, workspace, workspace_bytes, stream=None):
    _check(lib().mc_attn_plan(C.byref(pool), num_q_heads, batch, total_q, _ptr(cu_q), _ptr(begin),
                              _ptr(page_table), _ptr(cu_pages), _ptr(workspace), workspace_bytes,
                              _stream(stream)), "mc_attn_plan")


def mc_attn_plan_ahead(pool: mc_pool_desc, num_q_heads, batch, total_q, cu_q, begin, page_table,
                       cu_pages, ahead_tokens, workspace, workspace_bytes, stream=None):
    _check(lib().mc_attn_plan_ahead(C.byref(pool), num_q_heads, batch, total_q, _ptr(cu_q),
                                    _ptr(begin), _ptr(page_table), _ptr(cu_pages), ahead_tokens,
                                    _ptr(workspace), workspace_bytes, _stream(stream)),
           "mc_attn_plan_ahead")


def mc_attn_plan_check(workspace, stream=None):
    _check(lib().mc_attn_plan_check(_ptr(workspace), _stream(stream)), "mc_attn_plan_check")


def mc_prefix_prefill_attn(pool: mc_pool_desc, layer, q, num_q_heads, batch, total_q, cu_q, begin,
                           page_table, cu_pages, sm_scale, out, lse, workspace, workspace_bytes,
                           stream=None):
    _check(lib().mc_prefix_prefill_attn(C.byref(pool), layer, _ptr(q), num_q_heads, batch, total_q,
                                        _ptr(cu_q), _ptr(begin), _ptr(page_table), _ptr(cu_pages),
                                        float(sm_scale), _ptr(out), _ptr(lse), _ptr(workspace),
                                        workspace_bytes, _stream(stream)),
           "mc_prefix_prefill_attn")


def mc_prefix_prefill_attn_noalloc(pool: mc_pool_desc, layer, q, num_q_heads, batch, total_q, cu_q,
                                   begin, page_table, cu_pages, sm_scale, out, lse, stream=None):
    _check(lib().mc_prefix_prefill_attn_noalloc(C.byref(pool), layer, _ptr(q), num_q_heads, batch,
                                                total_q, _ptr(cu_q), _ptr(begin),
                                                _ptr(page_table), _ptr(cu_pages), float(sm_scale),
                                                _ptr(out), _ptr(lse), _stream(stream)),
           "mc_prefix_prefill_attn_noalloc")


def mc_kv_pack_range(pool: mc_pool_desc, layer_begin, layer_end, pages, n_table_pages, s0, s1,
                     sendbuf, stream=None):
    _check(lib().mc_kv_pack_range(C.byref(pool), layer_begin, layer_end, _ptr(pages),
                                  n_table_pages, s0, s1, _ptr(sendbuf), _stream(stream)),
           "mc_kv_pack_range")


def mc_kv_unpack_range(pool: mc_pool_desc, layer_begin, layer_end, pages, n_table_pages, s0, s1,
                       sendbuf, stream=None):
    _check(lib().mc_kv_unpack_range(C.byref(pool), layer_begin, layer_end, _ptr(pages),
                                    n_table_pages, s0, s1, _ptr(sendbuf), _stream(stream)),
           "mc_kv_unpack_range")


def mc_kv_pack_batch(pool: mc_pool_desc, layer_begin, layer_end, batch, page_table, cu_pages, s0,
                     s1, buf_offset, max_range_pages, sendbuf, stream=None):
    _check(lib().mc_kv_pack_batch(C.byref(pool), layer_begin, layer_end, batch, _ptr(page_table),
                                  _ptr(cu_pages), _ptr(s0), _ptr(s1), _ptr(buf_offset),
                                  max_range_pages, _ptr(sendbuf), _stream(stream)),
           "mc_kv_pack_batch")


def mc_kv_unpack_batch(pool: mc_pool_desc, layer_begin, layer_end, batch, page_table, cu_pages,
                       s0, s1, buf_offset, max_range_pages, sendbuf, stream=None):
    _check(lib().mc_kv_unpack_batch(C.byref(pool), layer_begin, layer_end, batch,
                                    _ptr(page_table), _ptr(cu_pages), _ptr(s0), _ptr(s1),
                                    _ptr(buf_offset), max_range_pages, _ptr(sendbuf),
                                    _stream(stream)), "mc_kv_unpack_batch")


def mc_plan_remote_send(sender_match, receiver_match, begin, end) -> dict:
    """Token ranges (begin, end) under "copy", "prefill", "send"."""
    p = mc_send_plan()
    _check(lib().mc_plan_remote_send(sender_match, receiver_match, begin, end, C.byref(p)),
           "mc_plan_remote_send")
    return {"copy": (p.copy_begin, p.copy_end), "prefill": (p.prefill_begin, p.prefill_end),
            "send": (p.send_begin, p.send_end)}


def mc_addr_compress(pages):
    """Page list -> list of (first page, count) runs."""
    n = len(pages)
    arr, runs, nr = _i32_array(pages), (C.c_int32 * (2 * max(n, 1)))(), C.c_int32(0)
    _check(lib().mc_addr_compress(arr, n, runs, C.byref(nr)), "mc_addr_compress")
    return [(runs[2 * i], runs[2 * i + 1]) for i in range(nr.value)]


def mc_addr_expand(runs, capacity=None):
    """List of (first page, count) runs -> page list."""
    flat = [int(x) for r in runs for x in r]
    if capacity is None:
        capacity = max(0, sum(max(0, int(c)) for _, c in runs))
    out, n = (C.c_int32 * max(capacity, 1))(), C.c_int32(0)
    _check(lib().mc_addr_expand(_i32_array(flat), len(runs), out, capacity, C.byref(n)),
           "mc_addr_expand")
    return [out[i] for i in range(n.value)]


def mc_prefix_index_create():
    h = C.c_void_p()
    _check(lib().mc_prefix_index_create(C.byref(h)), "mc_prefix_index_create")
    return h


def mc_prefix_index_destroy(index):
    _check(lib().mc_prefix_index_destroy(index), "mc_prefix_index_destroy")


def mc_prefix_index_insert(index, tokens, pages):
    _check(lib().mc_prefix_index_insert(index, _i32_array(tokens), len(tokens), _i32_array(pages)),
           "mc_prefix_index_insert")


def mc_prefix_index_match(index, tokens):
    """Returns (match_len, pages of the matched whole pages)."""
    out, m = (C.c_int32 * max(len(tokens) // 16, 1))(), C.c_int32(0)
    _check(lib().mc_prefix_index_match(index, _i32_array(tokens), len(tokens), out, C.byref(m)),
           "mc_prefix_index_match")
    return m.value, [out[i] for i in range(m.value // 16)]


def mc_prep_recv(index, alloc, prompt, end):
    """Returns (page list for prompt[0, end): matched pages then fresh ones, match_len)."""
    out, m = (C.c_int32 * max(-(-end // 16), 1))(), C.c_int32(0)
    _check(lib().mc_prep_recv(index, alloc, _i32_array(prompt), end, out, C.byref(m)),
           "mc_prep_recv")
    return [out[i] for i in range(-(-end // 16))], m.value


def mc_kv_fork_sequence(alloc, parent_pages, n_tokens):
    """Returns (child page list, (src page, dst page, slots) of the copy still to be made)."""
    n = -(-n_tokens // 16)
    out = (C.c_int32 * max(n, 1))()
    src, dst, slots = C.c_int32(-1), C.c_int32(-1), C.c_int32(0)
    _check(lib().mc_kv_fork_sequence(alloc, _i32_array(parent_pages), n_tokens, out, C.byref(src),
                                     C.byref(dst), C.byref(slots)), "mc_kv_fork_sequence")
    return [out[i] for i in range(n)], (src.value, dst.value, slots.value)


def mc_kv_copy_page(pool: mc_pool_desc, layer_begin, layer_end, src_page, dst_page, slots,
                    stream=None):
    _check(lib().mc_kv_copy_page(C.byref(pool), layer_begin, layer_end, src_page, dst_page, slots,
                                 _stream(stream)), "mc_kv_copy_page")
