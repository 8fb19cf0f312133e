"""ctypes binding of libtwilight.so - argument marshalling only.

Every function has the name and argument order of its C entry point
(include/twilight.h).  Tensors are torch CUDA tensors used purely as device
memory; the current torch stream is passed as the HIP stream.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("TWILIGHT_LIB") or os.path.join(_PKG, "libtwilight.so")   # override: tuning builds

TW_WS_SELECT, TW_WS_PRUNE, TW_WS_DECODE, TW_WS_DECODE_PER_HEAD, TW_WS_PRUNE_TOKENS, TW_WS_DS_SELECT, TW_WS_SELECT_PRUNE = 0, 1, 2, 3, 4, 5, 6
TW_STATUS_UNION_TRUNCATED, TW_STATUS_KEPT_TRUNCATED = 1, 2
TW_STATIC_SELECT_WS_BYTES = 8 << 20
KERNEL_NAMES = ["kquant_append", "page_score", "page_select", "int4_score", "topp", "union",
                "sparse_decode", "combine", "score_topp", "select_score_topp"]

_vp, _i32, _i64, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t


class twilight_kv_t(ctypes.Structure):
    _fields_ = [("batch", _i32), ("num_q_heads", _i32), ("num_kv_heads", _i32), ("head_dim", _i32),
                ("page_size", _i32), ("quant_group", _i32), ("max_pages_per_seq", _i32), ("quant_bits", _i32),
                ("num_pool_pages", _i64), ("page_table", _vp), ("seq_lens", _vp), ("k_pool", _vp),
                ("v_pool", _vp), ("kq_pool", _vp), ("kq_meta", _vp), ("page_minmax", _vp)]


class TwilightError(RuntimeError):
    pass


_lib = None


def lib():
    """Load libtwilight.so (built by paper_2502_02770_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise TwilightError("libtwilight.so not found at %s - run `python -m paper_2502_02770_amd.build`" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    kvp = ctypes.POINTER(twilight_kv_t)
    L.twilight_kquant_append.argtypes = [kvp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]
    L.twilight_select_pages.argtypes = [kvp, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp]
    L.twilight_select_pages_static.argtypes = [kvp, _vp, _vp, _vp, _vp, _i32, _vp]
    L.twilight_int4_score.argtypes = [kvp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]
    L.twilight_ds_select_tokens.argtypes = [kvp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp]
    L.twilight_append_select.argtypes = [kvp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp]
    L.twilight_select_prune.argtypes = [kvp, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
    L.twilight_topp_prune.argtypes = [kvp, _vp, _vp, _vp, _i32, _f32, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
    L.twilight_int4_score_tokens.argtypes = [kvp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]
    L.twilight_topp_prune_tokens.argtypes = [kvp, _vp, _vp, _vp, _i32, _f32, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
    L.twilight_sparse_decode.argtypes = [kvp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
    L.twilight_sparse_decode_per_head.argtypes = [kvp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
    L.twilight_workspace_bytes.argtypes = [ctypes.c_int, kvp, _i32, _i32]
    L.twilight_pinned_device_pointer.argtypes = [_vp, ctypes.POINTER(_vp)]
    L.twilight_pinned_device_pointer.restype = ctypes.c_int
    L.twilight_workspace_bytes.restype = _sz
    L.twilight_strerror.argtypes = [ctypes.c_int]
    L.twilight_strerror.restype = ctypes.c_char_p
    L.twilight_abi_version.restype = ctypes.c_int
    L.twilight_prof_enable.argtypes = [ctypes.c_int]
    L.twilight_prof_select.argtypes = [ctypes.c_int, ctypes.c_int]
    L.twilight_prof_collect.argtypes = [_vp, _vp, _i32]
    L.twilight_kernel_name.argtypes = [ctypes.c_int]
    L.twilight_decode_plan.argtypes = [kvp, ctypes.c_int, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
    L.twilight_decode_plan.restype = ctypes.c_int
    L.twilight_kernel_name.restype = ctypes.c_char_p
    for f in ("twilight_select_prune", "twilight_ds_select_tokens", "twilight_kquant_append", "twilight_select_pages", "twilight_select_pages_static", "twilight_append_select", "twilight_int4_score", "twilight_topp_prune",
              "twilight_int4_score_tokens", "twilight_topp_prune_tokens",
              "twilight_sparse_decode", "twilight_sparse_decode_per_head", "twilight_prof_enable", "twilight_prof_select", "twilight_prof_collect"):
        getattr(L, f).restype = ctypes.c_int
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code):
    if code != 0:
        raise TwilightError("twilight call failed (%d): %s" % (code, lib().twilight_strerror(code).decode()))


def make_kv(batch, num_q_heads, num_kv_heads, max_pages_per_seq, num_pool_pages, page_table, seq_lens,
            k_pool=None, v_pool=None, kq_pool=None, kq_meta=None, page_minmax=None, quant_bits=4):
    """Fill a twilight_kv_t from torch tensors (which the caller keeps alive)."""
    kv = twilight_kv_t()
    kv.batch, kv.num_q_heads, kv.num_kv_heads = batch, num_q_heads, num_kv_heads
    kv.head_dim, kv.page_size, kv.quant_group = 128, 16, 32
    kv.max_pages_per_seq, kv.quant_bits, kv.num_pool_pages = max_pages_per_seq, quant_bits, num_pool_pages
    for name, t in (("page_table", page_table), ("seq_lens", seq_lens), ("k_pool", k_pool), ("v_pool", v_pool),
                    ("kq_pool", kq_pool), ("kq_meta", kq_meta), ("page_minmax", page_minmax)):
        if t is None:
            setattr(kv, name, None)
        elif t.is_cuda:
            setattr(kv, name, t.data_ptr())
        else:                                       # offloaded K/V: pinned host memory, addressed from the device
            assert name in ("k_pool", "v_pool") and t.is_pinned(), "only k_pool / v_pool may be (pinned) host tensors"
            setattr(kv, name, pinned_device_pointer(t))
    return kv


def pinned_device_pointer(t):
    """Device-side address of a pinned host tensor (twilight_pinned_device_pointer)."""
    out = ctypes.c_void_p()
    _check(lib().twilight_pinned_device_pointer(ctypes.c_void_p(t.data_ptr()), ctypes.byref(out)))
    return out.value


def twilight_workspace_bytes(which, kv, max_sel=0, union_stride=0):
    return int(lib().twilight_workspace_bytes(which, ctypes.byref(kv), max_sel, union_stride))


def twilight_kquant_append(kv, k_new, v_new, start_pos, n_new, new_offsets, max_new):
    _check(lib().twilight_kquant_append(ctypes.byref(kv), _ptr(k_new), _ptr(v_new), _ptr(start_pos), _ptr(n_new),
                                        _ptr(new_offsets), int(max_new), _stream()))


def twilight_select_pages(kv, q, budget_tokens, sel_pages, sel_count, max_sel, ws):
    _check(lib().twilight_select_pages(ctypes.byref(kv), _ptr(q), _ptr(budget_tokens), _ptr(sel_pages),
                                       _ptr(sel_count), int(max_sel), _ptr(ws), ws.numel() * ws.element_size(),
                                       _stream()))


def twilight_select_pages_static(kv, q, budget_tokens, sel_pages, sel_count, max_sel):
    """The selector without a caller workspace and without any allocation (fixed scratch inside the library)."""
    _check(lib().twilight_select_pages_static(ctypes.byref(kv), _ptr(q), _ptr(budget_tokens), _ptr(sel_pages),
                                              _ptr(sel_count), int(max_sel), _stream()))


def twilight_ds_select_tokens(kv, q, channel_mask, budget_tokens, cand_tokens, cand_count, max_cand, ws):
    _check(lib().twilight_ds_select_tokens(ctypes.byref(kv), _ptr(q), _ptr(channel_mask), _ptr(budget_tokens),
                                           _ptr(cand_tokens), _ptr(cand_count), int(max_cand), _ptr(ws),
                                           ws.numel() * ws.element_size(), _stream()))


def twilight_append_select(kv, k_new, v_new, new_pos, q, budget_tokens, sel_pages, sel_count, max_sel, ws):
    _check(lib().twilight_append_select(ctypes.byref(kv), _ptr(k_new), _ptr(v_new), _ptr(new_pos), _ptr(q),
                                        _ptr(budget_tokens), _ptr(sel_pages), _ptr(sel_count), int(max_sel), _ptr(ws),
                                        ws.numel() * ws.element_size(), _stream()))


def twilight_select_prune(kv, k_new, v_new, new_pos, q, budget_tokens, p, sel_pages, sel_count, max_sel, kept_count, kept_idx,
                          kept_stride, union_count, union_idx, union_stride, status, ws):
    _check(lib().twilight_select_prune(ctypes.byref(kv), _ptr(k_new), _ptr(v_new), _ptr(new_pos), _ptr(q), _ptr(budget_tokens),
                                       float(p), _ptr(sel_pages), _ptr(sel_count), int(max_sel), _ptr(kept_count),
                                       _ptr(kept_idx), int(kept_stride), _ptr(union_count), _ptr(union_idx),
                                       int(union_stride), _ptr(status), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def twilight_int4_score(kv, q, sel_pages, sel_count, max_sel, scores, dots=None):
    _check(lib().twilight_int4_score(ctypes.byref(kv), _ptr(q), _ptr(sel_pages), _ptr(sel_count), int(max_sel),
                                     _ptr(scores), _ptr(dots), _stream()))


def twilight_topp_prune(kv, q, sel_pages, sel_count, max_sel, p, kept_count, kept_idx, kept_stride,
                        union_count, union_idx, union_stride, status, ws):
    _check(lib().twilight_topp_prune(ctypes.byref(kv), _ptr(q), _ptr(sel_pages), _ptr(sel_count), int(max_sel),
                                     float(p), _ptr(kept_count), _ptr(kept_idx), int(kept_stride),
                                     _ptr(union_count), _ptr(union_idx), int(union_stride), _ptr(status),
                                     _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def twilight_int4_score_tokens(kv, q, cand_tokens, cand_count, max_cand, scores, dots=None):
    _check(lib().twilight_int4_score_tokens(ctypes.byref(kv), _ptr(q), _ptr(cand_tokens), _ptr(cand_count), int(max_cand),
                                            _ptr(scores), _ptr(dots), _stream()))


def twilight_topp_prune_tokens(kv, q, cand_tokens, cand_count, max_cand, p, kept_count, kept_idx, kept_stride,
                               union_count, union_idx, union_stride, status, ws):
    _check(lib().twilight_topp_prune_tokens(ctypes.byref(kv), _ptr(q), _ptr(cand_tokens), _ptr(cand_count), int(max_cand),
                                            float(p), _ptr(kept_count), _ptr(kept_idx), int(kept_stride),
                                            _ptr(union_count), _ptr(union_idx), int(union_stride), _ptr(status),
                                            _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def twilight_sparse_decode(kv, q, union_count, union_idx, union_stride, out, lse, ws):
    _check(lib().twilight_sparse_decode(ctypes.byref(kv), _ptr(q), _ptr(union_count), _ptr(union_idx),
                                        int(union_stride), _ptr(out), _ptr(lse), _ptr(ws),
                                        ws.numel() * ws.element_size(), _stream()))


def twilight_sparse_decode_per_head(kv, q, kept_count, kept_idx, kept_stride, out, lse, ws):
    _check(lib().twilight_sparse_decode_per_head(ctypes.byref(kv), _ptr(q), _ptr(kept_count), _ptr(kept_idx),
                                                 int(kept_stride), _ptr(out), _ptr(lse), _ptr(ws),
                                                 ws.numel() * ws.element_size(), _stream()))


def twilight_decode_plan(kv, which=TW_WS_DECODE, dense=False):
    """-> (grid, chunk0, items_per_wg) of the attention kernel's launch for this cache shape."""
    g, c, i = _i32(), _i32(), _i32()
    _check(lib().twilight_decode_plan(ctypes.byref(kv), int(which), int(bool(dense)), ctypes.byref(g), ctypes.byref(c), ctypes.byref(i)))
    return g.value, c.value, i.value


def twilight_prof_enable(mode):
    _check(lib().twilight_prof_enable(int(mode)))


def twilight_prof_select(kernel_name, every=1):
    _check(lib().twilight_prof_select(KERNEL_NAMES.index(kernel_name), int(every)))


def twilight_prof_collect(cap=65536):
    """-> list of (kernel name, milliseconds) since the last collect."""
    ids = (ctypes.c_int32 * cap)()
    ms = (ctypes.c_float * cap)()
    n = lib().twilight_prof_collect(ids, ms, cap)
    return [(KERNEL_NAMES[ids[i]], float(ms[i])) for i in range(n)]
