"""ctypes binding of libqcache.so: same names as include/qcache.h, argument marshalling only.

Tensors are passed as torch tensors (their data_ptr() is taken) or as raw integer device
addresses; host integer arrays as Python sequences.  Every step of the attention path runs
inside the library's kernels.  If the library has not been built, importing works but the
first call raises: there is no fallback implementation.
"""
import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int32, c_int64, c_size_t, c_uint8, c_void_p

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqcache.so")

QC_OK, QC_EINVAL, QC_EORDER, QC_ECAPACITY, QC_EDEVICE = range(5)
QC_F32, QC_BF16 = 0, 1
QC_K, QC_V = 0, 1
QC_VLA, QC_GLA = 0, 1
QC_PLAN_KV, QC_PLAN_Q, QC_PLAN_WORKSPACE = 1, 2, 4
QC_STATIC_SCRATCH_BYTES = 4 << 20
DTYPE_CODE = {"f32": QC_F32, "bf16": QC_BF16}
MODE_CODE = {"vla": QC_VLA, "gla": QC_GLA}


class qc_config(ctypes.Structure):
    _fields_ = [("n_layers", c_int32), ("n_heads", c_int32), ("head_dim", c_int32), ("dtype", c_int32),
                ("max_batch", c_int32), ("max_seq", c_int32), ("max_vis", c_int32), ("max_text", c_int32),
                ("mode", c_int32), ("reserved", c_int32), ("prune_before_layer", c_int32), ("max_seq_late", c_int32),
                ("lazy_mask", POINTER(c_uint8))]


class qc_stats_t(ctypes.Structure):
    _fields_ = [("k_bytes", c_int64), ("v_bytes", c_int64), ("q_bytes", c_int64), ("tokens", c_int64),
                ("batch", c_int32), ("q_owner", c_int32), ("generated", c_int32), ("next_layer", c_int32)]


class QcError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (status_str(status), message))
        self.status = status


_PROTOTYPES = {
    "qc_kv_arena_bytes": (c_size_t, [POINTER(qc_config)]),
    "qc_q_arena_bytes": (c_size_t, [POINTER(qc_config)]),
    "qc_decode_workspace_bytes": (c_size_t, [POINTER(qc_config)]),
    "qc_kvcache_create": (c_int32, [POINTER(qc_config), c_void_p, c_size_t, POINTER(c_void_p)]),
    "qc_qcache_create": (c_int32, [POINTER(qc_config), c_void_p, c_size_t, POINTER(c_void_p)]),
    "qc_kvcache_destroy": (None, [c_void_p]),
    "qc_qcache_destroy": (None, [c_void_p]),
    "qc_reset": (c_int32, [c_void_p, c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32), c_int32, c_void_p]),
    "qc_reset_ragged": (c_int32, [c_void_p, c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                  POINTER(c_int32), c_int32, c_void_p]),
    "qc_page_table_bytes": (c_size_t, [POINTER(qc_config)]),
    "qc_reset_paged": (c_int32, [c_void_p, c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_uint8),
                                 c_void_p, c_size_t, c_int32, c_void_p]),
    "qc_seq_pages": (c_int32, [c_void_p, c_int32, c_int32, POINTER(c_int32), c_int32, POINTER(c_int32)]),
    "qc_pool_pages": (c_int32, [c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32)]),
    "qc_decode_split": (c_int32, [c_int32, c_int32, c_int32, POINTER(c_int32), POINTER(c_int32)]),
    "qc_pages_needed": (c_int32, [POINTER(qc_config), c_int32, c_int32, POINTER(c_int32)]),
    "qc_seq_leave": (c_int32, [c_void_p, c_void_p, c_int32, c_void_p]),
    "qc_seq_join": (c_int32, [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, c_void_p]),
    "qc_seq_grow": (c_int32, [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_void_p]),
    "qc_seq_extent": (c_int32, [c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                POINTER(c_int32)]),
    "qc_prefill": (c_int32, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                             POINTER(c_int32), c_int64, c_int64, POINTER(c_int32), POINTER(c_int32), c_float,
                             c_void_p]),
    "qc_decode": (c_int32, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                            POINTER(c_int32), POINTER(c_int32), c_float, c_void_p, c_size_t, c_void_p]),
    "qc_decode_static": (c_int32, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                   POINTER(c_int32), POINTER(c_int32), c_float, c_void_p]),
    "qc_decode_graph_create": (c_int32, [c_void_p, c_void_p, POINTER(c_void_p), POINTER(c_void_p), POINTER(c_void_p),
                                         POINTER(c_void_p), c_float, c_void_p, c_size_t, POINTER(c_void_p)]),
    "qc_decode_graph_launch": (c_int32, [c_void_p, c_void_p]),
    "qc_decode_graph_destroy": (None, [c_void_p]),
    "qc_stats": (c_int32, [c_void_p, c_void_p, POINTER(qc_stats_t)]),
    "qc_layer_rows": (c_int32, [c_void_p, c_int32, POINTER(c_int64), POINTER(c_int64)]),
    "qc_seq_len": (c_int32, [c_void_p, c_int32, POINTER(c_int32)]),
    "qc_locate": (c_int32, [c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, POINTER(c_int32),
                            POINTER(c_int64)]),
    "qc_project_qk": (c_int32, [c_void_p, c_int64, c_void_p, c_void_p, c_int64, c_void_p, c_void_p, c_int64, c_int64, c_int32,
                                c_int32, c_int32, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                POINTER(c_int32), c_int32, c_float, c_void_p]),
    "qc_select_workspace_bytes": (c_size_t, [POINTER(qc_config)]),
    "qc_last_row_attention": (c_int32, [c_void_p, c_int32, c_void_p, c_void_p, c_int64, c_float, c_void_p, c_size_t,
                                        c_void_p]),
    "qc_attention_similarity": (c_int32, [c_void_p, c_void_p, c_int64, c_int32, POINTER(c_int32), c_void_p, c_void_p,
                                          c_void_p]),
    "qc_lazy_mask_from_similarity": (c_int32, [POINTER(c_float), c_int32, c_float, POINTER(c_uint8)]),
    "qc_prune_select": (c_int32, [c_void_p, c_int64, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                  POINTER(c_int32), c_void_p, c_void_p]),
    "qc_gather_rows": (c_int32, [c_void_p, c_int64, c_void_p, c_int64, c_int64, c_void_p, c_int64, c_void_p]),
    "qc_prune": (c_int32, [c_void_p, c_void_p, POINTER(c_int32)]),
    "qc_plan_max_batch": (c_int32, [POINTER(qc_config), c_size_t, c_int32, POINTER(c_int32)]),
    "qc_timing_enable": (c_int32, [c_void_p, c_int32]),
    "qc_timing_read": (c_int32, [c_void_p, c_int32, POINTER(ctypes.c_double), POINTER(c_int64)]),
    "qc_status_str": (c_char_p, [c_int32]),
    "qc_last_error": (c_char_p, []),
}
EXPORTED = tuple(_PROTOTYPES)

_lib = None


def load_library():
    """Load libqcache.so (once) and set the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libqcache.so is missing: build it with __graft_entry__.build() or "
                               "python -m paper_2602_01901_amd.build (there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _i32(seq):
    if seq is None:
        return None
    seq = [int(v) for v in seq]
    return (c_int32 * max(len(seq), 1))(*seq)


def _check(status):
    if status != QC_OK:
        raise QcError(status, qc_last_error())
    return status


def status_str(status):
    return load_library().qc_status_str(int(status)).decode()


qc_status_str = status_str


def qc_last_error():
    return load_library().qc_last_error().decode()


def make_config(n_layers, n_heads, head_dim, dtype, max_batch, max_seq, max_vis, max_text, lazy_mask,
                mode="vla", prune_before_layer=0, max_seq_late=0):
    """Returns a qc_config; the mask buffer is kept alive by the returned object."""
    mask = (c_uint8 * max(len(lazy_mask), 1))(*[int(bool(x)) for x in lazy_mask])
    cfg = qc_config(n_layers, n_heads, head_dim, DTYPE_CODE.get(dtype, dtype), max_batch, max_seq, max_vis,
                    max_text, MODE_CODE.get(mode, mode), 0, prune_before_layer, max_seq_late,
                    ctypes.cast(mask, POINTER(c_uint8)))
    cfg._mask_keepalive = mask
    return cfg


def qc_kv_arena_bytes(cfg):
    return load_library().qc_kv_arena_bytes(byref(cfg))


def qc_q_arena_bytes(cfg):
    return load_library().qc_q_arena_bytes(byref(cfg))


def qc_decode_workspace_bytes(cfg):
    return load_library().qc_decode_workspace_bytes(byref(cfg))


def qc_kvcache_create(cfg, dev_arena, arena_bytes):
    out = c_void_p()
    _check(load_library().qc_kvcache_create(byref(cfg), _ptr(dev_arena), arena_bytes, byref(out)))
    return out


def qc_qcache_create(cfg, dev_arena, arena_bytes):
    out = c_void_p()
    _check(load_library().qc_qcache_create(byref(cfg), _ptr(dev_arena), arena_bytes, byref(out)))
    return out


def qc_kvcache_destroy(kv):
    load_library().qc_kvcache_destroy(kv)


def qc_qcache_destroy(qc):
    load_library().qc_qcache_destroy(qc)


def qc_reset(kv, qc, batch, vis_start, vis_len, zero_fill=1, stream=None):
    return _check(load_library().qc_reset(kv, qc, batch, _i32(vis_start), _i32(vis_len), int(zero_fill), stream))


def qc_reset_ragged(kv, qc, batch, vis_start, vis_len, cap_seq, cap_text, zero_fill=1, stream=None):
    return _check(load_library().qc_reset_ragged(kv, qc, batch, _i32(vis_start), _i32(vis_len), _i32(cap_seq),
                                                _i32(cap_text), int(zero_fill), stream))


def qc_page_table_bytes(cfg):
    return load_library().qc_page_table_bytes(byref(cfg))


def qc_reset_paged(kv, qc, batch, vis_start, vis_len, present, page_lists, page_list_bytes, zero_fill=1, stream=None):
    flags = None if present is None else (c_uint8 * len(present))(*[int(bool(x)) for x in present])
    return _check(load_library().qc_reset_paged(kv, qc, batch, _i32(vis_start), _i32(vis_len), flags, _ptr(page_lists),
                                               page_list_bytes, int(zero_fill), stream))


def qc_seq_pages(kv, b, pool):
    """The pages slot b holds in `pool` (0 positions, 1 text rows, 2 visual rows), in row order."""
    n = c_int32()
    _check(load_library().qc_seq_pages(kv, b, pool, None, 0, byref(n)))
    buf = (c_int32 * max(n.value, 1))()
    _check(load_library().qc_seq_pages(kv, b, pool, buf, n.value, byref(n)))
    return [buf[i] for i in range(n.value)]


def qc_decode_split(pairs, max_len, compute_units=256):
    """(key positions per workgroup, workgroups for the longest sequence) of an ordinary decode call."""
    chunk, n = c_int32(), c_int32()
    _check(load_library().qc_decode_split(pairs, max_len, compute_units, byref(chunk), byref(n)))
    return chunk.value, n.value


def qc_pool_pages(kv, pool):
    """(pages of `pool` in all, pages free at this moment)."""
    total, free = c_int32(), c_int32()
    _check(load_library().qc_pool_pages(kv, pool, byref(total), byref(free)))
    return total.value, free.value


def qc_pages_needed(cfg, length, vis_len):
    """Pages a sequence of `length` stored positions, vis_len of them visual, holds in the three pools."""
    buf = (c_int32 * 3)()
    _check(load_library().qc_pages_needed(byref(cfg), length, vis_len, buf))
    return [buf[0], buf[1], buf[2]]


def qc_seq_leave(kv, qc, b, stream=None):
    return _check(load_library().qc_seq_leave(kv, qc, b, stream))


def qc_seq_join(kv, qc, b, vis_start, vis_len, cap_seq, cap_text, stream=None):
    return _check(load_library().qc_seq_join(kv, qc, b, vis_start, vis_len, cap_seq, cap_text, stream))


def qc_seq_grow(kv, qc, b, cap_seq, cap_text, stream=None):
    return _check(load_library().qc_seq_grow(kv, qc, b, cap_seq, cap_text, stream))


def qc_seq_extent(kv, b):
    """(live, base_seq, base_text, base_vis) of slot b."""
    out = [c_int32() for _ in range(4)]
    _check(load_library().qc_seq_extent(kv, b, *[byref(x) for x in out]))
    return tuple(x.value for x in out)


def qc_prefill(kv, qc, layer, is_lazy, q, k, v, out, cu_seqlens, token_stride, head_stride, vis_start, vis_len,
               softmax_scale=0.0, stream=None):
    return _check(load_library().qc_prefill(kv, qc, layer, int(is_lazy), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                           _i32(cu_seqlens), token_stride, head_stride, _i32(vis_start),
                                           _i32(vis_len), softmax_scale, stream))


def qc_decode(kv, qc, layer, is_lazy, q, k, v, out, vis_start, vis_len, softmax_scale, workspace,
              workspace_bytes, stream=None):
    return _check(load_library().qc_decode(kv, qc, layer, int(is_lazy), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                          _i32(vis_start), _i32(vis_len), softmax_scale, _ptr(workspace),
                                          workspace_bytes, stream))


def qc_decode_static(kv, qc, layer, is_lazy, q, k, v, out, vis_start, vis_len, softmax_scale=0.0, stream=None):
    return _check(load_library().qc_decode_static(kv, qc, layer, int(is_lazy), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                                 _i32(vis_start), _i32(vis_len), softmax_scale, stream))


def _ptr_array(xs):
    return (c_void_p * max(len(xs), 1))(*[_ptr(x) for x in xs])


def qc_decode_graph_create(kv, qc, q, k, v, out, softmax_scale, workspace, workspace_bytes):
    """q, k, v, out: per-layer lists of tensors (or device addresses; None where a layer has none)."""
    g = c_void_p()
    _check(load_library().qc_decode_graph_create(kv, qc, _ptr_array(q), _ptr_array(k), _ptr_array(v), _ptr_array(out),
                                                softmax_scale, _ptr(workspace), workspace_bytes, byref(g)))
    return g


def qc_decode_graph_launch(graph, stream=None):
    return _check(load_library().qc_decode_graph_launch(graph, stream))


def qc_decode_graph_destroy(graph):
    load_library().qc_decode_graph_destroy(graph)


def qc_stats(kv, qc):
    st = qc_stats_t()
    _check(load_library().qc_stats(kv, qc, byref(st)))
    return {name: getattr(st, name) for name, _ in qc_stats_t._fields_}


def qc_layer_rows(kv, layer):
    rk, rv = c_int64(), c_int64()
    _check(load_library().qc_layer_rows(kv, layer, byref(rk), byref(rv)))
    return rk.value, rv.value


def qc_seq_len(kv, b):
    n = c_int32()
    _check(load_library().qc_seq_len(kv, b, byref(n)))
    return n.value


def qc_locate(kv, which, layer, b, h, pos):
    src, off = c_int32(), c_int64()
    _check(load_library().qc_locate(kv, which, layer, b, h, pos, byref(src), byref(off)))
    return src.value, off.value


def qc_project_qk(x, x_stride, w_q, w_k, w_stride, q, k, token_stride, head_stride, d_model, n_heads, head_dim, batch,
                  cu_seqlens, pos0, vis_start, vis_len, skip_span, rope_theta, stream=None):
    return _check(load_library().qc_project_qk(_ptr(x), x_stride, _ptr(w_q), _ptr(w_k), w_stride, _ptr(q), _ptr(k),
                                              token_stride, head_stride, d_model, n_heads, head_dim, batch,
                                              _i32(cu_seqlens), _i32(pos0), _i32(vis_start), _i32(vis_len),
                                              int(skip_span), rope_theta, stream))


def qc_select_workspace_bytes(cfg):
    return load_library().qc_select_workspace_bytes(byref(cfg))


def qc_last_row_attention(kv, layer, q_last, probs, probs_stride, softmax_scale, workspace, workspace_bytes,
                          stream=None):
    return _check(load_library().qc_last_row_attention(kv, layer, _ptr(q_last), _ptr(probs), probs_stride,
                                                      softmax_scale, _ptr(workspace), workspace_bytes, stream))


def qc_attention_similarity(probs_m, probs_n, stride, n_samples, lens, js_out, s_out, stream=None):
    return _check(load_library().qc_attention_similarity(_ptr(probs_m), _ptr(probs_n), stride, n_samples,
                                                        _i32(lens), _ptr(js_out), _ptr(s_out), stream))


def qc_lazy_mask_from_similarity(adjacent, eps):
    """Eq. 4 on the host: list of flags, one per layer (len(adjacent) + 1 layers)."""
    n = len(adjacent) + 1
    adj = (c_float * max(len(adjacent), 1))(*[float(x) for x in adjacent])
    out = (c_uint8 * n)()
    _check(load_library().qc_lazy_mask_from_similarity(adj, n, eps, out))
    return [int(x) for x in out]


def qc_prune_select(scores, stride, batch, cu_seqlens, vis_start, vis_len, keep, row_map, stream=None):
    return _check(load_library().qc_prune_select(_ptr(scores), stride, batch, _i32(cu_seqlens), _i32(vis_start),
                                                _i32(vis_len), _i32(keep), _ptr(row_map), stream))


def qc_gather_rows(src, src_stride, row_map, n_rows, row_bytes, dst, dst_stride, stream=None):
    return _check(load_library().qc_gather_rows(_ptr(src), src_stride, _ptr(row_map), n_rows, row_bytes, _ptr(dst),
                                               dst_stride, stream))


def qc_prune(kv, qc, keep):
    return _check(load_library().qc_prune(kv, qc, _i32(keep)))


def qc_plan_max_batch(cfg, budget_bytes, what):
    out = c_int32()
    _check(load_library().qc_plan_max_batch(byref(cfg), int(budget_bytes), int(what), byref(out)))
    return out.value


def qc_timing_enable(kv, enable):
    return _check(load_library().qc_timing_enable(kv, int(enable)))


def qc_timing_read(kv, which):
    """(total milliseconds, launches) of the dominant kernel since the last read; which: 0 prefill, 1 decode,
    2 decode calls of lazy layers in "gla" mode."""
    ms, n = ctypes.c_double(), c_int64()
    _check(load_library().qc_timing_read(kv, which, byref(ms), byref(n)))
    return ms.value, n.value
