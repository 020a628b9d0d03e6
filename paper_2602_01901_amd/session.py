"""Device-memory plumbing around the C ABI: arenas, workspace and handles for one decoder stack.

PyTorch is used for allocation and for the current stream only.  Every call forwards to the
library; nothing is computed here.
"""
import torch

from . import binding as B

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


class Session:
    def __init__(self, n_layers, n_heads, head_dim, dtype, lazy_mask, max_batch, max_seq, max_vis, max_text,
                 device="cuda:0", mode="vla", prune_before_layer=0, max_seq_late=0):
        if not torch.cuda.is_available():
            raise RuntimeError("the Lazy Attention library needs a GPU; there is no CPU path")
        B.load_library()
        self.device = torch.device(device)
        self.dtype = dtype
        self.torch_dtype = _TORCH_DTYPE[dtype]
        self.n_layers, self.n_heads, self.head_dim = n_layers, n_heads, head_dim
        self.lazy_mask = [int(bool(x)) for x in lazy_mask]
        self.mode = mode
        self.cfg = B.make_config(n_layers, n_heads, head_dim, dtype, max_batch, max_seq, max_vis, max_text,
                                 self.lazy_mask, mode=mode, prune_before_layer=prune_before_layer,
                                 max_seq_late=max_seq_late)
        self.kv_bytes = B.qc_kv_arena_bytes(self.cfg)
        self.q_bytes = B.qc_q_arena_bytes(self.cfg)
        self.ws_bytes = B.qc_decode_workspace_bytes(self.cfg)
        if self.kv_bytes == 0:
            raise B.QcError(B.QC_EINVAL, "invalid configuration")
        self.kv_arena = torch.empty(self.kv_bytes, dtype=torch.uint8, device=self.device)
        self.q_arena = torch.empty(max(self.q_bytes, 256), dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.device)
        self.kv = B.qc_kvcache_create(self.cfg, self.kv_arena, self.kv_bytes)
        self.qc = B.qc_qcache_create(self.cfg, self.q_arena, self.q_bytes)
        self.vis_start = self.vis_len = None
        self.batch = 0
        self._lib = B.load_library()
        self._ws_ptr = self.workspace.data_ptr()
        self._graphs = []
        self.page_lists = None

    @classmethod
    def for_workload(cls, w, device="cuda:0", mode="vla", prune_before_layer=0, max_seq_late=0):
        return cls(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.lazy_mask, w.batch, w.max_seq, w.max_vis,
                   w.max_text, device=device, mode=mode, prune_before_layer=prune_before_layer,
                   max_seq_late=max_seq_late)

    def _stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    def reset(self, vis_start, vis_len, zero_fill=True, cap_seq=None, cap_text=None, paged=False, present=None):
        """cap_seq / cap_text: optional per-sequence capacities (qc_reset_ragged).  paged: rows on pages
        (qc_reset_paged; `present` flags the slots that hold a sequence from the start, default all)."""
        self.vis_start, self.vis_len = list(vis_start), list(vis_len)
        self.batch = len(self.vis_start)
        # marshalled once per batch: the span arrays every later call repeats
        self._vs_c, self._vl_c = B._i32(self.vis_start), B._i32(self.vis_len)
        self.first_late, self.keep = None, None
        self._vl_by_layer = [(self.vis_len, self._vl_c)] * self.n_layers   # span lengths each layer's calls repeat
        if paged:
            nbytes = B.qc_page_table_bytes(self.cfg)
            if nbytes == 0:
                raise B.QcError(B.QC_EINVAL, "the configuration cannot be paged")
            if self.page_lists is None:
                self.page_lists = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            B.qc_reset_paged(self.kv, self.qc, self.batch, self.vis_start, self.vis_len, present, self.page_lists, nbytes,
                             int(zero_fill), self._stream())
        elif cap_seq is not None:
            B.qc_reset_ragged(self.kv, self.qc, self.batch, self.vis_start, self.vis_len, cap_seq, cap_text,
                              int(zero_fill), self._stream())
        else:
            B.qc_reset(self.kv, self.qc, self.batch, self.vis_start, self.vis_len, int(zero_fill), self._stream())

    def _set_span(self, b, vis_start, vis_len):
        self.vis_start[b], self.vis_len[b] = vis_start, vis_len
        self._vs_c, self._vl_c = B._i32(self.vis_start), B._i32(self.vis_len)
        self._vl_by_layer = [(self.vis_len, self._vl_c)] * self.n_layers

    def seq_leave(self, b):
        """Slot b of a batch with per-sequence capacities becomes free (between two decode steps)."""
        B.qc_seq_leave(self.kv, self.qc, b, self._stream())
        self._set_span(b, 0, 0)

    def seq_join(self, b, vis_start, vis_len, cap_seq=0, cap_text=0):
        """A new sequence takes free slot b; the next calls are a prefill pass over the joined slots only."""
        B.qc_seq_join(self.kv, self.qc, b, vis_start, vis_len, cap_seq, cap_text, self._stream())
        self._set_span(b, vis_start, vis_len)

    def seq_grow(self, b, cap_seq, cap_text):
        """Other capacities for the sequence in slot b; its rows move to a new extent where a pool's capacity changes."""
        B.qc_seq_grow(self.kv, self.qc, b, cap_seq, cap_text, self._stream())

    def prune(self, next_layer, keep):
        """Token pruning boundary before `next_layer` (the layer the prefill pass runs next): from there on
        sequence b keeps keep[b] of its visual tokens.  Later prefill calls take the shortened prompts."""
        B.qc_prune(self.kv, self.qc, keep)
        self.first_late, self.keep = next_layer, list(keep)
        late = (self.keep, B._i32(self.keep))
        self._vl_by_layer = [late if l >= next_layer else (self.vis_len, self._vl_c) for l in range(self.n_layers)]

    def prefill(self, layer, q, k, v, cu_seqlens, out=None, softmax_scale=0.0):
        """q, k, v: [tokens, H, D] tensors sharing strides.  Returns out.  In "gla" mode a lazy
        layer has no q and k: pass None for both."""
        if out is None:
            out = torch.empty_like(v)
        for t in (q, k, out):
            assert t is None or t.stride() == v.stride()
        assert v.stride(2) == 1
        B.qc_prefill(self.kv, self.qc, layer, self.lazy_mask[layer], q, k, v, out, cu_seqlens, v.stride(0),
                     v.stride(1), self.vis_start, self._vl_by_layer[layer][0], softmax_scale, self._stream())
        return out

    def decode(self, layer, q, k, v, out=None, softmax_scale=0.0, stream=None):
        """q, k, v: contiguous [B, H, D] tensors.  Returns out.  `stream` (a raw hipStream_t value)
        defaults to torch's current stream; tight loops may pass it to skip the lookup.  In "gla" mode a
        lazy layer has no q and k: pass None for both."""
        if out is None:
            out = torch.empty_like(v)
        assert v.is_contiguous() and out.is_contiguous()
        assert (q is None or q.is_contiguous()) and (k is None or k.is_contiguous())
        status = self._lib.qc_decode(self.kv, self.qc, layer, self.lazy_mask[layer],
                                     None if q is None else q.data_ptr(), None if k is None else k.data_ptr(),
                                     v.data_ptr(), out.data_ptr(), self._vs_c, self._vl_by_layer[layer][1], softmax_scale,
                                     self._ws_ptr, self.ws_bytes, self._stream() if stream is None else stream)
        if status != B.QC_OK:
            raise B.QcError(status, B.qc_last_error())
        return out

    def decode_graph(self, q, k, v, out, softmax_scale=0.0):
        """One decode step recorded as a HIP graph over per-layer lists of contiguous [B, H, D] buffers
        (None for q and k of lazy layers in "gla" mode).  Returns a handle for graph_launch."""
        g = B.qc_decode_graph_create(self.kv, self.qc, q, k, v, out, softmax_scale, self._ws_ptr, self.ws_bytes)
        self._graphs.append(g)
        return g

    def graph_launch(self, graph, stream=None):
        status = self._lib.qc_decode_graph_launch(graph, self._stream() if stream is None else stream)
        if status != B.QC_OK:
            raise B.QcError(status, B.qc_last_error())

    def stats(self):
        return B.qc_stats(self.kv, self.qc)

    def close(self):
        if self.kv is not None:
            for g in self._graphs:
                B.qc_decode_graph_destroy(g)
            self._graphs = []
            B.qc_kvcache_destroy(self.kv)
            B.qc_qcache_destroy(self.qc)
            self.kv = self.qc = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
