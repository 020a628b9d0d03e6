"""Byte layout of the K/V arena and the Q Cache arena, and resident-byte accounting
(test infrastructure).

The paper fixes what is stored ("Efficiency Analysis", KV Cache paragraph: a
lazy layer keeps only its text keys; every layer keeps all values; the Q Cache
is one layer's worth of visual queries) but not where.  This module states the
row layout the library is specified to use, in closed form, so that cache contents
can be compared byte for byte.  It covers the K and V row regions and the Q arena
and nothing else: whatever a library keeps behind the V region for its own
bookkeeping (per-sequence integers for its kernels, counters) is that library's
private matter, is not described here and is checked through its queries
(sequence lengths, row counts, row locations), never through this image.

  K region   layers in order; layer l holds [max_batch][H][capK(l)][D] elements,
             capK(l) = max_text for a lazy layer, max_seq otherwise.
  V region   follows the K region; layer l holds [max_batch][H][max_seq][D].
  Q arena    [max_batch][H][max_vis][D].

Row maps: V row = position.  K row = position in a normal layer.  In a lazy
layer positions before the span keep their index, positions after it move
down by vis_len, and positions inside the span have no row in that layer:
they resolve to the same position in the block's first layer.

Per-sequence capacities (`ragged`): the regions keep their sizes, but sequence b
owns cap_seq[b] rows per head in every [.., max_seq, ..] block, cap_text[b] in a
lazy layer's K block and vis_len[b] in the Q arena, and its rows start where the
rows of the sequences before it end: with base[b] = sum of the capacities of the
sequences before b, row r of head h sits at row index base[b]*H + h*cap[b] + r
of the region.  Equal capacities (cap_seq = max_seq, ...) give back the layout
above; the sums must fit the pools max_batch*max_seq, max_batch*max_text and
max_batch*max_vis.  The arena then wastes nothing on a batch of unequal lengths.

Slots and extents: a batch with per-sequence capacities is a list of slots, each
holding a sequence or free (capacity 0, no rows).  The run of cap[b] rows-per-head
that slot b owns in a pool, [base[b], base[b] + cap[b]), is its extent; the rule
above assigns the extents of a fresh batch back to back in slot order.  A
sequence that joins later gets, in each pool, the lowest base at which its
capacity fits between the extents of the sequences then present (`first_fit`);
nobody else moves, and a leaving sequence's rows keep their bytes until a later
extent covers them.  `ragged` then carries the bases explicitly.

Pages (`paged`): the regions keep their sizes (max_seq, max_text and max_vis are then multiples of
PAGE_ROWS = 64), but each is cut into pages of 64 rows for every head, [page][H][64][D], and a sequence
owns a list of pages per pool instead of one run of rows: row r of head h sits at row index
(pages[r // 64]*H + h)*64 + r % 64 of the region.  One list per sequence and pool serves every layer and
head: "seq" pages hold the V rows of every layer and the K rows of ordinary layers (and, under Global Lazy
Attention, the Q Cache rows), "text" pages the K rows of lazy layers, "vis" pages the Q Cache rows.  Pages
are handed out lowest free number first (`PagePools`), one pool after the other for each sequence in
slot order, when a sequence's rows first need them: at the start of its prefill pass for the prompt, and
before the decode step whose new row opens a page.  A sequence that leaves gives all its pages back; the
bytes stay until another sequence's rows cover them.

Separately sized late layers (`late`): when a token-pruning boundary is known
as the arena is sized, the layers from the boundary on hold max_seq_late
positions per sequence instead of max_seq; their K blocks (ordinary layers) and V
blocks shrink accordingly and the regions behind them move up.

Global Lazy Attention (mode "gla"; Eq. 5/6 and the sentence after Eq. 6: a lazy
layer stores no K rows, the Q Cache holds the queries of every token): capK(l) = 0
for a lazy layer, every key position of a lazy layer resolves to the same
position in the block's first layer, and the Q arena is
[max_batch][H][max_seq][D] with row = position.
"""
import numpy as np

ELEM_BYTES = {"f32": 4, "bf16": 2}
PAGE_ROWS = 64


def _round_up(x, m):
    return (x + m - 1) // m * m


class ArenaLayout:
    def __init__(self, n_layers, n_heads, head_dim, dtype, max_batch, max_seq, max_vis, max_text,
                 lazy_mask, mode="vla", ragged=None, late=None, paged=None):
        """ragged: None, or (cap_seq, cap_text, cap_vis) lists with one entry per slot of the batch (0 for a
        free slot), optionally followed by (base_seq, base_text, base_vis) when the extents were not
        assigned back to back (sequences joined later).
        late: None, or (first late layer, max_seq_late): the layers from there on hold max_seq_late
        positions per sequence instead of max_seq (a pruning boundary known when the arena is sized)."""
        self.late = late
        assert late is None or (ragged is None and 1 <= late[0] < n_layers and 1 <= late[1] <= max_seq)
        # paged: None, or {"seq": [pages of slot 0, pages of slot 1, ...], "text": [...], "vis": [...]}
        self.paged = None
        if paged is not None:
            assert ragged is None and late is None
            assert max_seq % PAGE_ROWS == 0 and (mode == "gla" or (max_text % PAGE_ROWS == 0 and max_vis % PAGE_ROWS == 0))
            pools = {"seq": max_batch * max_seq // PAGE_ROWS, "text": max_batch * max_text // PAGE_ROWS,
                     "vis": max_batch * max_vis // PAGE_ROWS}
            for kind in (("seq", "text", "vis") if mode == "vla" else ("seq",)):
                held = [pg for lst in paged[kind] for pg in lst]
                assert len(set(held)) == len(held), "a page is held twice"
                assert all(0 <= pg < pools[kind] for pg in held), "page outside its pool"
            self.paged = {k: [list(lst) for lst in v] for k, v in paged.items()}
        assert mode in ("vla", "gla")
        self.ragged = None
        if ragged is not None:
            cap_seq, cap_text, cap_vis = ([int(x) for x in r] for r in ragged[:3])
            assert len(cap_seq) == len(cap_text) == len(cap_vis) <= max_batch
            pools = {"seq": max_batch * max_seq, "text": max_batch * max_text, "vis": max_batch * max_vis}
            caps = {"seq": cap_seq, "text": cap_text, "vis": cap_vis}
            if len(ragged) == 3:
                bases = {k: [sum(c[:b]) for b in range(len(c))] for k, c in caps.items()}
            else:
                bases = dict(zip(("seq", "text", "vis"), ([int(x) for x in r] for r in ragged[3:6])))
            for kind in (("seq", "text", "vis") if mode == "vla" else ("seq",)):
                ext = sorted((b0, c) for b0, c in zip(bases[kind], caps[kind]) if c > 0)
                assert all(a0 + a1 <= b0 for (a0, a1), (b0, _) in zip(ext, ext[1:])), "extents overlap"
                assert not ext or (ext[0][0] >= 0 and ext[-1][0] + ext[-1][1] <= pools[kind])
            self.ragged = {k: (caps[k], bases[k]) for k in caps}
        self.mode = mode
        self.N, self.H, self.D = n_layers, n_heads, head_dim
        self.dtype = dtype
        self.e = ELEM_BYTES[dtype]
        self.max_batch, self.max_seq = max_batch, max_seq
        self.max_vis, self.max_text = max_vis, max_text
        self.lazy = [int(bool(x)) for x in lazy_mask]
        assert len(self.lazy) == n_layers and not (n_layers and self.lazy[0])

    def cap_v(self, l):
        return self.late[1] if (self.late is not None and l >= self.late[0]) else self.max_seq

    def cap_k(self, l):
        if not self.lazy[l]:
            return self.cap_v(l)
        return self.max_text if self.mode == "vla" else 0

    def cap_q(self):
        return self.max_vis if self.mode == "vla" else self.max_seq

    def k_layer_bytes(self, l):
        return self.max_batch * self.H * self.cap_k(l) * self.D * self.e

    def v_layer_bytes(self, l=0):
        return self.max_batch * self.H * self.cap_v(l) * self.D * self.e

    def off_k(self, l):
        return sum(self.k_layer_bytes(i) for i in range(l))

    def off_v(self, l):
        return self.off_k(self.N) + sum(self.v_layer_bytes(i) for i in range(l))

    def rows_bytes(self):
        """Bytes of the K and V row regions together: everything this module describes of the K/V arena."""
        return self.off_v(self.N)

    def _row_index(self, kind, uniform_cap, b, h, row):
        """Row index inside a region of `kind` rows ("seq", "text" or "vis")."""
        if self.paged is not None:
            pages = self.paged[kind][b]
            assert 0 <= row < len(pages) * PAGE_ROWS, "row on a page the sequence does not hold"
            return (pages[row // PAGE_ROWS] * self.H + h) * PAGE_ROWS + row % PAGE_ROWS
        if self.ragged is None:
            return (b * self.H + h) * uniform_cap + row
        cap, base = self.ragged[kind]
        assert 0 <= row < max(cap[b], 1)
        return base[b] * self.H + h * cap[b] + row

    def _k_kind(self, l):
        return "text" if (self.lazy[l] and self.mode == "vla") else "seq"

    def q_arena_bytes(self):
        return self.max_batch * self.H * self.cap_q() * self.D * self.e

    def k_offset(self, l, b, h, row):
        return self.off_k(l) + self._row_index(self._k_kind(l), self.cap_k(l), b, h, row) * self.D * self.e

    def v_offset(self, l, b, h, row):
        return self.off_v(l) + self._row_index("seq", self.cap_v(l), b, h, row) * self.D * self.e

    def q_offset(self, b, h, row):
        kind = "vis" if self.mode == "vla" else "seq"
        return self._row_index(kind, self.cap_q(), b, h, row) * self.D * self.e

    def anchor(self, l):
        a = l - 1
        while self.lazy[a]:
            a -= 1
        return a

    def locate_k(self, l, b, h, pos, vis_start, vis_len):
        """(source layer, byte offset in the K/V arena) of the key of `pos` as layer l reads it."""
        if self.lazy[l] and self.mode == "gla":
            a = self.anchor(l)
            return a, self.k_offset(a, b, h, pos)
        if self.lazy[l] and vis_start <= pos < vis_start + vis_len:
            a = self.anchor(l)
            return a, self.k_offset(a, b, h, pos)
        row = pos
        if self.lazy[l] and pos >= vis_start + vis_len:
            row = pos - vis_len
        return l, self.k_offset(l, b, h, row)

    def locate_v(self, l, b, h, pos):
        return l, self.v_offset(l, b, h, pos)


def first_fit(extents, want, pool):
    """Lowest base at which `want` rows fit into a pool of `pool` rows beside the extents (base, rows) in
    use; None if no gap is wide enough.  A request for no rows sits at 0."""
    if want == 0:
        return 0
    for base in range(pool - want + 1):
        if all(base + want <= b0 or b0 + n <= base for b0, n in extents if n > 0):
            return base
    return None


def encode_rows(x, dtype):
    """fp64 rows -> raw bytes of the storage type; refuses values the type cannot hold exactly."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if not np.array_equal(x32.astype(np.float64), np.asarray(x, dtype=np.float64)):
        raise ValueError("cache rows are not exactly representable in fp32")
    if dtype == "f32":
        return x32.view(np.uint8)
    bits = x32.view(np.uint32)
    if np.any(bits & 0xFFFF):
        raise ValueError("cache rows are not exactly representable in bf16")
    return (bits >> 16).astype(np.uint16).view(np.uint8)


def _write_rows(img, layout, rows, offset_of_row):
    """Rows 0..n-1 of one (sequence, head) into the image: one run, or one run per page."""
    n, rowb = rows.shape[0], layout.D * layout.e
    step = PAGE_ROWS if layout.paged is not None else max(n, 1)
    raw = encode_rows(rows, layout.dtype).reshape(n, rowb) if n else None
    for r0 in range(0, n, step):
        r1 = min(r0 + step, n)
        o = offset_of_row(r0)
        img[o:o + (r1 - r0) * rowb] = raw[r0:r1].reshape(-1)


class PagePools:
    """Who holds which page, under the rule stated in the module's header: lowest free number first, the
    pools in the order seq, text, vis for each sequence in slot order."""

    def __init__(self, max_batch, max_seq, max_vis, max_text, mode="vla", any_lazy=True):
        self.mode = mode
        self.any_lazy = any_lazy
        size = {"seq": max_batch * max_seq // PAGE_ROWS, "text": max_batch * max_text // PAGE_ROWS,
                "vis": max_batch * max_vis // PAGE_ROWS}
        self.free = {k: list(range(n)) for k, n in size.items()}
        self.held = {k: [[] for _ in range(max_batch)] for k in size}

    def _kinds(self):
        return ("seq", "text", "vis") if (self.mode == "vla" and self.any_lazy) else ("seq",)

    def _grow_to(self, kind, b, rows):
        need = (rows + PAGE_ROWS - 1) // PAGE_ROWS - len(self.held[kind][b])
        if need > len(self.free[kind]):
            raise MemoryError("pool %s has %d free pages, %d wanted" % (kind, len(self.free[kind]), need))
        for _ in range(max(need, 0)):
            self.held[kind][b].append(self.free[kind].pop(0))

    def rows_of(self, length, vis_len):
        return {"seq": length, "text": length - vis_len, "vis": vis_len}

    def prefill(self, slots, lens, vis_lens):
        """The prompts of `slots` (in slot order) get their pages."""
        for b in sorted(slots):
            want = self.rows_of(lens[b], vis_lens[b])
            for kind in self._kinds():
                self._grow_to(kind, b, want[kind])

    def decode_step(self, slots, lens, vis_lens):
        """Before a decode step: every sequence of `slots` is about to store row lens[b] (and text row
        lens[b] - vis_lens[b])."""
        for b in sorted(slots):
            want = self.rows_of(lens[b] + 1, vis_lens[b])
            for kind in self._kinds():
                if kind != "vis":
                    self._grow_to(kind, b, want[kind])

    def leave(self, b):
        for kind in self.free:
            self.free[kind] = sorted(self.free[kind] + self.held[kind][b])
            self.held[kind][b] = []

    def tables(self):
        return {k: [list(x) for x in v] for k, v in self.held.items()}


def kv_rows_image(layout, stacks, onto=None):
    """Expected bytes of the K and V row regions (the first rows_bytes() bytes of the K/V arena) given one
    stack oracle (of the layout's mode) per slot (None for a free slot).  Unwritten bytes are zero, or keep
    what `onto` holds: an earlier image of the same arena (rows of sequences that have left stay behind)."""
    img = np.zeros(layout.rows_bytes(), dtype=np.uint8) if onto is None else onto.copy()
    rowb = layout.D * layout.e
    for b, st in enumerate(stacks):
        if st is None:
            continue
        for l in range(layout.N):
            for h in range(layout.H):
                for rows, offset_of in ((st.Kc[l][h], layout.k_offset), (st.Vc[l][h], layout.v_offset)):
                    _write_rows(img, layout, rows, lambda r: offset_of(l, b, h, r))
    return img


def q_arena_image(layout, stacks, onto=None):
    img = np.zeros(layout.q_arena_bytes(), dtype=np.uint8) if onto is None else onto.copy()
    rowb = layout.D * layout.e
    for b, st in enumerate(stacks):
        if st is None or st.q_owner < 0:
            continue
        for h in range(layout.H):
            _write_rows(img, layout, st.Qc[h], lambda r: layout.q_offset(b, h, r))
    return img


def resident_bytes(layout, stacks):
    """Bytes actually occupied by cached rows: dict(k_bytes, v_bytes, q_bytes, tokens)."""
    per_row = layout.H * layout.D * layout.e
    k = v = q = tokens = 0
    for st in stacks:
        if st is None:
            continue
        rk, rv, rq = st.resident_rows()
        k += rk * per_row
        v += rv * per_row
        q += rq * per_row
        tokens += st.len if st.len else st.prefill_len
    return {"k_bytes": k, "v_bytes": v, "q_bytes": q, "tokens": tokens}


def standard_kv_bytes(layout, lens):
    """K + V bytes of the same sequences without lazy layers (every layer keeps every row)."""
    return 2 * layout.N * sum(lens) * layout.H * layout.D * layout.e


def vla_kv_saving_closed_form(n_layers, n_lazy, vis_len, text_len):
    """"Efficiency Analysis", KV Cache paragraph: |V|/(|V|+|T|) * n/(2N), as an exact fraction."""
    from fractions import Fraction
    return Fraction(vis_len, vis_len + text_len) * Fraction(n_lazy, 2 * n_layers)


def gla_kv_saving_closed_form(n_layers, n_lazy):
    """"Efficiency Analysis", KV Cache paragraph: GLA saves n/(2N) of the KV cache, as an exact fraction."""
    from fractions import Fraction
    return Fraction(n_lazy, 2 * n_layers)


def q_cache_share_closed_form(n_layers):
    """Same paragraph: a Q Cache that holds every token is 1/(2N) of a standard KV cache."""
    from fractions import Fraction
    return Fraction(1, 2 * n_layers)


def max_batch_within(budget_bytes, n_layers, n_heads, head_dim, dtype, max_seq, max_vis, max_text, lazy_mask,
                     mode="vla", count_q=False, overhead=None):
    """Largest batch whose K and V rows (plus the Q arena with count_q) fit the budget: the comparison
    behind the maximum-batch figures of the "Efficiency Evaluation" paragraph.  Plain search upward.
    `overhead(batch, rows_bytes)` -> bytes an implementation keeps beside the rows (default: none)."""
    batch = 0
    while True:
        lay = ArenaLayout(n_layers, n_heads, head_dim, dtype, batch + 1, max_seq, max_vis, max_text, lazy_mask,
                          mode=mode)
        need = lay.rows_bytes() + (lay.q_arena_bytes() if count_q else 0)
        if overhead is not None:
            need += overhead(batch + 1, lay.rows_bytes())
        if need > budget_bytes:
            return batch
        batch += 1
