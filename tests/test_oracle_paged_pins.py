"""Pins for the paged arena layout (oracle.layout, `paged`, `PagePools`): offsets worked by hand, the
page hand-out rule replayed by hand, brute force that no two rows share bytes, and equality with the
uniform layout when every sequence holds its slot's pages in order."""
import numpy as np
import pytest

from oracle.layout import PAGE_ROWS, ArenaLayout, PagePools


def test_offsets_worked_by_hand():
    # 2 layers [normal, lazy], 2 heads of 64 bf16 elements (128-byte rows), 2 slots, 128 positions, 64 visual
    # and 64 text rows per slot: seq pool 4 pages, text pool 2, vis pool 2.  A page is 2 heads x 64 rows.
    tables = {"seq": [[3, 0], [1]], "text": [[1], [0]], "vis": [[0], [1]]}
    lay = ArenaLayout(2, 2, 64, "bf16", 2, 128, 64, 64, [0, 1], paged=tables)
    rb, page = 128, 2 * 64 * 128
    k1 = 2 * 2 * 128 * rb                       # layer 0's K block: max_batch*H*max_seq rows
    v0 = k1 + 2 * 2 * 64 * rb                   # layer 1 (lazy): max_batch*H*max_text rows
    # V, layer 0, slot 0, head 1, position 70: second page of the slot = page 0, row 6 of head 1
    assert lay.v_offset(0, 0, 1, 70) == v0 + 0 * page + (1 * 64 + 6) * rb
    # position 5 of the same: first page of the slot = page 3
    assert lay.v_offset(0, 0, 1, 5) == v0 + 3 * page + (1 * 64 + 5) * rb
    # K of the normal layer uses the same pages
    assert lay.k_offset(0, 0, 0, 64) == 0 * page + 0 * rb
    assert lay.k_offset(0, 1, 1, 63) == 1 * page + (64 + 63) * rb
    # K of the lazy layer: text pages; slot 0 holds text page 1
    assert lay.k_offset(1, 0, 1, 9) == k1 + 1 * page + (64 + 9) * rb
    # Q arena: vis pages
    assert lay.q_offset(1, 0, 7) == 1 * page + 7 * rb
    # a key inside the span of the lazy layer resolves to the first layer's row of the same position
    assert lay.locate_k(1, 0, 1, 66, 10, 60) == (0, 0 * page + (64 + 2) * rb)
    # behind the span: own text row 72 - 60 = 12
    assert lay.locate_k(1, 0, 1, 72, 10, 60) == (1, k1 + 1 * page + (64 + 12) * rb)
    with pytest.raises(AssertionError):         # position 128 lies on a page the slot does not hold
        lay.v_offset(0, 0, 0, 128)
    with pytest.raises(AssertionError):         # page 1 held by both slots
        ArenaLayout(2, 2, 64, "bf16", 2, 128, 64, 64, [0, 1], paged={"seq": [[1], [1]], "text": [[], []], "vis": [[], []]})
    with pytest.raises(AssertionError):         # the seq pool has 4 pages
        ArenaLayout(2, 2, 64, "bf16", 2, 128, 64, 64, [0, 1], paged={"seq": [[4], []], "text": [[], []], "vis": [[], []]})
    with pytest.raises(AssertionError):         # capacities must be whole pages
        ArenaLayout(2, 2, 64, "bf16", 2, 100, 64, 64, [0, 1], paged=tables)


def test_pages_in_slot_order_give_back_the_uniform_layout():
    args = (3, 2, 64, "f32", 3, 128, 64, 64, [0, 1, 0])
    a = ArenaLayout(*args)
    ident = {"seq": [[2 * b, 2 * b + 1] for b in range(3)], "text": [[b] for b in range(3)], "vis": [[b] for b in range(3)]}
    b_ = ArenaLayout(*args, paged=ident)
    assert a.rows_bytes() == b_.rows_bytes() and a.q_arena_bytes() == b_.q_arena_bytes()
    # with one head the page-major order is the slot-major order; with two heads a page interleaves the heads,
    # so only single-head stacks coincide row for row
    a1 = ArenaLayout(3, 1, 64, "f32", 3, 128, 64, 64, [0, 1, 0])
    b1 = ArenaLayout(3, 1, 64, "f32", 3, 128, 64, 64, [0, 1, 0], paged=ident)
    for l in range(3):
        for s in range(3):
            for r in range(a1.cap_k(l)):
                assert a1.k_offset(l, s, 0, r) == b1.k_offset(l, s, 0, r)
            for r in range(128):
                assert a1.v_offset(l, s, 0, r) == b1.v_offset(l, s, 0, r)
    for s in range(3):
        for r in range(64):
            assert a1.q_offset(s, 0, r) == b1.q_offset(s, 0, r)


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_rows_are_disjoint_and_inside_their_regions(mode):
    tables = {"seq": [[5, 0], [3], [1, 2, 4]], "text": [[2], [0], [1]], "vis": [[1], [], [0, 2]]}
    lay = ArenaLayout(3, 2, 64, "bf16", 3, 128, 64, 64, [0, 1, 0], mode=mode, paged=tables)
    rowb = 128
    owner = set()
    for l in range(3):
        for b in range(3):
            for h in range(2):
                kind = lay._k_kind(l)
                n_k = len(tables[kind][b]) * PAGE_ROWS if lay.cap_k(l) else 0
                for which, n in (("k", n_k), ("v", len(tables["seq"][b]) * PAGE_ROWS)):
                    for r in range(n):
                        off = lay.k_offset(l, b, h, r) if which == "k" else lay.v_offset(l, b, h, r)
                        lo, hi = (lay.off_k(l), lay.off_k(l + 1)) if which == "k" else (lay.off_v(l), lay.off_v(l) + lay.v_layer_bytes(l))
                        assert lo <= off and off + rowb <= hi and off % rowb == 0
                        assert off not in owner, "two rows share bytes"
                        owner.add(off)
    q_kind = "vis" if mode == "vla" else "seq"
    seen = set()
    for b in range(3):
        for h in range(2):
            for r in range(len(tables[q_kind][b]) * PAGE_ROWS):
                off = lay.q_offset(b, h, r)
                assert 0 <= off and off + rowb <= lay.q_arena_bytes() and off not in seen
                seen.add(off)


def test_page_hand_out_by_hand():
    """3 slots, 192 positions, 64 visual and 128 text rows each: 9 seq pages, 6 text pages, 3 vis pages."""
    pp = PagePools(3, 192, 64, 128)
    # prompts of 70 (20 visual), 64 (0 visual) and 130 (64 visual) tokens, slot after slot, pool after pool
    pp.prefill([0, 1, 2], [70, 64, 130], [20, 0, 64])
    t = pp.tables()
    assert t["seq"] == [[0, 1], [2], [3, 4, 5]]
    assert t["text"] == [[0], [1], [2, 3]]          # 50, 64 and 66 text rows
    assert t["vis"] == [[0], [], [1]]
    # a decode step: positions 70, 64 and 130 are stored; slot 1 opens a new page in both of its pools
    pp.decode_step([0, 1, 2], [70, 64, 130], [20, 0, 64])
    t = pp.tables()
    assert t["seq"] == [[0, 1], [2, 6], [3, 4, 5]]
    assert t["text"] == [[0], [1, 4], [2, 3]]
    # slot 0 leaves: its pages are the lowest free ones again
    pp.leave(0)
    assert pp.free["seq"] == [0, 1, 7, 8] and pp.free["text"] == [0, 5] and pp.free["vis"] == [0, 2]
    # a sequence of 100 tokens (30 visual) joins slot 0
    pp.prefill([0], {0: 100}, {0: 30})
    t = pp.tables()
    assert t["seq"][0] == [0, 1] and t["text"][0] == [0, 5] and t["vis"][0] == [0]
    # the pool runs dry: 2 free seq pages left (7, 8), a step that needs more fails before it changes anything
    pp.leave(1)
    assert pp.free["seq"] == [2, 6, 7, 8]
    with pytest.raises(MemoryError):
        pp.prefill([1], {1: 64 * 5}, {1: 0})


def test_global_mode_uses_the_position_pages_for_everything():
    pp = PagePools(2, 128, 64, 64, mode="gla")
    pp.prefill([0, 1], [65, 3], [10, 1])
    assert pp.tables() == {"seq": [[0, 1], [2]], "text": [[], []], "vis": [[], []]}
    lay = ArenaLayout(2, 1, 64, "bf16", 2, 128, 64, 64, [0, 1], mode="gla", paged=pp.tables())
    assert lay.q_offset(1, 0, 2) == (2 * 64 + 2) * 128     # Q Cache row = position, on the sequence's page
    assert lay.q_offset(0, 0, 64) == (1 * 64 + 0) * 128
