"""Pins for the per-sequence-capacity arena layout (oracle.layout, `ragged`): worked by hand, against the
equal-capacity layout, and by brute force over every row."""
import numpy as np
import pytest

from oracle.layout import ArenaLayout


def test_offsets_worked_by_hand():
    # 2 heads of 64 bf16 elements: a row is 128 bytes.  Two sequences with 8 and 16 positions.
    lay = ArenaLayout(2, 2, 64, "bf16", 2, 12, 6, 6, [0, 1], ragged=([8, 16], [4, 8], [3, 5]))
    row = 128
    # V region of layer 1: sequence 1 starts after sequence 0's 8 rows x 2 heads; head 1 after head 0's 16 rows
    assert lay.v_offset(1, 1, 1, 3) - lay.off_v(1) == (8 * 2 + 1 * 16 + 3) * row
    assert lay.v_offset(0, 0, 1, 0) - lay.off_v(0) == (0 + 1 * 8 + 0) * row
    # layer 1 is lazy: its K block holds text rows only, 4 and 8 per head
    assert lay.k_offset(1, 1, 0, 7) - lay.off_k(1) == (4 * 2 + 0 * 8 + 7) * row
    assert lay.k_offset(0, 1, 0, 7) - lay.off_k(0) == (8 * 2 + 0 * 16 + 7) * row
    # Q arena: 3 and 5 visual rows per head
    assert lay.q_offset(1, 1, 4) == (3 * 2 + 1 * 5 + 4) * row
    # region sizes are those of the pools, whatever the split
    assert lay.off_k(1) == 2 * 2 * 12 * row and lay.off_k(2) - lay.off_k(1) == 2 * 2 * 6 * row


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_equal_capacities_give_back_the_uniform_layout(mode):
    args = (4, 3, 64, "f32", 3, 20, 12, 9, [0, 1, 1, 0])
    a = ArenaLayout(*args, mode=mode)
    b = ArenaLayout(*args, mode=mode, ragged=([20] * 3, [9] * 3, [12] * 3))
    assert a.rows_bytes() == b.rows_bytes() and a.q_arena_bytes() == b.q_arena_bytes()
    for l in range(4):
        for s in range(3):
            for h in range(3):
                for r in range(a.cap_k(l)):
                    assert a.k_offset(l, s, h, r) == b.k_offset(l, s, h, r)
                for r in range(20):
                    assert a.v_offset(l, s, h, r) == b.v_offset(l, s, h, r)
    for s in range(3):
        for h in range(3):
            for r in range(a.cap_q()):
                assert a.q_offset(s, h, r) == b.q_offset(s, h, r)


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_rows_are_disjoint_and_inside_their_regions(mode):
    caps = ([24, 8, 40, 8], [16, 0, 8, 8], [10, 8, 30, 0])
    lay = ArenaLayout(3, 2, 64, "bf16", 4, 20, 12, 8, [0, 1, 0], mode=mode, ragged=caps)
    rowb = 128
    owner = np.full(lay.rows_bytes() // rowb, -1, dtype=np.int64)
    tag = 0
    for l in range(3):
        k_caps = caps[0] if lay._k_kind(l) == "seq" else caps[1]
        for b in range(4):
            for h in range(2):
                rows = k_caps[b] if lay.cap_k(l) else 0
                for which, n in (("k", rows), ("v", caps[0][b])):
                    for r in range(n):
                        off = lay.k_offset(l, b, h, r) if which == "k" else lay.v_offset(l, b, h, r)
                        lo, hi = (lay.off_k(l), lay.off_k(l + 1)) if which == "k" else (lay.off_v(l), lay.off_v(l) + lay.v_layer_bytes(l))
                        assert lo <= off and off + rowb <= hi and off % rowb == 0
                        assert owner[off // rowb] == -1, "two rows share bytes"
                        owner[off // rowb] = tag
                        tag += 1
    q_caps = caps[2] if mode == "vla" else caps[0]
    seen = set()
    for b in range(4):
        for h in range(2):
            for r in range(q_caps[b]):
                off = lay.q_offset(b, h, r)
                assert 0 <= off and off + rowb <= lay.q_arena_bytes() and off not in seen
                seen.add(off)


def test_pools_bound_the_capacities():
    with pytest.raises(AssertionError):
        ArenaLayout(2, 1, 64, "bf16", 2, 10, 5, 5, [0, 1], ragged=([16, 8], [4, 4], [2, 2]))     # 24 > 2 x 10 positions
    with pytest.raises(AssertionError):
        ArenaLayout(2, 1, 64, "bf16", 2, 10, 5, 5, [0, 1], ragged=([8, 8], [8, 4], [2, 2]))      # 12 > 2 x 5 text rows
    ArenaLayout(2, 1, 64, "bf16", 2, 10, 5, 5, [0, 1], mode="gla", ragged=([8, 8], [8, 4], [2, 2]))  # text rows size nothing under GLA


def test_smaller_late_layers_worked_by_hand_and_against_the_uniform_layout():
    row = 128
    # 4 layers (layer 2 lazy), boundary before layer 1: layers 1..3 hold 8 positions instead of 20
    lay = ArenaLayout(4, 2, 64, "bf16", 3, 20, 12, 9, [0, 0, 1, 0], late=(1, 8))
    assert [lay.cap_k(l) for l in range(4)] == [20, 8, 9, 8]
    assert [lay.cap_v(l) for l in range(4)] == [20, 8, 8, 8]
    assert lay.off_k(1) == 3 * 2 * 20 * row and lay.off_k(2) - lay.off_k(1) == 3 * 2 * 8 * row
    assert lay.off_v(0) == lay.off_k(4) == 3 * 2 * (20 + 8 + 9 + 8) * row
    assert lay.off_v(2) - lay.off_v(0) == 3 * 2 * (20 + 8) * row
    assert lay.v_offset(3, 2, 1, 5) - lay.off_v(3) == ((2 * 2 + 1) * 8 + 5) * row
    assert lay.k_offset(1, 1, 0, 7) - lay.off_k(1) == ((1 * 2 + 0) * 8 + 7) * row
    # a late capacity equal to max_seq changes nothing
    a = ArenaLayout(4, 2, 64, "bf16", 3, 20, 12, 9, [0, 0, 1, 0])
    b = ArenaLayout(4, 2, 64, "bf16", 3, 20, 12, 9, [0, 0, 1, 0], late=(1, 20))
    assert a.rows_bytes() == b.rows_bytes()
    assert all(a.v_offset(l, 2, 1, 19) == b.v_offset(l, 2, 1, 19) and a.off_k(l) == b.off_k(l) for l in range(4))


def test_first_fit_by_hand():
    """Extents in a pool of 30 rows: [4, 10) and [15, 20) in use.  Gaps: [0, 4), [10, 15), [20, 30)."""
    from oracle.layout import first_fit
    used = [(15, 5), (4, 6)]
    assert first_fit(used, 4, 30) == 0          # exactly the first gap
    assert first_fit(used, 5, 30) == 10         # too long for the first, exactly the second
    assert first_fit(used, 6, 30) == 20
    assert first_fit(used, 10, 30) == 20        # to the pool's last row
    assert first_fit(used, 11, 30) is None
    assert first_fit(used, 0, 30) == 0          # nothing wanted
    assert first_fit([], 30, 30) == 0 and first_fit([], 31, 30) is None
    assert first_fit([(0, 0), (7, 0)], 30, 30) == 0     # free slots hold no rows


def test_explicit_extents_by_hand():
    """Two slots of a VLA stack [normal, lazy], H = 2, D = 64, bf16 (128-byte rows), max_batch 2, max_seq 16,
    max_vis 6, max_text 8.  Slot 0 sits at position base 16 (cap 8), text base 5 (cap 4), Q base 2 (cap 3);
    slot 1 at 0 (cap 16), 0 (cap 5), 0 (cap 2): the order of the extents need not be the order of the slots."""
    lay = ArenaLayout(2, 2, 64, "bf16", 2, 16, 6, 8, [0, 1], ragged=([8, 16], [4, 5], [3, 2], [16, 0], [5, 0], [2, 0]))
    rb = 128
    k1 = 2 * 2 * 16 * rb                        # layer 0's K block holds max_batch*H*max_seq rows
    v0 = k1 + 2 * 2 * 8 * rb                    # layer 1 (lazy) holds max_batch*H*max_text rows
    # V, layer 0: slot 0 head 1 row 3 -> row index 16*2 + 1*8 + 3 = 43
    assert lay.v_offset(0, 0, 1, 3) == v0 + 43 * rb
    # lazy layer's K: slot 0 head 1 row 2 -> 5*2 + 1*4 + 2 = 16; slot 1 head 1 row 4 -> 0*2 + 1*5 + 4 = 9
    assert lay.k_offset(1, 0, 1, 2) == k1 + 16 * rb
    assert lay.k_offset(1, 1, 1, 4) == k1 + 9 * rb
    # Q arena: slot 0 head 0 row 0 -> 2*2 = 4; slot 1 head 1 row 1 -> 0 + 1*2 + 1 = 3
    assert lay.q_offset(0, 0, 0) == 4 * rb and lay.q_offset(1, 1, 1) == 3 * rb
    # a key inside the span of a lazy layer resolves to the first layer's row of the same position
    assert lay.locate_k(1, 0, 1, 2, 1, 3) == (0, (16 * 2 + 8 + 2) * rb)
    with pytest.raises(AssertionError):         # overlapping extents: [0, 16) and [8, 16)
        ArenaLayout(2, 2, 64, "bf16", 2, 16, 6, 8, [0, 1], ragged=([8, 16], [4, 5], [3, 2], [8, 0], [5, 0], [2, 0]))
    with pytest.raises(AssertionError):         # past the pool's end: 28 + 8 > 32
        ArenaLayout(2, 2, 64, "bf16", 2, 16, 6, 8, [0, 1], ragged=([8, 16], [4, 5], [3, 2], [28, 0], [5, 0], [2, 0]))
