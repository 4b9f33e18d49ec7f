"""Pins of the oracle's rearrangement composition with several sub-sequences per example and
modality (Sec. 6, subsequence assembly), independent of the oracle's own placement code."""
import numpy as np
import pytest

import oracle
import workloads as wl
from test_oracle_dispatch import dst_starts, encoder_rows


def piece_case(cid, shrink, keep, seed, max_pieces=4):
    w = wl.WORKLOADS[cid]
    L = (wl.draw_lengths(w)[:keep] // shrink).astype(np.int32)
    split = wl.draw_modality_split(w, L)
    return w, L, split, wl.draw_piece_layout(split, seed, max_pieces)


@pytest.mark.parametrize("cid,shrink,keep,seed", [(4, 16, 300, 1), (1, 1, 64, 2), (3, 2, 400, 3)])
def test_tag_placement_built_in_numpy(cid, shrink, keep, seed):
    """Expected buffer from the assignment's fields alone: example s's run of modality rows, in
    original-order numbering, is dealt out piece by piece at start(s) + piece_off.  The three
    modalities' pieces must tile the packed batch exactly once."""
    w, L, split, lay = piece_case(cid, shrink, keep, seed)
    H, Dm, De = 12, w.D, max(2, w.D // 2)
    masg = oracle.balance(L, Dm, w.a, w.b)
    start = dst_starts(masg, Dm)
    T = int(L.sum())
    packed = np.full((T, H), 0xFFFF, dtype=np.uint16)
    want = np.full((T, H), 0xFFFF, dtype=np.uint16)
    hits = np.zeros(T, dtype=np.int32)
    for m in range(3):
        sub = np.ascontiguousarray(split[:, m])
        pp, po, pl = lay[m]
        easg = None if m == 0 else oracle.balance(sub, De, 1, 4 + m)
        salt = m * (1 << 30)
        rows, cu0 = encoder_rows(sub, easg, De, H, salt)
        oracle.pack_composed_pieces(rows, packed, pp, po, pl, easg, masg)
        for s in range(len(L)):
            taken = 0
            for p in range(pp[s], pp[s + 1]):
                d0 = start[s] + po[p]
                want[d0: d0 + pl[p]] = wl.token_tag_np(salt + cu0[s] + taken + np.arange(pl[p]), H)
                hits[d0: d0 + pl[p]] += 1
                taken += pl[p]
            assert taken == sub[s]
    assert (hits == 1).all()
    assert np.array_equal(packed, want)


def test_one_piece_per_example_is_the_plain_composition():
    w = wl.WORKLOADS[4]
    L = (wl.draw_lengths(w)[:350] // 8).astype(np.int32)
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, 5)
    H, De = 8, 6
    masg = oracle.balance(L, w.D, w.a, w.b)
    T = int(L.sum())
    for m in range(3):
        sub = np.ascontiguousarray(split[:, m])
        easg = oracle.balance(sub, De, 1, 9) if m else None
        rows, _ = encoder_rows(sub, easg, De, H, 11 * m)
        a = np.full((T, H), 0xEEEE, dtype=np.uint16)
        b = a.copy()
        oracle.pack_composed(rows, a, sub, sub_off[:, m], easg, masg)
        # one piece per example, also for empty sub-sequences (a piece of length 0)
        pp = np.arange(len(L) + 1, dtype=np.int32)
        oracle.pack_composed_pieces(rows, b, pp, sub_off[:, m], sub, easg, masg)
        assert np.array_equal(a, b)
        # an instance sub-range gives the matching slice
        lo, hi = 3, 9
        part = np.full((int(masg.tok_off[hi] - masg.tok_off[lo]), H), 0xEEEE, dtype=np.uint16)
        oracle.pack_composed_pieces(rows, part, pp, sub_off[:, m], sub, easg, masg, lo, hi)
        assert np.array_equal(part, a[int(masg.tok_off[lo]): int(masg.tok_off[hi])])


def test_cutting_a_piece_in_two_changes_nothing():
    w, L, split, lay = piece_case(4, 16, 200, 9, max_pieces=2)
    H = 6
    masg = oracle.balance(L, w.D, w.a, w.b)
    T = int(L.sum())
    sub = np.ascontiguousarray(split[:, 1])
    pp, po, pl = lay[1]
    easg = oracle.balance(sub, 5, 1, 3)
    rows, _ = encoder_rows(sub, easg, 5, H, 0)
    a = np.zeros((T, H), dtype=np.uint16)
    oracle.pack_composed_pieces(rows, a, pp, po, pl, easg, masg)
    # cut every piece of two or more rows after its first row
    npp, npo, npl = [0], [], []
    for s in range(len(L)):
        for p in range(pp[s], pp[s + 1]):
            if pl[p] >= 2:
                npo += [po[p], po[p] + 1]
                npl += [1, pl[p] - 1]
            else:
                npo.append(po[p])
                npl.append(pl[p])
        npp.append(len(npo))
    b = np.zeros((T, H), dtype=np.uint16)
    oracle.pack_composed_pieces(rows, b, np.array(npp, np.int32), np.array(npo, np.int32), np.array(npl, np.int32),
                                easg, masg)
    assert np.array_equal(a, b)


def test_refused_layouts():
    L = np.array([10, 6, 8], dtype=np.int32)
    asg = oracle.balance(L, 2, 0, 1)
    rows = wl.token_tag_np(np.arange(12), 4)
    out = np.zeros((24, 4), dtype=np.uint16)
    pp = np.array([0, 2, 3, 4], dtype=np.int32)
    ok_off, ok_len = np.array([0, 5, 1, 2], np.int32), np.array([3, 5, 2, 2], np.int32)
    oracle.pack_composed_pieces(rows, out, pp, ok_off, ok_len, None, asg)
    for off, ln in (([0, 2, 1, 2], [3, 5, 2, 2]),      # second piece starts inside the first
                    ([5, 0, 1, 2], [5, 3, 2, 2]),      # pieces of an example in descending order
                    ([0, 6, 1, 2], [3, 5, 2, 2]),      # piece runs past the end of its sequence (10 rows)
                    ([0, 5, 1, -1], [3, 5, 2, 2]),     # negative offset
                    ([0, 5, 1, 2], [3, -5, 2, 2])):    # negative length
        with pytest.raises(oracle.OracleError):
            oracle.pack_composed_pieces(rows, out, pp, np.array(off, np.int32), np.array(ln, np.int32), None, asg)
    # an encoder segment shorter than the example's pieces together is refused
    sub = np.array([8, 2, 2], dtype=np.int32)
    easg = oracle.balance(np.array([7, 2, 2], dtype=np.int32), 2, 0, 1)
    with pytest.raises(oracle.OracleError):
        oracle.pack_composed_pieces(rows, out, pp, ok_off, ok_len, easg, asg)
    assert int(sub.sum()) == 12
