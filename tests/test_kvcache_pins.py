"""Pins for the cache-layout definitions in oracle/kvcache.py (index and byte work, so every comparison is exact).

The expected values are typed by hand for tiny cases, or come from independent code: the scatter in the input
generator (workloads.make_paged / with_room) is the inverse of the gather under test and shares nothing with it.
"""
import numpy as np

import oracle
from paper_2402_05099_amd import workloads as wl


def labelled_pool(n_rows, Hkv=1, D=2, base=0):
    """row r holds the value base + r in every element, so a gathered row names where it came from"""
    return (np.arange(n_rows, dtype=np.uint16)[:, None, None] + np.uint16(base)) * np.ones((1, Hkv, D), np.uint16)


def test_paged_gather_hand_typed():
    # 4 pages of 4 rows; sequence 0 uses pages 2 then 0 (6 rows), sequence 1 nothing, sequence 2 page 3 (1 row)
    K, V = labelled_pool(16), labelled_pool(16, base=100)
    table = np.array([[2, 0, -1], [-1, -1, -1], [3, -1, -1]], np.int32)
    Ks, Vs, off = oracle.paged_to_packed(K, V, table, 4, np.array([6, 0, 1], np.int32))
    assert off.tolist() == [0, 6, 6]
    assert Ks[:, 0, 0].tolist() == [8, 9, 10, 11, 0, 1, 12]
    assert Vs[:, 0, 1].tolist() == [108, 109, 110, 111, 100, 101, 112]


def test_paged_gather_inverts_the_generator_scatter():
    w = wl.make_workload("p", 71, 9, 4, 2, 64, [(1, 8, 9)], 0, 70)
    for ps in (16, 32, 64):
        pg = wl.make_paged(w, ps, reserve=5)
        Ks, Vs, off = oracle.paged_to_packed(pg.K, pg.V, pg.table, ps, w.lengths)
        assert np.array_equal(off, w.offsets) and np.array_equal(Ks, w.Ks) and np.array_equal(Vs, w.Vs)
        used = pg.table[pg.table >= 0]
        assert len(set(used.tolist())) == used.size and used.max() < pg.n_pages   # a page has one owner


def test_paged_attention_is_invariant_under_page_placement():
    # the same logical rows behind two different physical placements give the same attention
    w = wl.make_workload("p", 72, 5, 4, 2, 64, [(1, 20, 5)], 3, 40)
    ref = oracle.attention(w)
    for ps in (16, 32):
        pg = wl.make_paged(w, ps)
        Ks, Vs, off = oracle.paged_to_packed(pg.K, pg.V, pg.table, ps, w.lengths)
        lv = [(l.K, l.V, l.kv_off, l.seq_off) for l in w.levels]
        got = oracle.attention_arrays(w.Q, w.Hkv, lv, Ks, Vs, off, w.lengths, w.scale)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


def test_append_hand_typed_packed():
    # two sequences with room for 3 rows each; lengths 1 and 3 (full): the second drops its new row
    Ks, Vs = labelled_pool(6), labelled_pool(6, base=50)
    Kn = np.array([[[[70, 70]]], [[[71, 71]]]], np.uint16)[:, 0]   # [B=2, Hkv=1, D=2]
    Vn = Kn + np.uint16(10)
    K2, V2, L2 = oracle.kv_append(Ks, Vs, np.array([0, 3], np.int32), np.array([1, 3], np.int32), 3, Kn, Vn)
    assert L2.tolist() == [2, 3]
    assert K2[:, 0, 0].tolist() == [0, 70, 2, 3, 4, 5]
    assert V2[:, 0, 0].tolist() == [50, 80, 52, 53, 54, 55]
    assert Ks[1, 0, 0] == 1   # inputs untouched


def test_append_several_rows_hits_the_capacity_midway():
    Ks, Vs = labelled_pool(8), labelled_pool(8, base=50)
    Kn = (np.arange(6, dtype=np.uint16).reshape(2, 3, 1, 1) + np.uint16(200)) * np.ones((1, 1, 1, 2), np.uint16)
    K2, V2, L2 = oracle.kv_append(Ks, Vs, np.array([0, 4], np.int32), np.array([0, 2], np.int32), 4, Kn, Kn)
    assert L2.tolist() == [3, 4]
    assert K2[:, 0, 0].tolist() == [200, 201, 202, 3, 4, 5, 203, 204]   # sequence 1 keeps two of its three rows


def test_append_hand_typed_paged():
    # pages of 4 rows; sequence 0 (length 4) crosses into its second page 1; sequence 1 (length 2) stays in page 0
    K, V = labelled_pool(12), labelled_pool(12, base=50)
    table = np.array([[2, 1], [0, -1]], np.int32)
    Kn = np.array([[[90, 90]], [[91, 91]]], np.uint16)
    K2, V2, L2 = oracle.kv_append_paged(K, V, table, 4, np.array([4, 2], np.int32), 8, Kn, Kn)
    assert L2.tolist() == [5, 3]
    want = list(range(12))
    want[4] = 90    # page 1, row 0
    want[2] = 91    # page 0, row 2
    assert K2[:, 0, 0].tolist() == want


def test_append_then_gather_equals_appending_to_the_packed_rows():
    w = wl.make_workload("p", 73, 7, 4, 2, 64, [], 0, 37, nq=2)
    Kn, Vn = wl.new_rows(w)
    Kr, Vr, offr, cap = wl.with_room(w, 3)
    K2, V2, L2 = oracle.kv_append(Kr, Vr, offr, w.lengths, cap, Kn, Vn)
    assert np.array_equal(L2, np.minimum(w.lengths + 2, cap))
    pg = wl.make_paged(w, 16, reserve=3)
    Kp, Vp, Lp = oracle.kv_append_paged(pg.K, pg.V, pg.table, 16, w.lengths, pg.capacity, Kn, Vn)
    assert np.array_equal(Lp, L2)
    Kg, Vg, offg = oracle.paged_to_packed(Kp, Vp, pg.table, 16, Lp)
    for b in range(w.B):
        n = int(L2[b])
        assert np.array_equal(Kg[offg[b]: offg[b] + n], K2[offr[b]: offr[b] + n])
        assert np.array_equal(Vg[offg[b]: offg[b] + n], V2[offr[b]: offr[b] + n])
        old = int(w.lengths[b])
        assert np.array_equal(K2[offr[b] + old: offr[b] + n], Kn[b, : n - old])   # the new rows, in token order
