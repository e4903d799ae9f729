"""The acceptance rule the parity tests apply (tests/helpers.py), exercised on hand-made cases on the CPU:
lists it must accept and lists with a planted mistake it must refuse."""
import numpy as np
import pytest

from helpers import check_topk, tol

PAD = 0xFFFFFFFF


def _case():
    # 10 items; threshold 10 with a band of about 1.1e-3: items 0..3 certain survivors, 4..6 inside the band,
    # 7..9 clearly pruned; full distances in item order except that certain survivor 3 is the farthest
    P = np.array([1.0, 2.0, 3.0, 4.0, 10.0002, 9.9998, 10.0005, 11.0, 12.0, 13.0])
    D = np.array([20.0, 21.0, 22.0, 40.0, 23.0, 21.5, 25.0, 5.0, 6.0, 7.0])
    return P, D, 10.0


def _list(ids, D, topk, order=True):
    ids = sorted(ids, key=lambda i: D[i]) if order else list(ids)
    out_ids = np.array(ids + [PAD] * (topk - len(ids)), dtype=np.int64)
    out_dist = np.array([D[i] for i in ids] + [np.inf] * (topk - len(ids)))
    return out_ids, out_dist


def test_band_items_may_fill_the_list_and_push_the_farthest_certain_survivor_out():
    P, D, t = _case()
    assert tol(t) > 6e-4
    topk = 5                                    # 4 certain survivors < topk < 7 with the band items
    check_topk(P, D, t, topk, *_list([0, 1, 2, 4, 5], D, topk))      # all three band items survived: 3 is pushed out
    check_topk(P, D, t, topk, *_list([0, 1, 2, 4, 3], D, topk))      # only one band item survived
    with pytest.raises(AssertionError):
        check_topk(P, D, t, topk, *_list([0, 1, 4, 5, 6], D, topk))  # a clearly closer certain survivor (2) is missing
    with pytest.raises(AssertionError):
        check_topk(P, D, t, topk, *_list([0, 1, 2, 4, 7], D, topk))  # a pruned item returned


def test_short_lists_hold_every_certain_survivor():
    P, D, t = _case()
    topk = 8                                    # more room than survivors and band items together
    check_topk(P, D, t, topk, *_list([0, 1, 2, 4, 5, 6, 3], D, topk))
    check_topk(P, D, t, topk, *_list([0, 1, 2, 3], D, topk))
    with pytest.raises(AssertionError):
        check_topk(P, D, t, topk, *_list([0, 1, 2, 4, 5, 6], D, topk))   # certain survivor 3 missing although there is room
    with pytest.raises(AssertionError):
        check_topk(P, D, t, topk, *_list([0, 1, 3, 2], D, topk, order=False))   # not ascending


def test_full_lists_respect_the_kth_distance():
    P, D, t = _case()
    topk = 3
    check_topk(P, D, t, topk, *_list([0, 1, 2], D, topk))
    check_topk(P, D, t, topk, *_list([0, 1, 5], D, topk))                # a band item that is nearer takes a place
    with pytest.raises(AssertionError):
        check_topk(P, D, t, topk, *_list([0, 1, 4], D, topk))            # a band item that is farther than the third cannot
    with pytest.raises(AssertionError):
        check_topk(P, D, t, topk, *_list([0, 1, 3], D, topk))            # farther than the k-th distance
    with pytest.raises(AssertionError):
        out_ids, out_dist = _list([0, 1, 2], D, topk)
        out_dist[1] += 0.1
        check_topk(P, D, t, topk, out_ids, out_dist)                     # a distance off
