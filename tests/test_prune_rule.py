"""The grouped search kernel skips a fast-code tuple when its crude distance P satisfies
P > D_k * (1 + 1e-5) - S_min  (fp32; D_k = the list's topk-th distance, S_min = the fp32 sum of
the remaining tables' smallest entries).  This must never skip an item that could enter the
list: for non-negative tables every item of such a tuple has an fp32 distance (k ascending,
as every kernel adds it up) above D_k.  Checked here on the CPU, in numpy fp32, on the
adversarial side: items that take the smallest entry of every remaining table."""
import numpy as np


def fp32_sum(P, cols):
    d = np.float32(P)
    for c in cols:
        d = np.float32(d + np.float32(c))
    return d


def test_a_pruned_tuple_cannot_hold_a_list_entry():
    rng = np.random.default_rng(7)
    one = np.float32(1.0) + np.float32(1e-5)
    for trial in range(300):
        slow = rng.integers(1, 15)
        scale = np.float32(10.0 ** rng.uniform(-3, 4))
        tables = (rng.random((slow, 256), dtype=np.float32) ** 2 * scale).astype(np.float32)
        if trial % 7 == 0:
            tables[rng.integers(0, slow)] *= np.float32(1e-6)      # one table that hardly matters
        if trial % 11 == 0:
            tables[:, 0] = 0.0                                     # exact zeros as minima
        mins = tables.min(axis=1)
        smin = np.float32(0.0)
        for v in mins:
            smin = np.float32(smin + v)
        # a list bound: the distance of some item
        Dk = fp32_sum(np.float32(rng.random() * scale), tables[np.arange(slow), rng.integers(0, 256, slow)])
        tb = np.float32(np.float32(Dk * one) - smin)
        if not tb > 0:
            tb = np.float32(0.0)
        # crude distances just above the pruning threshold, then further out
        P = tb
        for step in range(200):
            P = np.nextafter(P, np.float32(np.inf), dtype=np.float32) if step < 100 else np.float32(P * np.float32(1.01) + np.float32(1e-30))
            assert P > tb
            # the closest any item of that tuple can be: the smallest entry of every remaining table
            assert fp32_sum(P, mins) > Dk, (trial, step, P, tb, Dk, smin)
            # and a random item of it
            assert fp32_sum(P, tables[np.arange(slow), rng.integers(0, 256, slow)]) > Dk


def test_a_tuple_at_the_bound_itself_is_kept():
    # all-zero remaining tables: D = P, so a tuple with P == D_k must stay (ties are decided by id later)
    Dk = np.float32(3.25)
    one = np.float32(1.0) + np.float32(1e-5)
    tb = np.float32(np.float32(Dk * one) - np.float32(0.0))
    assert not (Dk > tb)
    # and with everything zero nothing at zero is skipped
    tb0 = np.float32(np.float32(np.float32(0.0) * one) - np.float32(0.0))
    assert not (np.float32(0.0) > tb0)
