"""Shared test helpers: threshold rules (computed with the CPU oracle) and the
acceptance rule that compares a GPU result with the oracle's."""
import numpy as np

PAD_ID = 0xFFFFFFFF


def tol(x):
    """Tolerance of the parity bar: 1e-4 * (|x| + 1)."""
    return 1e-4 * (np.abs(x) + 1.0)


def thresholds_kth(P, kth, factor=1.0):
    """t_q = factor * (kth-smallest crude distance of query q), rounded to fp32."""
    kth = min(kth, P.shape[1])
    part = np.partition(P, kth - 1, axis=1)[:, kth - 1]
    return (factor * part).astype(np.float32)


def thresholds_quantile(P, frac):
    """t_q = the ceil(frac*N)-th smallest crude distance of query q, rounded to fp32."""
    n = max(1, int(np.ceil(frac * P.shape[1])))
    return thresholds_kth(P, n, 1.0)


def check_candidates(P_q, t, ids, partial, count, cap):
    """Acceptance rule (i) for one query.  P_q: oracle crude distances [N] (f64);
    t: fp32 threshold; ids/partial: GPU list (first min(count,cap) entries valid)."""
    n = int(min(count, cap))
    got = np.asarray(ids[:n], dtype=np.int64)
    assert len(np.unique(got)) == n, "duplicate candidate ids"
    assert n == 0 or got.max() < P_q.shape[0], "candidate id out of range"
    t = float(t)
    band = tol(t) if np.isfinite(t) else 0.0
    must = np.nonzero(P_q < t - band)[0]
    may_not = P_q[got] > t + band
    assert not may_not.any(), "candidate beyond the threshold band"
    if count <= cap:
        missing = np.setdiff1d(must, got, assume_unique=True)
        assert missing.size == 0, "survivor missing from candidate list: %s" % missing[:8]
    err = np.abs(np.asarray(partial[:n], dtype=np.float64) - P_q[got])
    assert (err <= tol(P_q[got])).all(), "cand_partial off by %g" % err.max()


def check_topk(P_q, D_q, t, topk, out_ids, out_dist):
    """Acceptance rules (ii) and (iii) for one query.  D_q: oracle full distance
    of every item [N] (f64, computed for all items, not only survivors)."""
    t = float(t)
    band = tol(t) if np.isfinite(t) else 0.0
    out_ids = np.asarray(out_ids, dtype=np.int64)
    out_dist = np.asarray(out_dist, dtype=np.float64)
    valid = out_ids != PAD_ID
    nv = int(valid.sum())
    assert valid[:nv].all(), "padding must be a suffix"
    assert np.isinf(out_dist[nv:]).all() and (out_dist[nv:] > 0).all()
    ids = out_ids[:nv]
    assert len(np.unique(ids)) == nv, "duplicate ids in result"
    assert nv == 0 or ids.max() < P_q.shape[0]
    # (ii) distances
    err = np.abs(out_dist[:nv] - D_q[ids])
    assert (err <= tol(D_q[ids])).all(), "distance off by %g" % err.max()
    # ascending within tolerance
    if nv > 1:
        assert (np.diff(out_dist[:nv]) >= -2 * tol(out_dist[1:nv])).all(), "result not ascending"
    # every returned id is a survivor or lies in the threshold band
    assert (P_q[ids] <= t + band).all(), "returned id was pruned by the oracle"
    # (iii) set rule
    sure = np.nonzero(P_q < t - band)[0]           # certainly survivors
    maybe = np.nonzero(P_q <= t + band)[0]         # survivors or in the band
    assert nv >= min(topk, sure.size), "too few results"
    assert nv <= min(topk, maybe.size)
    if sure.size >= topk:
        # Items in the threshold band may or may not survive, and one that does can push a
        # certain survivor out of the list.  So: nothing returned may be farther than the
        # k-th distance with no band item surviving, and every certain survivor closer than
        # the k-th distance with ALL band items surviving must be there.
        Dk = np.partition(D_q[sure], topk - 1)[topk - 1]
        assert (D_q[ids] <= Dk + tol(Dk)).all(), "returned id farther than the k-th distance"
        Dk_all = np.partition(D_q[maybe], topk - 1)[topk - 1]
        need = sure[D_q[sure] < Dk_all - tol(Dk_all)]
        missing = np.setdiff1d(need, ids)
        assert missing.size == 0, "clearly-closer survivor missing: %s" % missing[:8]
    elif maybe.size <= topk:
        missing = np.setdiff1d(sure, ids)
        assert missing.size == 0, "survivor missing from a short result"
    else:
        # fewer certain survivors than topk, but with the band items more than topk: the band items that
        # survive can fill the list and push the farthest certain survivors out
        Dk_all = np.partition(D_q[maybe], topk - 1)[topk - 1]
        need = sure[D_q[sure] < Dk_all - tol(Dk_all)]
        missing = np.setdiff1d(need, ids)
        assert missing.size == 0, "clearly-closer survivor missing: %s" % missing[:8]


def tiled_loop_analysis(P_q, D_q, sigma, topk, bounds, band):
    """Follows the oracle's tiled search loop (crude comparison against the list as it stands at the
    start of a tile) for one query on the oracle's own crude distances P_q and distances D_q, and
    reports which of its decisions a computation with rounding errors up to band(x) could take
    differently.  Returns (list ids ascending by (D, id), least and most exact comparisons, clean);
    clean: no item within the band of a tile's threshold could enter the list, and neither the cut
    of the list nor its furthest element (whose crude distance is the next threshold) hangs on
    distances closer than the band.  With band = 0 this is the oracle's loop itself."""
    ids = np.empty(0, dtype=np.int64)
    lo = hi = 0
    clean = True
    for r in range(len(bounds) - 1):
        a, b = int(bounds[r]), int(bounds[r + 1])
        tile = np.arange(a, b, dtype=np.int64)
        maybe = np.empty(0, dtype=np.int64)
        if ids.size == topk:
            t = P_q[ids[-1]] + sigma
            w = band(t)
            sure = tile[P_q[a:b] < t - w]
            if w > 0:
                maybe = tile[np.abs(P_q[a:b] - t) <= w]
        else:
            sure = tile
        lo += sure.size
        hi += sure.size + maybe.size
        cand = np.concatenate([ids, sure])
        order = cand[np.lexsort((cand, D_q[cand]))]
        ids = order[:topk]
        if ids.size == topk:
            Dk = D_q[ids[-1]]
            w = band(Dk)
            if maybe.size and (D_q[maybe] <= Dk + w).any():
                clean = False
            if w > 0 and order.size > topk and D_q[order[topk]] - Dk <= w:
                clean = False
            if w > 0 and topk > 1 and Dk - D_q[ids[-2]] <= w:
                clean = False
    return ids, lo, hi, clean
