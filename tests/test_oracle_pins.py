"""Pins for the CPU oracle: each test checks oracle/icq_oracle.c against something
the paper or the mathematics fixes, computed here in numpy by a different route
(reconstruction and brute force, sub-vector PQ tables, closed-form constants,
hand-worked values).  A dropped term, a wrong index, a transposed operand or a
wrong comparison sign in the oracle fails at least one of them."""
import os

import numpy as np
import pytest

from oracle import icq_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.Philox(key=[seed, 77]))


def disjoint_support_codebooks(g, K, m, d, scale=None):
    """Codebooks with pairwise-disjoint, interleaved coordinate supports (the ICQ
    zero pattern of Sec. 3.1 taken to its limit): inter-codebook inner products
    are all zero, so the constant cross term eps is 0."""
    perm = g.permutation(d)
    groups = np.array_split(perm, K)
    cb = np.zeros((K, m, d), dtype=np.float32)
    for k in range(K):
        s = 1.0 if scale is None else scale[k]
        cb[k][:, groups[k]] = (s * g.standard_normal((m, len(groups[k])))).astype(np.float32)
    return cb, groups


def constant_eps_codebooks(g, K, m, d_block):
    """c_{k,j} = u_{k,j} + a_k: u_{k,.} lives in coordinate block k, the offsets a_k
    all live in one extra block.  Then c_k^T c_l = a_k^T a_l for k != l whatever
    the codewords: eps = sum_{k != l} a_k^T a_l, a non-zero constant (the
    composite-quantization constraint of Sec. 2)."""
    d = (K + 1) * d_block
    cb = np.zeros((K, m, d), dtype=np.float32)
    a = g.standard_normal((K, d_block)).astype(np.float32)
    for k in range(K):
        cb[k][:, k * d_block:(k + 1) * d_block] = g.standard_normal((m, d_block)).astype(np.float32)
        cb[k][:, K * d_block:] = a[k]
    a64 = a.astype(np.float64)
    gram = a64 @ a64.T
    eps = gram.sum() - np.trace(gram)
    return cb, eps


def np_reconstruct(cb, codes):
    K = cb.shape[0]
    x = np.zeros((codes.shape[1], cb.shape[2]), dtype=np.float64)
    for k in range(K):
        x += cb[k].astype(np.float64)[codes[k]]
    return x


def np_knn(x, queries, topk):
    out = []
    for q in queries.astype(np.float64):
        dist = ((q[None, :] - x) ** 2).sum(axis=1)
        order = np.lexsort((np.arange(x.shape[0]), dist))[:topk]
        out.append((order, dist[order]))
    return out


# ---------------------------------------------------------------- P8: worked values
def _golden():
    vals = {}
    with open(os.path.join(GOLDEN, "micro_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = np.array([float(r) for r in rest])
    return vals


def test_micro_example_matches_hand_worked_values():
    gold = _golden()
    cb = np.array([[[1, 0], [-1, 0]], [[0, 1], [0, -1]]], dtype=np.float32)
    q = np.array([[0.5, 0.25]], dtype=np.float32)
    codes = np.array([[0, 0, 1, 1, 0], [0, 1, 0, 1, 0]], dtype=np.uint8)
    T = orc.lut(cb, q)
    assert np.array_equal(T[0, 0], gold["T0"]) and np.array_equal(T[0, 1], gold["T1"])
    P = orc.partial(T, codes, 1)
    assert np.array_equal(P[0], gold["P"])
    ids, dist, D = orc.adc_exhaustive(T, codes, 5, want_all=True)
    assert np.array_equal(D[0], gold["D"])
    t = np.array([1.0], dtype=np.float32)
    ids, dist, cnt, P2, D2 = orc.search(T, codes, 1, t, 2, want_all=True)
    assert cnt[0] == 3
    assert np.array_equal(np.nonzero(~np.isnan(D2[0]))[0], gold["survivors"].astype(int))
    assert np.array_equal(ids[0], gold["top2_ids"].astype(np.uint32))
    assert np.array_equal(dist[0], gold["top2_dist"])
    ids4, dist4, cnt4 = orc.search(T, codes, 1, t, 4)
    assert ids4[0, 3] == 0xFFFFFFFF and np.isposinf(dist4[0, 3]) and ids4[0, 2] == 1
    # strictness of "<": an item whose crude distance equals t is pruned
    t_eq = np.array([0.3125], dtype=np.float32)
    assert orc.search(T, codes, 1, t_eq, 2)[2][0] == 0
    # identity on item 0: D - (K-1)||q||^2 + eps == ||q - xbar||^2
    assert D[0, 0] - 0.3125 == gold["true_dist_item0"][0]
    x = orc.reconstruct(cb, codes, [0])
    assert np.array_equal(x[0], [1.0, 1.0])


# ---------------------------------------------------------------- P1: CQ distance identity
@pytest.mark.parametrize("kind", ["disjoint", "const_eps"])
def test_cq_distance_identity(kind):
    g = _rng(1)
    K, m, N, Q = 5, 16, 400, 7
    if kind == "disjoint":
        cb, _ = disjoint_support_codebooks(g, K, m, 23)
        eps = 0.0
    else:
        cb, eps = constant_eps_codebooks(g, K, m, 3)
        assert abs(eps) > 1e-3
    d = cb.shape[2]
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    _, _, D = orc.adc_exhaustive(T, codes, 1, want_all=True)
    x = np_reconstruct(cb, codes)
    q64 = queries.astype(np.float64)
    true = ((q64[:, None, :] - x[None, :, :]) ** 2).sum(axis=2)
    qn = (q64 ** 2).sum(axis=1)[:, None]
    lhs = D - (K - 1) * qn + eps
    np.testing.assert_allclose(lhs, true, rtol=1e-12, atol=1e-12)
    # the same identity through the two-step search with nothing pruned
    inf = np.full(Q, np.inf, dtype=np.float32)
    _, _, cnt, P, D2 = orc.search(T, codes, 2, inf, 3, want_all=True)
    assert (cnt == N).all()
    np.testing.assert_allclose(D2 - (K - 1) * qn + eps, true, rtol=1e-12, atol=1e-12)
    # the oracle's own reconstruction agrees with numpy's
    np.testing.assert_allclose(orc.reconstruct(cb, codes, np.arange(N)), x, rtol=0, atol=1e-15)


# ---------------------------------------------------------------- P2: t = +inf == exhaustive ADC
def test_infinite_threshold_equals_exhaustive_adc():
    g = _rng(2)
    K, m, d, N, Q, topk = 6, 256, 20, 3000, 9, 25
    cb = g.standard_normal((K, m, d)).astype(np.float32)   # dense: no CQ property needed
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    e_ids, e_dist = orc.adc_exhaustive(T, codes, topk)
    inf = np.full(Q, np.inf, dtype=np.float32)
    for Kf in (1, 2, 5, 6):
        ids, dist, cnt = orc.search(T, codes, Kf, inf, topk)
        assert np.array_equal(ids, e_ids)
        # K-term sums in the same (ascending k) order: bit-identical
        assert np.array_equal(dist, e_dist)
        assert (cnt == N).all()


# ---------------------------------------------------------------- P3: ADC top-k == brute-force k-NN
def test_adc_topk_equals_bruteforce_knn_on_cq_codebooks():
    g = _rng(3)
    K, m, N, Q, topk = 4, 32, 1500, 6, 12
    cb, _ = disjoint_support_codebooks(g, K, m, 16)
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    src = g.integers(0, N, size=Q)
    x = np_reconstruct(cb, codes)
    queries = (x[src] + 0.1 * g.standard_normal((Q, 16))).astype(np.float32)
    T = orc.lut(cb, queries)
    a_ids, a_dist = orc.adc_exhaustive(T, codes, topk)
    b_ids, b_dist = orc.bruteforce_knn(cb, codes, queries, topk)
    ref = np_knn(x, queries, topk)
    qn = (queries.astype(np.float64) ** 2).sum(axis=1)
    for q in range(Q):
        assert np.array_equal(b_ids[q], ref[q][0])            # oracle brute force vs numpy brute force
        np.testing.assert_allclose(b_dist[q], ref[q][1], rtol=1e-13)
        assert np.array_equal(a_ids[q], b_ids[q])             # Eq. 1: table sums rank like true distances
        np.testing.assert_allclose(a_dist[q] - (K - 1) * qn[q], b_dist[q], rtol=1e-11, atol=1e-11)
        assert a_ids[q][0] == src[q] or a_dist[q][0] <= a_dist[q][1]


# ---------------------------------------------------------------- P4: PQ special case
def test_pq_special_case_matches_subvector_tables():
    g = _rng(4)
    K, m, d, Q = 4, 64, 24, 5
    sub = d // K
    cb = np.zeros((K, m, d), dtype=np.float32)
    for k in range(K):
        cb[k][:, k * sub:(k + 1) * sub] = g.standard_normal((m, sub)).astype(np.float32)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    q64 = queries.astype(np.float64)
    for k in range(K):
        blk = slice(k * sub, (k + 1) * sub)
        # textbook PQ asymmetric table: sub-query against sub-codewords
        t_pq = ((q64[:, None, blk] - cb[k][None, :, blk].astype(np.float64)) ** 2).sum(axis=2)
        rest = (q64 ** 2).sum(axis=1) - (q64[:, blk] ** 2).sum(axis=1)
        np.testing.assert_allclose(T[:, k, :], t_pq + rest[:, None], rtol=1e-13, atol=1e-13)
    # and the K-table sum is the PQ-ADC distance plus the constant (K-1)||q||^2
    N = 300
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    _, _, D = orc.adc_exhaustive(T, codes, 1, want_all=True)
    x = np_reconstruct(cb, codes)
    pq = ((q64[:, None, :] - x[None]) ** 2).sum(axis=2)
    np.testing.assert_allclose(D, pq + (K - 1) * (q64 ** 2).sum(axis=1)[:, None], rtol=1e-12)


# ---------------------------------------------------------------- P5: filter / select commute
def test_filter_and_select_commute_and_survivors_are_monotone():
    g = _rng(5)
    K, Kf, m, d, N, Q, topk = 5, 2, 256, 12, 4000, 8, 15
    cb = (g.standard_normal((K, m, d)) * (0.6 ** np.arange(K))[:, None, None]).astype(np.float32)
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    P = orc.partial(T, codes, Kf)
    _, _, D_all = orc.adc_exhaustive(T, codes, 1, want_all=True)
    prev = None
    for frac in (0.002, 0.01, 0.2):
        n = int(np.ceil(frac * N))
        t = np.partition(P, n - 1, axis=1)[:, n - 1].astype(np.float32)
        ids, dist, cnt, P2, D2 = orc.search(T, codes, Kf, t, topk, want_all=True)
        assert np.array_equal(P2, P)
        for q in range(Q):
            keep = np.nonzero(P[q] < np.float64(t[q]))[0]
            assert cnt[q] == keep.size
            order = keep[np.lexsort((keep, D_all[q][keep]))][:topk]
            exp_ids = np.full(topk, 0xFFFFFFFF, dtype=np.uint32)
            exp_ids[:order.size] = order
            assert np.array_equal(ids[q], exp_ids)
            assert np.array_equal(dist[q][:order.size], D_all[q][order])
            assert np.array_equal(np.nonzero(~np.isnan(D2[q]))[0], keep)
        surv = ~np.isnan(D2)
        if prev is not None:
            assert (prev <= surv).all()          # S(t1) subset of S(t2) for t1 < t2
        prev = surv


# ---------------------------------------------------------------- P6: lossless pruning on ICQ-structured codebooks
def test_lossless_pruning_invariant_on_icq_structure():
    g = _rng(6)
    K, Kf, m, d, N, Q, topk = 6, 2, 64, 30, 2000, 10, 8
    # all supports disjoint; the two fast codebooks carry most of the variance
    cb, groups = disjoint_support_codebooks(g, K, m, d, scale=[2.0, 2.0, 0.3, 0.3, 0.3, 0.3])
    psi = np.concatenate(groups[:Kf])
    psibar = np.concatenate(groups[Kf:])
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    x = np_reconstruct(cb, codes)
    src = g.integers(0, N, size=Q)
    queries = (x[src] + 0.05 * g.standard_normal((Q, d))).astype(np.float32)
    q64 = queries.astype(np.float64)
    T = orc.lut(cb, queries)
    P = orc.partial(T, codes, Kf)
    # closed form: P - const_q is the exact distance inside the fast subspace
    const = (Kf - 1) * (q64[:, psi] ** 2).sum(axis=1) + Kf * (q64[:, psibar] ** 2).sum(axis=1)
    d_psi = ((q64[:, None, psi] - x[None][:, :, psi]) ** 2).sum(axis=2)
    np.testing.assert_allclose(P - const[:, None], d_psi, rtol=1e-11, atol=1e-11)
    ref = np_knn(x, queries, topk)
    t = np.array([ref[q][1][topk - 1] * (1 + 1e-6) + const[q] + 1e-6 for q in range(Q)], dtype=np.float32)
    ids, dist, cnt = orc.search(T, codes, Kf, t, topk)
    assert (cnt < N // 2).all(), "threshold should really prune"
    for q in range(Q):
        assert np.array_equal(ids[q], ref[q][0]), "a true nearest neighbour was pruned"


# ---------------------------------------------------------------- P7: degenerate settings
def test_kf_equals_k_and_padding():
    g = _rng(7)
    K, m, d, N, Q = 3, 256, 8, 500, 4
    cb = g.standard_normal((K, m, d)).astype(np.float32)
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    P = orc.partial(T, codes, K)
    t = np.partition(P, 4, axis=1)[:, 4].astype(np.float32)      # 5th smallest, rounded to fp32: 4 or 5 strictly below
    ids, dist, cnt, P2, D2 = orc.search(T, codes, K, t, 10, want_all=True)
    for q in range(Q):
        keep = ~np.isnan(D2[q])
        assert np.array_equal(D2[q][keep], P[q][keep])           # stage 2 adds nothing
        n = int(cnt[q])
        assert n in (4, 5) and (ids[q][n:] == 0xFFFFFFFF).all() and np.isposinf(dist[q][n:]).all()
        assert (np.diff(dist[q][:n]) >= 0).all()
    # empty database
    e = np.zeros((K, 0), dtype=np.uint8)
    ids, dist, cnt = orc.search(T, e, 1, t, 3)
    assert (cnt == 0).all() and (ids == 0xFFFFFFFF).all()


def test_tie_break_is_by_id():
    cb = np.zeros((1, 2, 1), dtype=np.float32)
    cb[0, 1, 0] = 1.0
    q = np.array([[0.0]], dtype=np.float32)
    codes = np.array([[1, 0, 0, 1, 0]], dtype=np.uint8)
    T = orc.lut(cb, q)
    ids, dist = orc.adc_exhaustive(T, codes, 5)
    assert ids[0].tolist() == [1, 2, 4, 0, 3]
    assert dist[0].tolist() == [0, 0, 0, 1, 1]


def test_lut_against_expanded_form_at_benchmark_shape():
    """||q-c||^2 == ||q||^2 - 2<q,c> + ||c||^2 (a different route, via a matmul)."""
    g = _rng(8)
    K, m, d, Q = 3, 256, 96, 5
    cb = g.standard_normal((K, m, d)).astype(np.float32)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    q64, c64 = queries.astype(np.float64), cb.astype(np.float64).reshape(K * m, d)
    ref = (q64 ** 2).sum(1)[:, None] - 2 * q64 @ c64.T + (c64 ** 2).sum(1)[None]
    np.testing.assert_allclose(T.reshape(Q, K * m), ref, rtol=1e-12)


# ================================================================ the paper's serial loop (Sec. 3.4),
# the sample threshold derived from it, and the operation counts
def _golden_file(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = np.array([float(r) for r in rest])
    return vals


def _micro_tables():
    cb = np.array([[[1, 0], [-1, 0]], [[0, 1], [0, -1]]], dtype=np.float32)
    q = np.array([[0.5, 0.25]], dtype=np.float32)
    return orc.lut(cb, q)


def test_running_search_matches_hand_worked_trace():
    gold = _golden_file("running_example.txt")
    T = _micro_tables()
    codes = np.stack([gold["codes0"], gold["codes1"]]).astype(np.uint8)
    topk = int(gold["topk"][0])
    sigma = np.array([gold["sigma"][0]])
    ids, dist, refined = orc.running_search(T, codes, 1, sigma, topk)
    assert np.array_equal(ids[0], gold["ids"].astype(np.uint32))
    assert np.array_equal(dist[0], gold["dist"])
    assert refined[0] == int(gold["refined"][0])
    assert orc.sample_thresholds(T, codes, 1, sigma, topk, 4)[0] == gold["thr_M4"][0]
    assert orc.sample_thresholds(T, codes, 1, sigma, topk, 7)[0] == gold["thr_M7"][0]
    assert orc.sample_thresholds(T, codes, 1, sigma, topk, 100)[0] == gold["thr_M7"][0]   # M beyond N
    assert np.isposinf(orc.sample_thresholds(T, codes, 1, sigma, 8, 7)[0])                 # fewer items than topk
    ops, summary = orc.op_counts(7, 2, 1, refined, 2.0)
    assert ops[0] == gold["ops_icq"][0] and summary[1] == gold["ops_adc"][0]
    assert summary[0] == gold["ops_icq"][0] and summary[2] == gold["ops_icq"][0] / gold["ops_adc"][0]
    assert abs(summary[3] - gold["effective_bits"][0]) < 1e-15
    # a longer list than items: everything is refined, padding follows
    ids9, dist9, ref9 = orc.running_search(T, codes, 1, sigma, 9)
    assert ref9[0] == 7 and ids9[0, 7] == 0xFFFFFFFF and np.isposinf(dist9[0, 8])
    assert np.array_equal(ids9[0, :7], [4, 2, 6, 1, 3, 5, 0])


def test_tiled_running_search_matches_hand_worked_traces():
    gold = _golden_file("running_example.txt")
    T = _micro_tables()
    codes = np.stack([gold["codes0"], gold["codes1"]]).astype(np.uint8)
    topk = int(gold["topk"][0])
    sigma = np.array([gold["sigma"][0]])
    for tag in ("a", "b"):
        ids, dist, refined = orc.running_search_tiled(T, codes, 1, sigma, topk, gold["tiles_" + tag].astype(np.int64))
        assert np.array_equal(ids[0], gold["ids"].astype(np.uint32))
        assert np.array_equal(dist[0], gold["dist"])
        assert refined[0] == int(gold["refined_" + tag][0]), tag


def _random_case(seed, K=6, Kf=2, N=4000, Q=7, d=12):
    g = _rng(seed)
    cb = (g.standard_normal((K, 256, d)) * (0.7 ** np.arange(K))[:, None, None]).astype(np.float32)
    codes = g.integers(0, 256, size=(K, N), dtype=np.uint8)
    queries = g.standard_normal((Q, d)).astype(np.float32)
    T = orc.lut(cb, queries)
    return T, codes


def test_running_search_with_infinite_margin_is_exhaustive_adc():
    T, codes = _random_case(21)
    Q, N, topk = T.shape[0], codes.shape[1], 30
    e_ids, e_dist = orc.adc_exhaustive(T, codes, topk)
    ids, dist, refined = orc.running_search(T, codes, 2, np.full(Q, np.inf), topk)
    assert np.array_equal(ids, e_ids) and np.array_equal(dist, e_dist)
    assert (refined == N).all()


def test_running_search_loses_nothing_when_the_margin_exceeds_the_spread_of_the_slow_terms():
    """D = P + S with S the sum over the slow codebooks.  An item i of the true top-k has
    D(i) <= D(f) for the furthest list element f, hence P(i) <= P(f) + S(f) - S(i)
    <= P(f) + (max S - min S): with a margin above that spread the crude comparison never
    prunes a true neighbour, whatever the codebooks, and the list stays exact."""
    T, codes = _random_case(22)
    Q, N, topk, Kf = T.shape[0], codes.shape[1], 20, 2
    P = orc.partial(T, codes, Kf)
    _, _, D = orc.adc_exhaustive(T, codes, 1, want_all=True)
    S = D - P
    spread = S.max(axis=1) - S.min(axis=1)
    e_ids, e_dist = orc.adc_exhaustive(T, codes, topk)
    ids, dist, refined = orc.running_search(T, codes, Kf, spread * 1.0001, topk)
    assert np.array_equal(ids, e_ids) and np.array_equal(dist, e_dist)
    assert (refined < N).all()          # and it still prunes
    # a much smaller margin prunes more and (on these dense codebooks) loses neighbours
    ids0, _, refined0 = orc.running_search(T, codes, Kf, np.zeros(Q), topk)
    assert (refined0 < refined).all()
    assert (ids0 != e_ids).any()


def test_tiled_running_search_special_cases():
    """Tiles of one item are the serial loop; one tile is the exhaustive search; the two tiles
    [0, M) and [M, N) are the static threshold of the first M items applied to the rest."""
    T, codes = _random_case(23, N=3000)
    Q, N, Kf, topk = T.shape[0], codes.shape[1], 2, 10
    sigma = np.linspace(0.0, 3.0, Q)
    ids, dist, refined = orc.running_search(T, codes, Kf, sigma, topk)
    ids1, dist1, refined1 = orc.running_search_tiled(T, codes, Kf, sigma, topk, np.arange(N + 1))
    assert np.array_equal(ids, ids1) and np.array_equal(dist, dist1) and np.array_equal(refined, refined1)
    # empty tiles change nothing
    b = np.sort(np.concatenate([np.arange(N + 1), [0, 5, 5, N]]))
    ids2, dist2, refined2 = orc.running_search_tiled(T, codes, Kf, sigma, topk, b)
    assert np.array_equal(ids, ids2) and np.array_equal(refined, refined2)
    # one tile: no crude comparison at all
    e_ids, e_dist = orc.adc_exhaustive(T, codes, topk)
    idsw, distw, refinedw = orc.running_search_tiled(T, codes, Kf, sigma, topk, np.array([0, N]))
    assert np.array_equal(idsw, e_ids) and np.array_equal(distw, e_dist) and (refinedw == N).all()
    # two tiles against the composition of two other oracle functions
    M = 400
    thr = orc.sample_thresholds(T, codes, Kf, sigma, topk, M)
    P = orc.partial(T, codes, Kf)
    D = orc.adc_exhaustive(T, codes, topk, want_all=True)[2]
    ids3, dist3, refined3 = orc.running_search_tiled(T, codes, Kf, sigma, topk, np.array([0, M, N]))
    for q in range(Q):
        keep = np.concatenate([np.arange(M), M + np.nonzero(P[q, M:] < thr[q])[0]])
        assert refined3[q] == keep.size
        order = keep[np.lexsort((keep, D[q, keep]))][:topk]
        assert np.array_equal(ids3[q], order.astype(np.uint32))
        assert np.array_equal(dist3[q], D[q, order])
    # an infinite margin makes every crude comparison hold, whatever the tiles
    b4 = np.unique(np.concatenate([[0], np.arange(M, N + 1, 100), [N]]))
    ids4, dist4, refined4 = orc.running_search_tiled(T, codes, Kf, np.full(Q, np.inf), topk, b4)
    assert np.array_equal(ids4, e_ids) and np.array_equal(dist4, e_dist) and (refined4 == N).all()


def test_running_search_with_margin_minus_infinity_keeps_the_first_items():
    T, codes = _random_case(23)
    Q, topk = T.shape[0], 15
    ids, dist, refined = orc.running_search(T, codes, 2, np.full(Q, -np.inf), topk)
    assert (refined == topk).all()
    e_ids, e_dist = orc.adc_exhaustive(T, codes[:, :topk], topk)     # the first topk items, ordered
    assert np.array_equal(ids, e_ids) and np.array_equal(dist, e_dist)


def test_running_search_on_items_in_ascending_order_of_distance():
    """Visited nearest first, the list is final after topk items: nothing ever replaces an
    element, the furthest element stays item topk-1, so an item i >= topk gets the exact
    comparison iff P(i) < P(topk-1) + sigma -- a closed form for the refined count."""
    T, codes = _random_case(24, Q=1)
    Kf, topk = 2, 12
    _, _, D = orc.adc_exhaustive(T, codes, 1, want_all=True)
    order = np.argsort(D[0], kind="stable")
    codes_sorted = np.ascontiguousarray(codes[:, order])
    P = orc.partial(T, codes_sorted, Kf)[0]
    for sigma in (0.0, 0.3, 2.0):
        ids, dist, refined = orc.running_search(T, codes_sorted, Kf, np.array([sigma]), topk)
        assert np.array_equal(ids[0], np.arange(topk))
        expect = topk + int((P[topk:] < P[topk - 1] + sigma).sum())
        assert refined[0] == expect


def test_sample_threshold_is_the_crude_distance_of_the_kth_neighbour_plus_margin():
    T, codes = _random_case(25)
    Q, N, Kf, topk = T.shape[0], codes.shape[1], 2, 10
    sigma = np.linspace(0.0, 1.5, Q)
    P = orc.partial(T, codes, Kf)
    for M in (N, 500):
        e_ids, _ = orc.adc_exhaustive(T, codes[:, :M], topk)
        thr = orc.sample_thresholds(T, codes, Kf, sigma, topk, M)
        assert np.array_equal(thr, P[np.arange(Q), e_ids[:, topk - 1]] + sigma)
    # searching with that threshold keeps every item the serial loop could ever list once its
    # first M items are in: the k-th neighbour of the sample itself survives (P(f) < P(f) + sigma)
    thr = orc.sample_thresholds(T, codes, Kf, sigma + 0.5, topk, 500).astype(np.float32)
    ids, _, cnt = orc.search(T, codes, Kf, thr, topk)
    assert (cnt >= topk).all()


def test_op_counts_closed_forms():
    N, K, Kf = 1000, 8, 2
    ops, s = orc.op_counts(N, K, Kf, np.full(5, N), 64.0)      # everything refined: the one-step search
    assert (ops == N * K).all() and s[2] == 1.0 and s[3] == 64.0
    ops, s = orc.op_counts(N, K, Kf, np.zeros(5, dtype=np.int64), 64.0)   # nothing refined
    assert (ops == N * Kf).all() and s[2] == Kf / K and s[3] == 64.0 * Kf / K
    ops, s = orc.op_counts(N, K, Kf, np.array([10, 30]), 64.0)
    assert np.array_equal(ops, [N * Kf + 60, N * Kf + 180]) and s[0] == N * Kf + 120


# ================================================================ greedy encoding
def test_encode_with_one_codebook_is_the_nearest_codeword():
    g = _rng(31)
    cb = g.standard_normal((1, 200, 9)).astype(np.float32)
    x = g.standard_normal((500, 9)).astype(np.float32)
    codes, err = orc.encode(cb, x, want_err=True)
    d2 = ((x.astype(np.float64)[:, None, :] - cb[0].astype(np.float64)[None, :, :]) ** 2).sum(axis=2)
    assert np.array_equal(codes[0], d2.argmin(axis=1))
    assert np.allclose(err, d2.min(axis=1), rtol=1e-12, atol=0)


def test_encode_on_disjoint_supports_is_the_subvector_assignment_and_the_global_optimum():
    g = _rng(32)
    K, m, d, N = 3, 4, 7, 40
    cb, groups = disjoint_support_codebooks(g, K, m, d)
    x = g.standard_normal((N, d)).astype(np.float32)
    codes, err = orc.encode(cb, x, want_err=True)
    # (a) per codebook: nearest codeword within its own coordinates (product-quantization assignment)
    for k in range(K):
        sub = x.astype(np.float64)[:, groups[k]]
        cw = cb[k].astype(np.float64)[:, groups[k]]
        assert np.array_equal(codes[k], ((sub[:, None, :] - cw[None, :, :]) ** 2).sum(axis=2).argmin(axis=1))
    # (b) brute force over all m^K code combinations: nothing reconstructs x better
    best = np.full(N, np.inf)
    cb64 = cb.astype(np.float64)
    for j0 in range(m):
        for j1 in range(m):
            for j2 in range(m):
                rec = cb64[0, j0] + cb64[1, j1] + cb64[2, j2]
                best = np.minimum(best, ((x.astype(np.float64) - rec) ** 2).sum(axis=1))
    assert np.allclose(err, best, rtol=1e-12, atol=1e-15)
    # (c) the error it reports is ||x - reconstruction||^2
    rec = orc.reconstruct(cb, codes, np.arange(N))
    assert np.allclose(err, ((x.astype(np.float64) - rec) ** 2).sum(axis=1), rtol=1e-12, atol=1e-15)


def test_encode_returns_the_codes_of_a_reconstruction():
    g = _rng(33)
    K, m, d, N = 5, 256, 40, 300
    cb, _ = disjoint_support_codebooks(g, K, m, d)
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    x = orc.reconstruct(cb, codes, np.arange(N)).astype(np.float32)    # exact: supports are disjoint
    again, err = orc.encode(cb, x, want_err=True)
    assert np.array_equal(again, codes)
    assert (err == 0).all()


def _errors_numpy(cb, x, codes):
    rec = np.zeros((x.shape[0], x.shape[1]))
    for k in range(cb.shape[0]):
        rec += cb[k].astype(np.float64)[codes[k]]
    return ((x.astype(np.float64) - rec) ** 2).sum(axis=1)


def test_quantization_error_is_the_squared_distance_to_the_reconstruction():
    g = _rng(34)
    K, m, d, N = 4, 50, 13, 200
    cb = g.standard_normal((K, m, d)).astype(np.float32)
    x = g.standard_normal((N, d)).astype(np.float32)
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8)
    err = orc.quantization_error(cb, x, codes)
    assert np.allclose(err, _errors_numpy(cb, x, codes), rtol=1e-12, atol=1e-15)
    rec = orc.reconstruct(cb, codes, np.arange(N))
    assert np.allclose(err, ((x.astype(np.float64) - rec) ** 2).sum(axis=1), rtol=1e-12, atol=1e-15)
    # the greedy encoder's own error output is the same quantity
    codes_g, err_g = orc.encode(cb, x, want_err=True)
    assert np.allclose(orc.quantization_error(cb, x, codes_g), err_g, rtol=1e-10, atol=1e-13)


def test_icm_never_increases_the_error_and_ends_where_no_single_change_helps():
    g = _rng(35)
    K, m, d, N = 4, 16, 10, 120
    cb = (g.standard_normal((K, m, d)) * (0.8 ** np.arange(K))[:, None, None]).astype(np.float32)
    x = (g.standard_normal((N, d)) * 1.5).astype(np.float32)
    for start in (orc.encode(cb, x), g.integers(0, m, size=(K, N), dtype=np.uint8)):
        codes, prev = start.copy(), orc.quantization_error(cb, x, start)
        same0, ch0 = orc.encode_icm(cb, x, codes, 0)
        assert np.array_equal(same0, codes) and ch0.size == 0
        for sweep in range(30):
            nxt, changed = orc.encode_icm(cb, x, codes, 1)
            err = orc.quantization_error(cb, x, nxt)
            assert (err <= prev * (1 + 1e-12) + 1e-15).all()              # never worse, item by item
            assert changed[0] == (nxt != codes).sum()
            strictly = err < prev * (1 - 1e-12)
            assert ((nxt != codes).any(axis=0) <= strictly).all()       # a change always pays
            codes, prev = nxt, err
            if changed[0] == 0:
                break
        assert changed[0] == 0, "no fixed point after 30 sweeps"
        # several sweeps in one call = the same sweeps one by one
        multi, ch = orc.encode_icm(cb, x, start, sweep + 1)
        assert np.array_equal(multi, codes) and ch[-1] == 0
        # fixed point: brute force over every single sub-code change finds nothing strictly better
        cb64 = cb.astype(np.float64)
        for k in range(K):
            rest = x.astype(np.float64) - sum(cb64[l][codes[l]] for l in range(K) if l != k)
            d2 = ((rest[:, None, :] - cb64[k][None, :, :]) ** 2).sum(axis=2)
            assert (d2.min(axis=1) >= prev * (1 - 1e-12) - 1e-15).all()


def test_icm_against_brute_force_on_a_tiny_codebook_set():
    """m^K = 125 combinations: the optimum is a fixed point, and refinement started from the greedy
    codes ends between the optimum and the greedy error."""
    g = _rng(36)
    K, m, d, N = 3, 5, 4, 300
    cb = g.standard_normal((K, m, d)).astype(np.float32)
    x = g.standard_normal((N, d)).astype(np.float32)
    cb64, x64 = cb.astype(np.float64), x.astype(np.float64)
    best = np.full(N, np.inf)
    arg = np.zeros((K, N), dtype=np.uint8)
    for j0 in range(m):
        for j1 in range(m):
            for j2 in range(m):
                e = ((x64 - (cb64[0, j0] + cb64[1, j1] + cb64[2, j2])) ** 2).sum(axis=1)
                better = e < best
                best[better] = e[better]
                arg[:, better] = np.array([[j0], [j1], [j2]], dtype=np.uint8)
    stay, changed = orc.encode_icm(cb, x, arg, 2)
    assert np.array_equal(stay, arg) and (changed == 0).all()
    greedy, err_g = orc.encode(cb, x, want_err=True)
    refined, _ = orc.encode_icm(cb, x, greedy, 20)
    err_r = orc.quantization_error(cb, x, refined)
    assert (err_r >= best - 1e-12).all() and (err_r <= err_g + 1e-12).all()
    assert err_r.mean() < err_g.mean() and (err_r < err_g - 1e-9).sum() > N // 10    # and it does help
    assert (np.abs(err_r - best) < 1e-12).mean() > 0.5                                # often all the way


def test_icm_on_disjoint_supports_reaches_the_optimum_in_one_sweep_from_anywhere():
    g = _rng(37)
    K, m, d, N = 3, 4, 7, 60
    cb, groups = disjoint_support_codebooks(g, K, m, d)
    x = g.standard_normal((N, d)).astype(np.float32)
    optimum = orc.encode(cb, x)                    # pinned above as the brute-force optimum
    start = g.integers(0, m, size=(K, N), dtype=np.uint8)
    one, _ = orc.encode_icm(cb, x, start, 1)
    e1, e0 = orc.quantization_error(cb, x, one), orc.quantization_error(cb, x, optimum)
    assert np.allclose(e1, e0, rtol=1e-12, atol=1e-15)
    # with one codebook a sweep is the nearest codeword whatever the start
    cb1 = g.standard_normal((1, 30, 5)).astype(np.float32)
    x1 = g.standard_normal((80, 5)).astype(np.float32)
    c1, _ = orc.encode_icm(cb1, x1, g.integers(0, 30, size=(1, 80), dtype=np.uint8), 1)
    assert np.allclose(orc.quantization_error(cb1, x1, c1), orc.quantization_error(cb1, x1, orc.encode(cb1, x1)),
                       rtol=1e-12, atol=1e-15)


# ================================================================ quantities around the fast set
def test_online_variance_equals_the_variance_of_the_concatenated_batches():
    g = _rng(41)
    d, n, B = 11, 37, 9
    batches = [(g.standard_normal((n, d)) * g.uniform(0.2, 3.0, size=d) + g.uniform(-2, 2, size=d)).astype(np.float32)
               for _ in range(B)]
    mean, var = np.zeros(d), np.zeros(d)
    for b, x in enumerate(batches, start=1):
        bm, bv = orc.batch_moments(x)
        assert np.allclose(bm, x.astype(np.float64).mean(axis=0), rtol=1e-13, atol=1e-15)
        assert np.allclose(bv, x.astype(np.float64).var(axis=0), rtol=1e-12, atol=1e-15)
        mean, var = orc.online_variance(mean, var, bm, bv, b)
        allx = np.concatenate(batches[:b]).astype(np.float64)
        assert np.allclose(mean, allx.mean(axis=0), rtol=1e-12, atol=1e-13)
        assert np.allclose(var, allx.var(axis=0), rtol=1e-11, atol=1e-13)


def test_prior_densities_integrate_to_their_weights_and_the_skew_normal_mean_is_textbook():
    pi1, s1, pi2, mu2, s2, a2 = 0.8, 0.5, 0.2, 3.0, 1.2, -10.0
    grid = np.linspace(-12.0, 12.0, 240_001)
    xi, pm, pn = orc.subspace_mask(grid, pi1, s1, pi2, mu2, s2, a2, want_densities=True)
    h = grid[1] - grid[0]
    assert abs(pm.sum() * h - pi1) < 1e-9 and abs(pn.sum() * h - pi2) < 1e-9
    delta = a2 / np.sqrt(1.0 + a2 * a2)
    assert abs((grid * pn).sum() * h / pi2 - (mu2 + s2 * delta * np.sqrt(2.0 / np.pi))) < 1e-8
    assert np.array_equal(xi, (pn > pm).astype(np.uint8))
    # far left the major mode wins, around the minor mode's bulk the minor one does
    assert xi[np.searchsorted(grid, 0.0)] == 0 and xi[np.searchsorted(grid, 2.5)] == 1


def test_subspace_boundary_in_the_symmetric_special_case():
    """alpha2 = 0 makes the skew normal a normal; with equal weights and equal widths
    N(x; mu, s) > N(x; 0, s)  <=>  x > mu/2."""
    lam = np.array([0.0, 0.7, 0.99, 1.01, 1.5, 4.0])
    xi = orc.subspace_mask(lam, 0.5, 0.8, 0.5, 2.0, 0.8, 0.0)
    assert np.array_equal(xi, [0, 0, 0, 1, 1, 1])


def test_fast_set_and_margin_on_codebooks_built_inside_and_outside_psi():
    g = _rng(42)
    K, m, d = 5, 16, 12
    xi = np.zeros(d, dtype=np.uint8)
    xi[[1, 4, 5, 9]] = 1
    cb = np.zeros((K, m, d), dtype=np.float32)
    inside, outside = np.nonzero(xi)[0], np.nonzero(xi == 0)[0]
    cb[0][:, inside] = g.standard_normal((m, inside.size))           # fast: all norm inside psi
    cb[1][:, outside] = g.standard_normal((m, outside.size))         # slow
    cb[2][:, inside] = g.standard_normal((m, inside.size))           # fast but for ONE codeword
    cb[2][3] = 0.0
    cb[2][3, outside[0]] = 1.0
    cb[3] = g.standard_normal((m, d)).astype(np.float32)             # mostly outside: 8 of 12 dimensions
    cb[3][:, inside] *= 0.01
    cb[4][:, inside] = 3.0 * g.standard_normal((m, inside.size))     # mixed but dominated by psi
    cb[4][:, outside] = 0.01 * g.standard_normal((m, outside.size))
    assert np.array_equal(orc.fast_set(cb, xi), [1, 0, 0, 0, 1])
    lam = g.uniform(0.1, 2.0, size=d)
    assert orc.margin(lam, xi) == lam[outside[0]] + lam[outside[1:]].sum() or \
        abs(orc.margin(lam, xi) - lam[outside].sum()) < 1e-15
    assert orc.margin(lam, np.ones(d, dtype=np.uint8)) == 0.0
    assert abs(orc.margin(lam, np.zeros(d, dtype=np.uint8)) - lam.sum()) < 1e-15


def test_tiled_loop_analysis_without_a_band_is_the_oracles_tiled_loop():
    """The helper the GPU parity test judges rounding-sensitive decisions with follows the same loop."""
    from helpers import tiled_loop_analysis
    T, codes = _random_case(31, N=5000)
    Q, N, Kf, topk = T.shape[0], codes.shape[1], 2, 12
    sigma = np.linspace(0.0, 2.0, Q)
    bounds = np.array([0, 5, 40, 41, 700, 2500, N])
    ids, dist, refined = orc.running_search_tiled(T, codes, Kf, sigma, topk, bounds)
    P = orc.partial(T, codes, Kf)
    D = orc.adc_exhaustive(T, codes, topk, want_all=True)[2]
    for q in range(Q):
        got, lo, hi, clean = tiled_loop_analysis(P[q], D[q], sigma[q], topk, bounds, lambda x: 0.0)
        assert clean and lo == hi == refined[q]
        assert np.array_equal(got.astype(np.uint32), ids[q])
