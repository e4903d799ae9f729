"""The seeded input generators: reproducible, of the stated shapes, and with the structure the
recipes promise (checked through the CPU checker's encoder where codes are not drawn)."""
import numpy as np

from oracle import icq_oracle as orc
from paper_1912_08756_amd import synth


def test_workloads_are_reproducible_and_reduced_copies_share_the_codebooks():
    a, b = synth.make("C3", N=5000, Q=7), synth.make("C3", N=5000, Q=7)
    for key in ("codebooks", "codes", "queries", "query_sources"):
        assert np.array_equal(a[key], b[key])
    c = synth.make("C3", N=300, Q=2)
    assert np.array_equal(a["codebooks"], c["codebooks"])
    assert a["codes"].shape == (8, 5000) and a["codes"].dtype == np.uint8
    assert a["queries"].shape == (7, 96) and a["queries"].dtype == np.float32
    assert not np.array_equal(a["codebooks"], synth.make("C3", N=10, Q=1, seed=5)["codebooks"])


def test_clustered_codes_copy_their_centre_with_probability_nine_tenths():
    cfg = synth.make("C3", N=200_000, Q=1)
    pairs = cfg["codes"][0].astype(np.int64) * 256 + cfg["codes"][1]
    top = np.sort(np.bincount(pairs, minlength=65536))[::-1]
    # 1000 centres hold 0.81 of the items between them; the slow rows are uniform
    assert 0.78 <= top[:1000].sum() / 200_000 <= 0.84
    assert np.bincount(cfg["codes"][5], minlength=256).max() < 2 * 200_000 / 256


def test_mixture_vectors_are_reproducible_and_cluster_around_reconstructions():
    a, b = synth.make_vectors("C3", N=6000, Q=5), synth.make_vectors("C3", N=6000, Q=5)
    for key in ("codebooks", "x", "cluster", "queries", "query_sources"):
        assert np.array_equal(a[key], b[key])
    assert a["x"].shape == (6000, 96) and a["x"].dtype == np.float32 and "codes" not in a
    # blocks of rows are drawn independently: a longer array starts with the same rows, whatever the threads
    big = synth.make_vectors("C3", N=70_000, Q=1)
    x2, pick2 = synth.make_mixture_vectors(big["codebooks"], 70_000, 1000, 1.0, big["seed"], workers=1)
    assert np.array_equal(x2, big["x"]) and np.array_equal(pick2, big["cluster"])
    x3, _ = synth.make_mixture_vectors(big["codebooks"], 66_000, 1000, 1.0, big["seed"], workers=3)
    assert np.array_equal(x3, big["x"][:66_000])
    # within a cluster the scatter has the stated deviation
    for c in np.unique(a["cluster"])[:20]:
        rows = a["x"][a["cluster"] == c].astype(np.float64)
        if len(rows) >= 8:
            assert 0.8 <= rows.std(axis=0, ddof=1).mean() <= 1.2
    # queries are noisy copies of drawn vectors: much nearer their source than the cluster scatter
    gap = np.linalg.norm(a["queries"] - a["x"][a["query_sources"]], axis=1)
    assert (gap < 0.1 * np.linalg.norm(a["x"][a["query_sources"]], axis=1)).all()


def test_encoded_mixture_shares_the_first_sub_codes_within_a_cluster():
    cfg = synth.make_vectors("C3", N=3000, Q=1, n_centres=30)
    codes = orc.encode(cfg["codebooks"], cfg["x"])
    share = []
    for k in range(3):
        share.append(np.mean([(codes[k][cfg["cluster"] == c] == np.bincount(codes[k][cfg["cluster"] == c]).argmax()).mean()
                              for c in range(30)]))
    assert share[0] > 0.99 and 0.85 < share[1] < 0.99 and 0.15 < share[2] < 0.6
