"""Seeded synthetic inputs for the ICQ query-time path.

This module only *draws data*: codebooks, one-byte sub-codes and query vectors
with the shapes of the workloads the search is measured on.  It holds none of
the search arithmetic (no lookup tables, no partial or full distances, no
thresholds), so the GPU path's tests and the CPU checker can both be fed from
it without sharing any of the method's code.

Recipe (all draws from numpy's counter-based Philox generator, keyed by
(seed, stream) so every array is reproducible on its own):

* codebooks   c_{k,j} ~ N(0, sigma_k^2 I_d), k = 0..K-1, j = 0..m-1, float32.
* codes       [K][N] uint8, codebook-major; "uniform": every sub-code uniform
              in 0..m-1; "clustered": 1000 centre codes drawn uniformly, each
              item picks a centre uniformly and copies the centre's fast
              sub-codes (k < Kf) with probability 0.9 (else uniform); slow
              sub-codes uniform.  This gives a skewed fast-code histogram,
              bursty survivors and many exact ties in the crude distance.
* queries     Q items drawn uniformly with replacement; query = the item's
              reconstruction sum_k c_{k,code_k} plus Gaussian noise: for the
              tiny config N(0, 0.01^2) + N(0, 0.05^2) per component, otherwise
              per-component std 0.05 * rms(||xbar||) / sqrt(d) (noise norm is
              about 5 % of a typical data norm).

Database vectors themselves are never materialised (the path consumes codes
only); reconstructions are formed for the Q query sources alone.

A second recipe draws database VECTORS instead of codes (`make_vectors`), for
indexes whose codes come from the encoder rather than from a generator:

* vectors     1000 centres, each the reconstruction of a uniformly drawn code;
              x_i = centre of a uniformly drawn cluster + N(0, spread^2 I_d),
              float32, spread = 1 (the per-component deviation of the first
              codebook: with sigma_k = 2^-k the nearest first codeword is then
              the centre's for practically every vector of a cluster, the
              second for about 94 %, the third for about 30 %).
* queries     Q vectors drawn uniformly with replacement plus per-component
              noise of std 0.05 * rms(||x||) / sqrt(d).
"""
import numpy as np

BASE_SEED = 191208756

# name -> shape of the workload.  sigma: ("list", [...]) or ("geom", ratio).
CONFIGS = {
    "C0": dict(d=32, K=4, Kf=1, m=256, N=10_000, Q=100, topk=10,
               sigma=("list", [1.0, 0.5, 0.25, 0.125]), codes="uniform", noise="tiny", batch=100),
    "C1": dict(d=128, K=8, Kf=2, m=256, N=1_000_000, Q=10_000, topk=100,
               sigma=("geom", 0.5), codes="uniform", noise="rel", batch=10_000),
    "C2": dict(d=960, K=16, Kf=4, m=256, N=1_000_000, Q=1_000, topk=100,
               sigma=("geom", 0.8), codes="uniform", noise="rel", batch=1_000),
    "C3": dict(d=96, K=8, Kf=2, m=256, N=10_000_000, Q=10_000, topk=100,
               sigma=("geom", 0.5), codes="clustered", noise="rel", batch=256),
    "C4": dict(d=96, K=16, Kf=4, m=256, N=100_000_000, Q=1_000, topk=100,
               sigma=("geom", 0.8), codes="uniform", noise="rel", batch=128),
}
_STREAM_CODEBOOKS, _STREAM_CODES, _STREAM_QUERIES, _STREAM_CENTRES, _STREAM_VECTORS = 1, 2, 3, 4, 5


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def sigmas(spec, K):
    kind, val = spec
    if kind == "list":
        assert len(val) == K
        return np.asarray(val, dtype=np.float64)
    return float(val) ** np.arange(K, dtype=np.float64)


def make_codebooks(K, m, d, sigma, seed):
    g = _rng(seed, _STREAM_CODEBOOKS)
    cb = g.standard_normal((K, m, d), dtype=np.float32)
    cb *= sigma.astype(np.float32)[:, None, None]
    return cb


def make_codes(K, Kf, m, N, kind, seed):
    g = _rng(seed, _STREAM_CODES)
    codes = g.integers(0, m, size=(K, N), dtype=np.uint8 if m <= 256 else np.uint16)
    if kind == "clustered":
        gc = _rng(seed, _STREAM_CENTRES)
        n_centres = 1000
        centres = gc.integers(0, m, size=(Kf, n_centres), dtype=np.uint8)
        pick = gc.integers(0, n_centres, size=N)
        for k in range(Kf):
            keep = gc.random(N) < 0.9
            codes[k] = np.where(keep, centres[k][pick], codes[k])
    return np.ascontiguousarray(codes, dtype=np.uint8)


def make_queries(codebooks, codes, Q, noise, seed):
    K, m, d = codebooks.shape
    N = codes.shape[1]
    g = _rng(seed, _STREAM_QUERIES)
    src = g.integers(0, N, size=Q)
    xbar = np.zeros((Q, d), dtype=np.float64)
    for k in range(K):
        xbar += codebooks[k][codes[k, src]].astype(np.float64)
    if noise == "tiny":
        x = xbar + 0.01 * g.standard_normal((Q, d))
        q = x + 0.05 * g.standard_normal((Q, d))
    else:
        rms = np.sqrt(np.mean(np.sum(xbar * xbar, axis=1))) if Q > 0 else 0.0
        q = xbar + (0.05 * rms / np.sqrt(d)) * g.standard_normal((Q, d))
    return np.ascontiguousarray(q, dtype=np.float32), src


def make(name, N=None, Q=None, seed=None, **override):
    """Draw one workload.  N / Q / any CONFIGS key may be overridden to get a
    reduced copy of the same recipe.  Returns a dict with codebooks [K][m][d]
    f32, codes [K][N] u8, queries [Q][d] f32 and the shape parameters."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    if N is not None:
        cfg["N"] = int(N)
    if Q is not None:
        cfg["Q"] = int(Q)
    if seed is None:
        seed = BASE_SEED + sorted(CONFIGS).index(name)
    K, Kf, m, d = cfg["K"], cfg["Kf"], cfg["m"], cfg["d"]
    sig = sigmas(cfg["sigma"], K)
    cb = make_codebooks(K, m, d, sig, seed)
    codes = make_codes(K, Kf, m, cfg["N"], cfg["codes"], seed)
    queries, src = make_queries(cb, codes, cfg["Q"], cfg["noise"], seed)
    cfg.update(name=name, seed=seed, codebooks=cb, codes=codes, queries=queries, query_sources=src)
    return cfg


_VECTOR_CHUNK = 1 << 16        # rows per independently keyed block of the vector stream (part of the recipe)


def make_mixture_vectors(codebooks, N, n_centres, spread, seed, workers=None):
    """[N][d] float32 vectors of a Gaussian mixture whose centres are reconstructions of
    uniformly drawn codes; returns (x, cluster index of every vector).  Rows come in blocks of
    65536, block j from the Philox stream (seed, vector stream) at counter word 3 = j, so blocks
    are independent of each other and of N and can be drawn by several threads."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    K, m, d = codebooks.shape
    gc = _rng(seed, _STREAM_CENTRES)
    centre_codes = gc.integers(0, m, size=(K, n_centres))
    centres = np.zeros((n_centres, d), dtype=np.float32)
    for k in range(K):
        centres += codebooks[k][centre_codes[k]]
    pick = gc.integers(0, n_centres, size=N)
    x = np.empty((N, d), dtype=np.float32)

    def block(j):
        lo, hi = j * _VECTOR_CHUNK, min(N, (j + 1) * _VECTOR_CHUNK)
        g = np.random.Generator(np.random.Philox(key=[int(seed), _STREAM_VECTORS], counter=[0, 0, 0, j]))
        part = x[lo:hi]
        g.standard_normal(out=part, dtype=np.float32)
        part *= np.float32(spread)
        part += centres[pick[lo:hi]]

    blocks = range((N + _VECTOR_CHUNK - 1) // _VECTOR_CHUNK)
    workers = workers or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(block, blocks))
    return x, pick


def make_vectors(name, N=None, Q=None, seed=None, n_centres=1000, spread=1.0):
    """A workload's shape with database vectors in place of codes: codebooks [K][m][d],
    x [N][d] f32 (Gaussian mixture), queries [Q][d] f32 (noisy copies of drawn vectors)."""
    cfg = dict(CONFIGS[name])
    if N is not None:
        cfg["N"] = int(N)
    if Q is not None:
        cfg["Q"] = int(Q)
    if seed is None:
        seed = BASE_SEED + 100 + sorted(CONFIGS).index(name)
    del cfg["codes"]                      # the generator kind of `make`: here the codes come from an encoder
    K, m, d = cfg["K"], cfg["m"], cfg["d"]
    cb = make_codebooks(K, m, d, sigmas(cfg["sigma"], K), seed)
    x, pick = make_mixture_vectors(cb, cfg["N"], n_centres, spread, seed)
    g = _rng(seed, _STREAM_QUERIES)
    src = g.integers(0, cfg["N"], size=cfg["Q"])
    xs = x[src].astype(np.float64)
    rms = np.sqrt(np.mean(np.sum(xs * xs, axis=1))) if cfg["Q"] > 0 else 0.0
    q = xs + (0.05 * rms / np.sqrt(d)) * g.standard_normal((cfg["Q"], d))
    cfg.update(name=name, seed=seed, codebooks=cb, x=x, cluster=pick, n_centres=n_centres, spread=spread,
               queries=np.ascontiguousarray(q, dtype=np.float32), query_sources=src)
    return cfg
