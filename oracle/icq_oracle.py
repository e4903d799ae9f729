"""ctypes loader for the CPU oracle (oracle/icq_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
cpu_baseline leg may import this module.  It shares nothing with the GPU
library and never falls back to it.  Argument marshalling only; every number is
computed by the C file, whose functions cite the passages of arxiv 1912.08756
they follow.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "icq_oracle.c")
_LIB = os.path.join(_HERE, "libicq_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP over queries)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(
        ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
         "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def build_sanitize_check(sanitize, out_dir=None):
    """Compile oracle/sanitize_check.c -- the oracle plus a driver that calls every function on
    small awkward inputs and prints the results -- plainly or with the address and
    undefined-behaviour sanitizers (host code only).  Returns the executable's path."""
    out_dir = out_dir or _HERE
    exe = os.path.join(out_dir, "sanitize_check_san" if sanitize else "sanitize_check_plain")
    flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
             if sanitize else ["-O2"])
    subprocess.check_call(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra"] + flags +
                          ["-o", exe, os.path.join(_HERE, "sanitize_check.c"), "-lm"])
    return exe


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build(force=True)
        lib = ctypes.CDLL(_LIB)
        c_f = ctypes.POINTER(ctypes.c_float)
        c_d = ctypes.POINTER(ctypes.c_double)
        c_u8 = ctypes.POINTER(ctypes.c_uint8)
        c_u32 = ctypes.POINTER(ctypes.c_uint32)
        c_i64 = ctypes.POINTER(ctypes.c_int64)
        i, i64 = ctypes.c_int, ctypes.c_int64
        lib.icq_oracle_lut.argtypes = [c_f, i, i, i, c_f, i, c_d]
        lib.icq_oracle_partial.argtypes = [c_d, i, i, c_u8, i64, i, i, c_d]
        lib.icq_oracle_search.argtypes = [c_d, i, i, c_u8, i64, i, i, c_f, i, c_u32, c_d, c_i64, c_d, c_d]
        lib.icq_oracle_adc_exhaustive.argtypes = [c_d, i, i, c_u8, i64, i, i, c_u32, c_d, c_d]
        lib.icq_oracle_reconstruct.argtypes = [c_f, i, i, i, c_u8, i64, c_i64, i64, c_d]
        lib.icq_oracle_bruteforce_knn.argtypes = [c_f, i, i, i, c_u8, i64, c_f, i, i, c_u32, c_d]
        lib.icq_oracle_running_search.argtypes = [c_d, i, i, c_u8, i64, i, i, c_d, i, c_u32, c_d, c_i64]
        lib.icq_oracle_running_search_tiled.argtypes = [c_d, i, i, c_u8, i64, i, i, c_d, i, c_i64, i, c_u32, c_d, c_i64]
        lib.icq_oracle_sample_thresholds.argtypes = [c_d, i, i, c_u8, i64, i, i, c_d, i, i64, c_d]
        lib.icq_oracle_op_counts.argtypes = [i64, i, i, i, c_i64, ctypes.c_double, c_d, c_d]
        dbl = ctypes.c_double
        lib.icq_oracle_batch_moments.argtypes = [c_f, i64, i, c_d, c_d]
        lib.icq_oracle_online_variance.argtypes = [c_d, c_d, c_d, c_d, i, i64]
        lib.icq_oracle_subspace_mask.argtypes = [c_d, i, dbl, dbl, dbl, dbl, dbl, dbl, c_u8, c_d, c_d]
        lib.icq_oracle_fast_set.argtypes = [c_f, i, i, i, c_u8, c_u8]
        lib.icq_oracle_margin.argtypes = [c_d, c_u8, i]
        lib.icq_oracle_margin.restype = dbl
        lib.icq_oracle_encode.argtypes = [c_f, i, i, i, c_f, i64, c_u8, c_d]
        lib.icq_oracle_quantization_error.argtypes = [c_f, i, i, i, c_f, i64, c_u8, c_d]
        lib.icq_oracle_encode_icm.argtypes = [c_f, i, i, i, c_f, i64, c_u8, i, c_i64]
        lib.icq_oracle_threads.restype = i
        for name in ("lut", "partial", "search", "adc_exhaustive", "reconstruct", "bruteforce_knn",
                     "running_search", "running_search_tiled", "sample_thresholds", "op_counts", "encode", "quantization_error", "encode_icm",
                     "batch_moments", "online_variance", "subspace_mask", "fast_set"):
            getattr(lib, "icq_oracle_" + name).restype = None
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _chk(a, dtype, shape):
    a = np.ascontiguousarray(a, dtype=dtype)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


def threads():
    return int(_load().icq_oracle_threads())


def lut(codebooks, queries):
    """T[q][k][j] = ||q - c_{k,j}||^2 in double.  codebooks [K][m][d], queries [Q][d]."""
    K, m, d = codebooks.shape
    cb = _chk(codebooks, np.float32, (K, m, d))
    Q = queries.shape[0]
    qs = _chk(queries, np.float32, (Q, d))
    T = np.empty((Q, K, m), dtype=np.float64)
    _load().icq_oracle_lut(_p(cb, ctypes.c_float), K, m, d, _p(qs, ctypes.c_float), Q, _p(T, ctypes.c_double))
    return T


def partial(T, codes, Kf):
    """P[q][i] = crude distance over the first Kf codebooks.  codes [K][N] uint8."""
    Q, K, m = T.shape
    N = codes.shape[1]
    T = _chk(T, np.float64, (Q, K, m))
    cd = _chk(codes, np.uint8, (K, N))
    P = np.empty((Q, N), dtype=np.float64)
    _load().icq_oracle_partial(_p(T, ctypes.c_double), K, m, _p(cd, ctypes.c_uint8), N, Kf, Q, _p(P, ctypes.c_double))
    return P


def search(T, codes, Kf, thresholds, topk, want_all=False):
    """Two-step search.  Returns (ids [Q][topk] u32, dist [Q][topk] f64, count [Q] i64)
    and, with want_all, also (P [Q][N], D [Q][N] with NaN for pruned items)."""
    Q, K, m = T.shape
    N = codes.shape[1]
    T = _chk(T, np.float64, (Q, K, m))
    cd = _chk(codes, np.uint8, (K, N))
    th = _chk(thresholds, np.float32, (Q,))
    ids = np.empty((Q, topk), dtype=np.uint32)
    dist = np.empty((Q, topk), dtype=np.float64)
    cnt = np.empty((Q,), dtype=np.int64)
    P = np.empty((Q, N), dtype=np.float64) if want_all else None
    D = np.empty((Q, N), dtype=np.float64) if want_all else None
    _load().icq_oracle_search(_p(T, ctypes.c_double), K, m, _p(cd, ctypes.c_uint8), N, Kf, Q,
                              _p(th, ctypes.c_float), topk, _p(ids, ctypes.c_uint32),
                              _p(dist, ctypes.c_double), _p(cnt, ctypes.c_int64),
                              _p(P, ctypes.c_double), _p(D, ctypes.c_double))
    if want_all:
        return ids, dist, cnt, P, D
    return ids, dist, cnt


def adc_exhaustive(T, codes, topk, want_all=False):
    """One-step exhaustive ADC top-k (and every distance with want_all)."""
    Q, K, m = T.shape
    N = codes.shape[1]
    T = _chk(T, np.float64, (Q, K, m))
    cd = _chk(codes, np.uint8, (K, N))
    ids = np.empty((Q, topk), dtype=np.uint32)
    dist = np.empty((Q, topk), dtype=np.float64)
    D = np.empty((Q, N), dtype=np.float64) if want_all else None
    _load().icq_oracle_adc_exhaustive(_p(T, ctypes.c_double), K, m, _p(cd, ctypes.c_uint8), N, Q, topk,
                                      _p(ids, ctypes.c_uint32), _p(dist, ctypes.c_double), _p(D, ctypes.c_double))
    if want_all:
        return ids, dist, D
    return ids, dist


def running_search(T, codes, Kf, sigma, topk):
    """The paper's serial search loop with margin sigma [Q].  Returns (ids [Q][topk] u32,
    dist [Q][topk] f64, refined [Q] i64 = items that got the exact comparison)."""
    Q, K, m = T.shape
    N = codes.shape[1]
    T = _chk(T, np.float64, (Q, K, m))
    cd = _chk(codes, np.uint8, (K, N))
    sg = _chk(sigma, np.float64, (Q,))
    ids = np.empty((Q, topk), dtype=np.uint32)
    dist = np.empty((Q, topk), dtype=np.float64)
    refined = np.empty((Q,), dtype=np.int64)
    _load().icq_oracle_running_search(_p(T, ctypes.c_double), K, m, _p(cd, ctypes.c_uint8), N, Kf, Q,
                                      _p(sg, ctypes.c_double), topk, _p(ids, ctypes.c_uint32),
                                      _p(dist, ctypes.c_double), _p(refined, ctypes.c_int64))
    return ids, dist, refined


def running_search_tiled(T, codes, Kf, sigma, topk, bounds):
    """The serial loop with the crude comparison's right side refreshed per tile of items;
    bounds [R+1] ascending from 0 to N.  Returns as running_search."""
    Q, K, m = T.shape
    N = codes.shape[1]
    T = _chk(T, np.float64, (Q, K, m))
    cd = _chk(codes, np.uint8, (K, N))
    sg = _chk(sigma, np.float64, (Q,))
    bd = np.ascontiguousarray(bounds, dtype=np.int64)
    if bd.ndim != 1 or bd.size < 2 or bd[0] != 0 or bd[-1] != N or (np.diff(bd) < 0).any():
        raise ValueError("bounds must ascend from 0 to N")
    ids = np.empty((Q, topk), dtype=np.uint32)
    dist = np.empty((Q, topk), dtype=np.float64)
    refined = np.empty((Q,), dtype=np.int64)
    _load().icq_oracle_running_search_tiled(_p(T, ctypes.c_double), K, m, _p(cd, ctypes.c_uint8), N, Kf, Q,
                                            _p(sg, ctypes.c_double), topk, _p(bd, ctypes.c_int64), bd.size - 1,
                                            _p(ids, ctypes.c_uint32), _p(dist, ctypes.c_double),
                                            _p(refined, ctypes.c_int64))
    return ids, dist, refined


def sample_thresholds(T, codes, Kf, sigma, topk, M):
    """t_q = P(topk-th nearest of the first M items) + sigma_q, double [Q]."""
    Q, K, m = T.shape
    N = codes.shape[1]
    T = _chk(T, np.float64, (Q, K, m))
    cd = _chk(codes, np.uint8, (K, N))
    sg = _chk(sigma, np.float64, (Q,))
    thr = np.empty((Q,), dtype=np.float64)
    _load().icq_oracle_sample_thresholds(_p(T, ctypes.c_double), K, m, _p(cd, ctypes.c_uint8), N, Kf, Q,
                                         _p(sg, ctypes.c_double), topk, M, _p(thr, ctypes.c_double))
    return thr


def op_counts(N, K, Kf, refined, code_bits):
    """(ops_icq [Q] f64, summary [4] f64 = mean ops_icq, ops_adc, ratio, effective code length)."""
    rf = np.ascontiguousarray(refined, dtype=np.int64)
    Q = rf.shape[0]
    ops = np.empty((Q,), dtype=np.float64)
    summary = np.empty((4,), dtype=np.float64)
    _load().icq_oracle_op_counts(N, K, Kf, Q, _p(rf, ctypes.c_int64), float(code_bits),
                                 _p(ops, ctypes.c_double), _p(summary, ctypes.c_double))
    return ops, summary


def encode(codebooks, x, want_err=False):
    """Greedy residual encoding in codebook order.  x [N][d] -> codes [K][N] u8 (and ||x - xbar||^2 [N])."""
    K, m, d = codebooks.shape
    cb = _chk(codebooks, np.float32, (K, m, d))
    N = x.shape[0]
    xs = _chk(x, np.float32, (N, d))
    codes = np.empty((K, N), dtype=np.uint8)
    err = np.empty((N,), dtype=np.float64) if want_err else None
    _load().icq_oracle_encode(_p(cb, ctypes.c_float), K, m, d, _p(xs, ctypes.c_float), N,
                              _p(codes, ctypes.c_uint8), _p(err, ctypes.c_double))
    return (codes, err) if want_err else codes


def quantization_error(codebooks, x, codes):
    """||x_i - xbar_i||^2 [N] f64 of codes [K][N]."""
    K, m, d = codebooks.shape
    cb = _chk(codebooks, np.float32, (K, m, d))
    N = x.shape[0]
    xs = _chk(x, np.float32, (N, d))
    cd = _chk(codes, np.uint8, (K, N))
    err = np.empty((N,), dtype=np.float64)
    _load().icq_oracle_quantization_error(_p(cb, ctypes.c_float), K, m, d, _p(xs, ctypes.c_float), N,
                                          _p(cd, ctypes.c_uint8), _p(err, ctypes.c_double))
    return err


def encode_icm(codebooks, x, codes, sweeps):
    """Coordinate descent over the codebooks from the given codes [K][N]; returns (codes, changed [sweeps])."""
    K, m, d = codebooks.shape
    cb = _chk(codebooks, np.float32, (K, m, d))
    N = x.shape[0]
    xs = _chk(x, np.float32, (N, d))
    cd = _chk(codes, np.uint8, (K, N)).copy()
    changed = np.zeros((max(sweeps, 0),), dtype=np.int64)
    _load().icq_oracle_encode_icm(_p(cb, ctypes.c_float), K, m, d, _p(xs, ctypes.c_float), N,
                                  _p(cd, ctypes.c_uint8), sweeps, _p(changed, ctypes.c_int64))
    return cd, changed


def batch_moments(x):
    """Population mean and variance per dimension of x [n][d] -> (mean [d], var [d]) f64."""
    n, d = x.shape
    xs = _chk(x, np.float32, (n, d))
    mean, var = np.empty(d), np.empty(d)
    _load().icq_oracle_batch_moments(_p(xs, ctypes.c_float), n, d, _p(mean, ctypes.c_double), _p(var, ctypes.c_double))
    return mean, var


def online_variance(mean, var, batch_mean, batch_var, b):
    """One step of the online variance estimate (batch number b, 1-based); returns new (mean, var)."""
    d = mean.shape[0]
    mean, var = _chk(mean, np.float64, (d,)).copy(), _chk(var, np.float64, (d,)).copy()
    bm, bv = _chk(batch_mean, np.float64, (d,)), _chk(batch_var, np.float64, (d,))
    _load().icq_oracle_online_variance(_p(mean, ctypes.c_double), _p(var, ctypes.c_double), _p(bm, ctypes.c_double),
                                       _p(bv, ctypes.c_double), d, b)
    return mean, var


def subspace_mask(lam, pi1, sigma1, pi2, mu2, sigma2, alpha2, want_densities=False):
    """xi [d] u8: 1 where the minor (skew-normal) mode wins; optionally the two weighted densities."""
    d = lam.shape[0]
    lm = _chk(lam, np.float64, (d,))
    xi = np.empty(d, dtype=np.uint8)
    pm = np.empty(d) if want_densities else None
    pn = np.empty(d) if want_densities else None
    _load().icq_oracle_subspace_mask(_p(lm, ctypes.c_double), d, pi1, sigma1, pi2, mu2, sigma2, alpha2,
                                     _p(xi, ctypes.c_uint8), _p(pm, ctypes.c_double), _p(pn, ctypes.c_double))
    return (xi, pm, pn) if want_densities else xi


def fast_set(codebooks, xi):
    K, m, d = codebooks.shape
    cb = _chk(codebooks, np.float32, (K, m, d))
    x = _chk(xi, np.uint8, (d,))
    fast = np.empty(K, dtype=np.uint8)
    _load().icq_oracle_fast_set(_p(cb, ctypes.c_float), K, m, d, _p(x, ctypes.c_uint8), _p(fast, ctypes.c_uint8))
    return fast


def margin(lam, xi):
    d = lam.shape[0]
    return float(_load().icq_oracle_margin(_p(_chk(lam, np.float64, (d,)), ctypes.c_double),
                                           _p(_chk(xi, np.uint8, (d,)), ctypes.c_uint8), d))


def reconstruct(codebooks, codes, items):
    """xbar_i = sum_k c_{k,code_k(i)} for i in items, double [len(items)][d]."""
    K, m, d = codebooks.shape
    N = codes.shape[1]
    cb = _chk(codebooks, np.float32, (K, m, d))
    cd = _chk(codes, np.uint8, (K, N))
    it = np.ascontiguousarray(items, dtype=np.int64)
    x = np.empty((it.shape[0], d), dtype=np.float64)
    _load().icq_oracle_reconstruct(_p(cb, ctypes.c_float), K, m, d, _p(cd, ctypes.c_uint8), N,
                                   _p(it, ctypes.c_int64), it.shape[0], _p(x, ctypes.c_double))
    return x


def bruteforce_knn(codebooks, codes, queries, topk):
    """Exact k-NN of each query among the reconstructions, by brute force."""
    K, m, d = codebooks.shape
    N = codes.shape[1]
    Q = queries.shape[0]
    cb = _chk(codebooks, np.float32, (K, m, d))
    cd = _chk(codes, np.uint8, (K, N))
    qs = _chk(queries, np.float32, (Q, d))
    ids = np.empty((Q, topk), dtype=np.uint32)
    dist = np.empty((Q, topk), dtype=np.float64)
    _load().icq_oracle_bruteforce_knn(_p(cb, ctypes.c_float), K, m, d, _p(cd, ctypes.c_uint8), N,
                                      _p(qs, ctypes.c_float), Q, topk, _p(ids, ctypes.c_uint32),
                                      _p(dist, ctypes.c_double))
    return ids, dist
