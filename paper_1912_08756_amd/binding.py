"""ctypes binding of libicq.so: the functions of include/icq.h under the same names.

Argument marshalling only.  Tensors are torch CUDA (ROCm) tensors used as plain
device memory; work is enqueued on torch's current stream.  Every step of the
search runs in the library's kernels: there is no CPU or PyTorch fallback, and a
missing library is an error.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libicq.so")

ICQ_OK, ICQ_ERR_ARG, ICQ_ERR_WORKSPACE, ICQ_ERR_HIP, ICQ_ERR_CAPACITY, ICQ_ERR_SCRATCH = 0, -1, -2, -3, -4, -5
ICQ_STATIC_SCRATCH_BYTES = 32 << 20
ICQ_PAD_ID = 0xFFFFFFFF
ICQ_LUT_W = 256

# name -> (restype, argtypes); mirrors include/icq.h one to one
_vp, _i, _i64, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
SIGNATURES = {
    "icq_strerror": (ctypes.c_char_p, [_i]),
    "icq_index_create": (_i, [ctypes.POINTER(_vp), _vp, _vp, _i, _i, _i, _i, _i64, _vp]),
    "icq_index_destroy": (None, [_vp]),
    "icq_index_export_codes": (_i, [_vp, _i, _vp, _vp]),
    "icq_index_set_scan_mode": (_i, [_vp, _i]),
    "icq_index_scan_positions": (_i, [_vp, _i, ctypes.POINTER(_i64)]),
    "icq_index_set_stage_timing": (_i, [_vp, _i]),
    "icq_index_stage_times": (_i, [_vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(_i), ctypes.POINTER(_i)]),
    "icq_workspace_bytes": (_i, [_vp, _i, _i64, _i, ctypes.POINTER(_sz)]),
    "icq_build_lut": (_i, [_vp, _vp, _i, _vp, _vp]),
    "icq_scan_fast": (_i, [_vp, _vp, _i, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "icq_refine": (_i, [_vp, _vp, _i, _vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _sz, _vp]),
    "icq_search": (_i, [_vp, _vp, _i, _vp, _i64, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "icq_search_static": (_i, [_vp, _vp, _i, _vp, _i64, _i, _vp, _vp, _vp, _vp]),
    "icq_running_workspace_bytes": (_i, [ctypes.POINTER(_vp), _i, _i, _i64, _i, ctypes.POINTER(_sz)]),
    "icq_search_running": (_i, [ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_uint32), _i, _vp, _i, _vp, _i64, _i, _vp, _vp,
                                _vp, _vp, _sz, _vp]),
    "icq_sample_thresholds": (_i, [_vp, _vp, _i, _vp, _i, _i64, _vp, _vp]),
    "icq_op_counts": (_i, [_vp, _vp, _i, _vp, _vp, _vp]),
    "icq_encode_workspace_bytes": (_i, [_vp, _i64, ctypes.POINTER(_sz)]),
    "icq_encode": (_i, [_vp, _vp, _i64, _vp, _vp, _sz, _vp]),
    "icq_encode_refine": (_i, [_vp, _vp, _i64, _vp, _i, _vp, _vp, _sz, _vp]),
    "icq_quantization_error": (_i, [_vp, _vp, _i64, _vp, _vp, _vp]),
    "icq_batch_moments": (_i, [_vp, _i64, _i, _vp, _vp, _vp]),
    "icq_online_variance_update": (_i, [_vp, _vp, _vp, _vp, _i, _i64, _vp]),
    "icq_subspace_mask": (_i, [_vp, _i] + [ctypes.c_double] * 6 + [_vp, _vp]),
    "icq_fast_set": (_i, [_vp, _vp, _vp, _vp]),
    "icq_margin": (_i, [_vp, _vp, _i, _vp, _vp]),
    "icq_machine_probe": (_i, [_i, _vp, _sz, _i, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), _vp]),
}
_lib = None


class IcqError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


def load():
    """Load libicq.so; raise if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "HIP library %s is missing: build it with `python -m paper_1912_08756_amd.build`"
                % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def strerror(code):
    return load().icq_strerror(int(code)).decode()


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, shape=None, name="tensor"):
    if t is None:
        return ctypes.c_void_p(0)
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return ctypes.c_void_p(t.data_ptr())


def _check(rc, where):
    if rc != ICQ_OK:
        raise IcqError(rc, where)


class Index:
    """Owner of an icq_index handle (destroyed with the object)."""

    def __init__(self, handle, K, m, d, Kf, N):
        self.handle, self.K, self.m, self.d, self.Kf, self.N = handle, K, m, d, Kf, N

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.icq_index_destroy(h)


def icq_index_create(codebooks, codes, Kf):
    """codebooks [K][m][d] f32, codes [K][N] u8 (device tensors) -> Index."""
    K, m, d = codebooks.shape
    N = codes.shape[1]
    h = ctypes.c_void_p(0)
    rc = load().icq_index_create(ctypes.byref(h), _dev(codebooks, torch.float32, name="codebooks"),
                                 _dev(codes, torch.uint8, (K, N), "codes"), K, m, d, Kf, N, _stream())
    _check(rc, "icq_index_create")
    return Index(h, K, m, d, Kf, N)


def icq_index_destroy(index):
    h, index.handle = index.handle, None
    if h:
        load().icq_index_destroy(h)


def icq_index_export_codes(index, from_items, codes_out):
    _check(load().icq_index_export_codes(index.handle, int(from_items),
                                         _dev(codes_out, torch.uint8, (index.K, index.N)),
                                         _stream()), "icq_index_export_codes")
    return codes_out


ICQ_SCAN_AUTO, ICQ_SCAN_STREAMED, ICQ_SCAN_GROUPED = 0, 1, 2


def icq_index_set_scan_mode(index, mode):
    _check(load().icq_index_set_scan_mode(index.handle, int(mode)), "icq_index_set_scan_mode")


def icq_index_scan_positions(index, Q):
    out = _i64(0)
    _check(load().icq_index_scan_positions(index.handle, int(Q), ctypes.byref(out)), "icq_index_scan_positions")
    return int(out.value)


def icq_index_set_stage_timing(index, enable):
    _check(load().icq_index_set_stage_timing(index.handle, int(bool(enable))), "icq_index_set_stage_timing")


def icq_index_stage_times(index):
    """((ms of table build, stage 1, stage 2 + list) averaged over the recorded icq_search calls,
    number of calls, most sub-batches in one of them); resets the record."""
    ms = (ctypes.c_float * 3)()
    calls, batches = _i(0), _i(0)
    _check(load().icq_index_stage_times(index.handle, ms, ctypes.byref(calls), ctypes.byref(batches)),
           "icq_index_stage_times")
    return [float(x) for x in ms], int(calls.value), int(batches.value)


def icq_workspace_bytes(index, Q, cap, topk):
    out = ctypes.c_size_t(0)
    _check(load().icq_workspace_bytes(index.handle, Q, cap, topk, ctypes.byref(out)), "icq_workspace_bytes")
    return int(out.value)


def icq_build_lut(index, queries, lut):
    Q = queries.shape[0]
    _check(load().icq_build_lut(index.handle, _dev(queries, torch.float32, (Q, index.d), "queries"), Q,
                                _dev(lut, torch.float32, (Q, index.K, ICQ_LUT_W), "lut"), _stream()),
           "icq_build_lut")
    return lut


def icq_scan_fast(index, lut, thresholds, cand_ids, cand_partial, cand_count, workspace):
    Q, cap = cand_ids.shape     # cand_partial may be None
    _check(load().icq_scan_fast(index.handle, _dev(lut, torch.float32, (Q, index.K, ICQ_LUT_W), "lut"), Q,
                                _dev(thresholds, torch.float32, (Q,), "thresholds"),
                                _dev(cand_ids, torch.int32, (Q, cap), "cand_ids"),
                                _dev(cand_partial, torch.float32, (Q, cap), "cand_partial"),
                                _dev(cand_count, torch.int32, (Q,), "cand_count"), cap,
                                _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()),
           "icq_scan_fast")


def icq_refine(index, lut, cand_ids, cand_partial, cand_count, topk, out_ids, out_dist, workspace):
    Q, cap = cand_ids.shape
    _check(load().icq_refine(index.handle, _dev(lut, torch.float32, (Q, index.K, ICQ_LUT_W), "lut"), Q,
                             _dev(cand_ids, torch.int32, (Q, cap), "cand_ids"),
                             _dev(cand_partial, torch.float32, (Q, cap), "cand_partial"),
                             _dev(cand_count, torch.int32, (Q,), "cand_count"), cap, topk,
                             _dev(out_ids, torch.int32, (Q, topk), "out_ids"),
                             _dev(out_dist, torch.float32, (Q, topk), "out_dist"),
                             _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()),
           "icq_refine")


def icq_search(index, queries, thresholds, cap, topk, out_ids, out_dist, out_survivors, workspace):
    Q = queries.shape[0]
    _check(load().icq_search(index.handle, _dev(queries, torch.float32, (Q, index.d), "queries"), Q,
                             _dev(thresholds, torch.float32, (Q,), "thresholds"), cap, topk,
                             _dev(out_ids, torch.int32, (Q, topk), "out_ids"),
                             _dev(out_dist, torch.float32, (Q, topk), "out_dist"),
                             _dev(out_survivors, torch.int32, (Q,), "out_survivors"),
                             _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()),
           "icq_search")


def icq_search_static(index, queries, thresholds, cap, topk, out_ids, out_dist, out_survivors):
    """icq_search on the library's built-in scratch array (no workspace, no allocation)."""
    Q = queries.shape[0]
    _check(load().icq_search_static(index.handle, _dev(queries, torch.float32, (Q, index.d), "queries"), Q,
                                    _dev(thresholds, torch.float32, (Q,), "thresholds"), cap, topk,
                                    _dev(out_ids, torch.int32, (Q, topk), "out_ids"),
                                    _dev(out_dist, torch.float32, (Q, topk), "out_dist"),
                                    _dev(out_survivors, torch.int32, (Q,), "out_survivors"), _stream()),
           "icq_search_static")


def _tile_handles(tiles):
    return (_vp * len(tiles))(*[t.handle for t in tiles])


def icq_running_workspace_bytes(tiles, Q, cap, topk):
    out = ctypes.c_size_t(0)
    _check(load().icq_running_workspace_bytes(_tile_handles(tiles), len(tiles), Q, cap, topk, ctypes.byref(out)),
           "icq_running_workspace_bytes")
    return int(out.value)


def icq_search_running(tiles, id_base, queries, sigma, cap, topk, out_ids, out_dist, out_refined, workspace):
    """tiles: indexes over consecutive id ranges (same codebooks); id_base: first item id of each (host ints);
    sigma: [Q] f32 device tensor or None."""
    Q = queries.shape[0]
    bases = (ctypes.c_uint32 * len(tiles))(*[int(x) for x in id_base])
    _check(load().icq_search_running(
        _tile_handles(tiles), bases, len(tiles), _dev(queries, torch.float32, (Q, tiles[0].d), "queries"), Q,
        _dev(sigma, torch.float32, (Q,), "sigma") if sigma is not None else None, cap, topk,
        _dev(out_ids, torch.int32, (Q, topk), "out_ids"), _dev(out_dist, torch.float32, (Q, topk), "out_dist"),
        _dev(out_refined, torch.int32, (Q,), "out_refined"),
        _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()), "icq_search_running")


def icq_sample_thresholds(index, lut, sigma, topk, M, thresholds_out):
    """sigma: [Q] f32 device tensor or None (zero margin)."""
    Q = lut.shape[0]
    _check(load().icq_sample_thresholds(
        index.handle, _dev(lut, torch.float32, (Q, index.K, ICQ_LUT_W), "lut"), Q,
        _dev(sigma, torch.float32, (Q,), "sigma") if sigma is not None else None, topk, M,
        _dev(thresholds_out, torch.float32, (Q,), "thresholds_out"), _stream()), "icq_sample_thresholds")


def icq_op_counts(index, refined, ops_out, summary_out):
    """refined [Q] int32 (survivor counts), ops_out [Q] int64, summary_out [4] float64 (device)."""
    Q = refined.shape[0]
    _check(load().icq_op_counts(index.handle, _dev(refined, torch.int32, (Q,), "refined"), Q,
                                _dev(ops_out, torch.int64, (Q,), "ops_out"),
                                _dev(summary_out, torch.float64, (4,), "summary_out"), _stream()), "icq_op_counts")


def icq_encode_workspace_bytes(index, N):
    out = ctypes.c_size_t(0)
    _check(load().icq_encode_workspace_bytes(index.handle, N, ctypes.byref(out)), "icq_encode_workspace_bytes")
    return int(out.value)


def icq_encode(index, x, codes_out, workspace):
    """x [N][d] f32, codes_out [K][N] u8 (device tensors)."""
    N = x.shape[0]
    _check(load().icq_encode(index.handle, _dev(x, torch.float32, (N, index.d), "x"), N,
                             _dev(codes_out, torch.uint8, (index.K, N), "codes_out"),
                             _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()),
           "icq_encode")


def icq_encode_refine(index, x, codes, sweeps, changed_out, workspace):
    """codes [K][N] u8 in/out; changed_out: [sweeps] int32 device tensor or None."""
    N = x.shape[0]
    _check(load().icq_encode_refine(index.handle, _dev(x, torch.float32, (N, index.d), "x"), N,
                                    _dev(codes, torch.uint8, (index.K, N), "codes"), int(sweeps),
                                    _dev(changed_out, torch.int32, (sweeps,), "changed_out") if changed_out is not None else None,
                                    _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()),
           "icq_encode_refine")


def icq_quantization_error(index, x, codes, err_out):
    """err_out [N] float64 (device) = ||x - reconstruction||^2 of codes [K][N]."""
    N = x.shape[0]
    _check(load().icq_quantization_error(index.handle, _dev(x, torch.float32, (N, index.d), "x"), N,
                                         _dev(codes, torch.uint8, (index.K, N), "codes"),
                                         _dev(err_out, torch.float64, (N,), "err_out"), _stream()),
           "icq_quantization_error")


def icq_batch_moments(x, mean_out, var_out):
    n, d = x.shape
    _check(load().icq_batch_moments(_dev(x, torch.float32, name="x"), n, d, _dev(mean_out, torch.float64, (d,)),
                                    _dev(var_out, torch.float64, (d,)), _stream()), "icq_batch_moments")


def icq_online_variance_update(mean, var, batch_mean, batch_var, b):
    d = mean.shape[0]
    _check(load().icq_online_variance_update(_dev(mean, torch.float64, (d,)), _dev(var, torch.float64, (d,)),
                                             _dev(batch_mean, torch.float64, (d,)), _dev(batch_var, torch.float64, (d,)),
                                             d, b, _stream()), "icq_online_variance_update")


def icq_subspace_mask(lam, pi1, sigma1, pi2, mu2, sigma2, alpha2, xi_out):
    d = lam.shape[0]
    _check(load().icq_subspace_mask(_dev(lam, torch.float64, (d,)), d, pi1, sigma1, pi2, mu2, sigma2, alpha2,
                                    _dev(xi_out, torch.uint8, (d,)), _stream()), "icq_subspace_mask")


def icq_fast_set(index, xi, fast_out):
    _check(load().icq_fast_set(index.handle, _dev(xi, torch.uint8, (index.d,)), _dev(fast_out, torch.uint8, (index.K,)),
                               _stream()), "icq_fast_set")


def icq_margin(lam, xi, sigma_out):
    d = lam.shape[0]
    _check(load().icq_margin(_dev(lam, torch.float64, (d,)), _dev(xi, torch.uint8, (d,)), d,
                             _dev(sigma_out, torch.float64, (1,)), _stream()), "icq_margin")


ICQ_PROBE_READ, ICQ_PROBE_READ_NT, ICQ_PROBE_LDS_B32, ICQ_PROBE_LDS_B64, ICQ_PROBE_LDS_B128, ICQ_PROBE_VALU, \
    ICQ_PROBE_ATOMIC, ICQ_PROBE_MFMA_F32, ICQ_PROBE_MFMA_F32_RANDOM = range(9)


def icq_machine_probe(kind, buffer, reps):
    """(ms per launch, work units per launch) of one probe kernel; buffer: uint8 device tensor >= 4 MiB."""
    ms, units = ctypes.c_double(0), ctypes.c_double(0)
    _check(load().icq_machine_probe(int(kind), _dev(buffer, torch.uint8, name="buffer"), buffer.numel(), int(reps),
                                    ctypes.byref(ms), ctypes.byref(units), _stream()), "icq_machine_probe")
    return float(ms.value), float(units.value)
