"""The C-ABI library loads without a GPU and exports every function that
include/icq.h declares; host-side argument checks reject bad input before any
device work (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "icq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(icq_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_path_calls():
    names = _declared_functions()
    for n in ("icq_build_lut", "icq_scan_fast", "icq_refine", "icq_search"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_1912_08756_amd import binding
    lib = binding.load()
    names = _declared_functions()
    assert sorted(binding.SIGNATURES) == names, "binding and header disagree"
    for n in names:
        assert getattr(lib, n) is not None


def test_missing_library_is_an_error(monkeypatch):
    from paper_1912_08756_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libicq.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_host_side_argument_checks():
    from paper_1912_08756_amd import binding
    lib = binding.load()
    assert binding.strerror(0) == "ok"
    assert "argument" in binding.strerror(binding.ICQ_ERR_ARG)
    h = ctypes.c_void_p(0)
    # null codebooks / bad shapes are rejected before any HIP call
    assert lib.icq_index_create(ctypes.byref(h), None, None, 4, 256, 32, 1, 0, None) == binding.ICQ_ERR_ARG
    one = ctypes.c_void_p(1)
    assert lib.icq_index_create(ctypes.byref(h), one, one, 0, 256, 32, 1, 10, None) == binding.ICQ_ERR_ARG
    assert lib.icq_index_create(ctypes.byref(h), one, one, 4, 257, 32, 1, 10, None) == binding.ICQ_ERR_ARG
    assert lib.icq_index_create(ctypes.byref(h), one, one, 4, 256, 32, 5, 10, None) == binding.ICQ_ERR_ARG
    assert lib.icq_index_create(ctypes.byref(h), one, one, 4, 256, 32, 0, 10, None) == binding.ICQ_ERR_ARG
    assert lib.icq_index_create(ctypes.byref(h), one, one, 4, 256, 32, 1, 2 ** 32, None) == binding.ICQ_ERR_ARG
    assert h.value is None
    out = ctypes.c_size_t(0)
    assert lib.icq_workspace_bytes(None, 1, 1, 1, ctypes.byref(out)) == binding.ICQ_ERR_ARG
    assert lib.icq_build_lut(None, one, 1, one, None) == binding.ICQ_ERR_ARG
    assert lib.icq_scan_fast(None, one, 1, one, one, one, one, 1, one, 0, None) == binding.ICQ_ERR_ARG
    assert lib.icq_refine(None, one, 1, one, one, one, 1, 1, one, one, one, 0, None) == binding.ICQ_ERR_ARG
    assert lib.icq_search(None, one, 1, one, 1, 1, one, one, None, one, 0, None) == binding.ICQ_ERR_ARG
    assert lib.icq_search_static(None, one, 1, one, 1, 1, one, one, None, None) == binding.ICQ_ERR_ARG
    assert "scratch" in binding.strerror(binding.ICQ_ERR_SCRATCH)
    lib.icq_index_destroy(None)


def test_host_side_argument_checks_of_the_policy_encoding_and_utility_calls():
    from paper_1912_08756_amd import binding
    lib = binding.load()
    E = binding.ICQ_ERR_ARG
    one = ctypes.c_void_p(1)
    out = ctypes.c_size_t(0)
    assert lib.icq_index_set_scan_mode(None, 0) == E
    assert lib.icq_index_scan_positions(None, 1, None) == E
    assert lib.icq_machine_probe(0, None, 1 << 22, 1, None, None, None) == E
    assert lib.icq_machine_probe(99, one, 1 << 22, 1, None, None, None) == E
    assert lib.icq_index_set_stage_timing(None, 1) == E
    assert lib.icq_index_stage_times(None, None, None, None) == E
    assert lib.icq_index_export_codes(None, 0, one, None) == E
    assert lib.icq_sample_thresholds(None, one, 1, None, 10, 100, one, None) == E
    assert lib.icq_running_workspace_bytes(None, 1, 1, 10, 10, ctypes.byref(out)) == E
    assert lib.icq_search_running(None, None, 1, one, 1, None, 10, 10, one, one, one, one, 1 << 20, None) == E
    assert lib.icq_op_counts(None, one, 1, one, one, None) == E
    assert lib.icq_encode_workspace_bytes(None, 10, ctypes.byref(out)) == E
    assert lib.icq_encode(None, one, 10, one, one, 1 << 20, None) == E
    assert lib.icq_encode_refine(None, one, 10, one, 1, None, one, 1 << 20, None) == E
    assert lib.icq_quantization_error(None, one, 10, one, one, None) == E
    # the utilities take no index: bad sizes and null pointers
    assert lib.icq_batch_moments(one, -1, 4, one, one, None) == E
    assert lib.icq_batch_moments(one, 10, 0, one, one, None) == E
    assert lib.icq_batch_moments(None, 10, 4, one, one, None) == E
    assert lib.icq_online_variance_update(one, one, one, one, 4, 0, None) == E
    assert lib.icq_online_variance_update(None, one, one, one, 4, 1, None) == E
    assert lib.icq_subspace_mask(one, 4, 0.8, 0.0, 0.2, 1.0, 1.0, -10.0, one, None) == E      # sigma1 must be > 0
    assert lib.icq_subspace_mask(one, 4, 0.8, 1.0, 0.2, 1.0, float("nan"), -10.0, one, None) == E
    assert lib.icq_subspace_mask(None, 4, 0.8, 1.0, 0.2, 1.0, 1.0, -10.0, one, None) == E
    assert lib.icq_fast_set(None, one, one, None) == E
    assert lib.icq_margin(one, one, 0, one, None) == E
    assert lib.icq_margin(one, None, 4, one, None) == E
