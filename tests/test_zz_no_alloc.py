"""icq_search_static -- icq_search on the library's built-in scratch array, for callers that
cannot allocate -- against icq_search with a caller workspace: same kernels, so the rows must
be identical.  Two calls in a row, the second with a smaller input, because the array keeps
the first call's contents."""
import numpy as np
import pytest

from helpers import thresholds_quantile
from oracle import icq_oracle as orc
from paper_1912_08756_amd import synth

pytestmark = pytest.mark.gpu


def _case(torch, b, name, N, Q, topk, cap, frac):
    cfg = synth.make(name, N=N, Q=Q)
    T = orc.lut(cfg["codebooks"], cfg["queries"])
    thr = thresholds_quantile(orc.partial(T, cfg["codes"], cfg["Kf"]), frac)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    index = b.icq_index_create(dev(cfg["codebooks"]), dev(cfg["codes"]), cfg["Kf"])
    queries, thr_d = dev(cfg["queries"]), dev(thr)
    out = {}
    for which in ("workspace", "static"):
        ids = torch.full((Q, topk), -7, dtype=torch.int32, device="cuda")
        dist = torch.full((Q, topk), -7.0, dtype=torch.float32, device="cuda")
        surv = torch.full((Q,), -7, dtype=torch.int32, device="cuda")
        if which == "workspace":
            ws = torch.empty(b.icq_workspace_bytes(index, Q, cap, topk), dtype=torch.uint8, device="cuda")
            b.icq_search(index, queries, thr_d, cap, topk, ids, dist, surv, ws)
        else:
            assert b.icq_workspace_bytes(index, Q, cap, topk) <= b.ICQ_STATIC_SCRATCH_BYTES
            b.icq_search_static(index, queries, thr_d, cap, topk, ids, dist, surv)
        torch.cuda.synchronize()
        out[which] = (ids.cpu().numpy(), dist.cpu().numpy(), surv.cpu().numpy())
    for a, c in zip(out["workspace"], out["static"]):
        assert np.array_equal(a, c)
    assert (out["static"][2] > 0).all() and (out["static"][0][:, 0] >= 0).all()
    # and the rows are the oracle's wherever no tie or band case can reorder them
    o_ids, _, o_cnt = orc.search(T, cfg["codes"], cfg["Kf"], thr, topk)
    same = (out["static"][0].view(np.uint32) == o_ids).all(axis=1)
    assert same.mean() > 0.8
    return index


def test_search_on_the_built_in_scratch_matches_search_with_a_workspace():
    import torch
    from paper_1912_08756_amd import binding as b
    b.load()
    # item-by-item stage 1 with candidate lists and keys in the scratch array (Kf = 4) ...
    _case(torch, b, "C2", N=60_000, Q=96, topk=100, cap=2048, frac=0.01)
    # ... then a smaller call on the same array (fewer queries, shorter lists, grouped stage 1)
    _case(torch, b, "C1", N=30_000, Q=40, topk=10, cap=512, frac=0.01)
    # ... and the item-by-item form again, smaller than the first
    _case(torch, b, "C2", N=20_000, Q=24, topk=50, cap=1024, frac=0.02)


def test_a_call_beyond_the_scratch_array_is_refused():
    import torch
    from paper_1912_08756_amd import binding as b
    cfg = synth.make("C2", N=20_000, Q=64)     # Kf = 4: candidate lists and keys live in the workspace
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    index = b.icq_index_create(dev(cfg["codebooks"]), dev(cfg["codes"]), cfg["Kf"])
    Q, topk, cap = cfg["Q"], 10, 1 << 20       # 64 lists of 2^20 ids do not fit 32 MiB
    assert b.icq_workspace_bytes(index, Q, cap, topk) > b.ICQ_STATIC_SCRATCH_BYTES
    ids = torch.empty((Q, topk), dtype=torch.int32, device="cuda")
    dist = torch.empty((Q, topk), dtype=torch.float32, device="cuda")
    with pytest.raises(b.IcqError) as e:
        b.icq_search_static(index, dev(cfg["queries"]), torch.zeros(Q, device="cuda"), cap, topk, ids, dist, None)
    assert e.value.code == b.ICQ_ERR_SCRATCH
