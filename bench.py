#!/usr/bin/env python3
"""Throughput of the ICQ query-time path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--streams 2]

A step is one pass of the whole path (table build, stage-1 scan, stage-2 refine,
top-k) over the workload's whole query set, one icq_search call per query batch of
the size the workload names, inputs resident in HBM.  The default workload is the
largest one: N = 1e8 items, K = 16, Kf = 4, 1000 queries in batches of 128, top-100.
The calls of a step alternate between two HIP streams (one workspace each), so one
batch's stage 2 runs beside the next batch's stage 1; the same steps are timed on
one stream first, and the stage times and rooflines come from that pass.
Prints ONE JSON line: queries/s; `roofline` for the dominant kernel of that step
with the resource that binds it, its work model and the time of its launches
measured by events on the launch stream inside the one-stream calls; the same for
stage 2; the step with stage 1 walking all Kf fast rows item by item; the stage-1
scan on a 400 MB fast-code array with one, two and four queries per pass (bound by
HBM); the CPU oracle timed on the host cores as a baseline, its lists doubling as
the oracle-matched check; and every other workload shape, each checked against
the oracle by the acceptance rule.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E
# Plain vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 lane operations per second (the
# published 157.3 TFLOP/s fp32 counts a fused multiply-add as two and assumes the packed two-wide
# form; an add, a compare or a bit operation is one operation in one lane)
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# LDS: table reads are priced per lane address against the rate measured for 16-byte reads of a
# conflict-free table (profiles/machine_limits.txt: 9.3e12, 11.4e12 and 7.7e12 addresses per second for
# 4-, 8- and 16-byte reads -- about 16 per clock and CU whatever the width); the four-queries-per-pass
# kernels read 16 bytes (the four queries' entries) per address
LDS_PEAK_GADDR = 7720.0                     # 1e9 addresses per second, 16-byte reads
SURVIVE_FRAC = 0.01


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def sampled_thresholds(torch, b, cb_dev, codes_dev, queries_dev, Kf, frac, n_sample, seed):
    """Per-query threshold = the frac-quantile of the crude distance over a random
    sample of items.  The crude distances come from the library itself (table
    build + stage-1 scan with an infinite threshold on an index over the sample);
    only the quantile pick is a torch op.  Input preparation, not timed."""
    K, N = codes_dev.shape
    Q = queries_dev.shape[0]
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    pick = torch.randint(0, N, (n_sample,), device="cuda", generator=g)
    sample_codes = codes_dev[:, pick].contiguous()
    idx = b.icq_index_create(cb_dev, sample_codes, Kf)
    kth = max(1, int(math.ceil(frac * n_sample)))
    thr = torch.empty(Q, dtype=torch.float32, device="cuda")
    step = 2048
    for q0 in range(0, Q, step):
        qs = queries_dev[q0:q0 + step].contiguous()
        nq = qs.shape[0]
        lut = torch.empty((nq, K, 256), dtype=torch.float32, device="cuda")
        b.icq_build_lut(idx, qs, lut)
        ids = torch.empty((nq, n_sample), dtype=torch.int32, device="cuda")
        part = torch.empty((nq, n_sample), dtype=torch.float32, device="cuda")
        cnt = torch.empty((nq,), dtype=torch.int32, device="cuda")
        ws = torch.empty(b.icq_workspace_bytes(idx, nq, n_sample, 1), dtype=torch.uint8, device="cuda")
        inf = torch.full((nq,), float("inf"), dtype=torch.float32, device="cuda")
        b.icq_scan_fast(idx, lut, inf, ids, part, cnt, ws)
        torch.cuda.synchronize()
        assert int(cnt.min()) == n_sample and int(cnt.max()) == n_sample
        thr[q0:q0 + nq] = torch.kthvalue(part, kth, dim=1).values
    torch.cuda.synchronize()
    del idx
    return thr


def event_time_ms(torch, fn, reps):
    """Average duration of fn() over reps, by events on the launch stream."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / reps


def hbm_leg(torch, b, steps, warmup):
    """Stage-1 scan of a 400 MB fast-code array (N = 1e8, Kf = 4) for one, two and four
    queries per pass: every code byte is read from HBM once per pass, so the kernel
    is bound by the code stream (with four queries the table reads weigh as much)."""
    from paper_1912_08756_amd import synth
    N, Kf, d = 100_000_000, 4, 96
    g = torch.Generator(device="cuda")
    g.manual_seed(4)
    codes = torch.randint(0, 256, (Kf, N), dtype=torch.uint8, device="cuda", generator=g)
    cb = torch.from_numpy(synth.make_codebooks(Kf, 256, d, synth.sigmas(("geom", 0.8), Kf), 4)).cuda()
    idx = b.icq_index_create(cb, codes, Kf)
    out = {}
    for Q, grouped in ((1, False), (2, False), (4, False), (1, True), (2, True)):
        # item by item over all four rows (the 400 MB stream), or over the two rows left when the
        # items are ordered by their first two fast sub-codes
        b.icq_index_set_scan_mode(idx, b.ICQ_SCAN_GROUPED if grouped else b.ICQ_SCAN_STREAMED)
        npos = b.icq_index_scan_positions(idx, Q)
        src = codes[:, :Q].long()
        q = torch.stack([sum(cb[k, src[k, i]] for k in range(Kf)) for i in range(Q)]).contiguous()
        q = q + 0.05 * q.norm(dim=1, keepdim=True) / math.sqrt(d) * torch.randn((Q, d), device="cuda", generator=g)
        thr = sampled_thresholds(torch, b, cb, codes, q, Kf, SURVIVE_FRAC, 65536, 5)
        cap = int(N * SURVIVE_FRAC * 2)
        lut = torch.empty((Q, Kf, 256), dtype=torch.float32, device="cuda")
        b.icq_build_lut(idx, q, lut)
        ids = torch.empty((Q, cap), dtype=torch.int32, device="cuda")
        cnt = torch.empty((Q,), dtype=torch.int32, device="cuda")
        ws = torch.empty(b.icq_workspace_bytes(idx, Q, cap, 1), dtype=torch.uint8, device="cuda")

        def run():
            b.icq_scan_fast(idx, lut, thr, ids, None, cnt, ws)
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        # the library's own events on the launch stream: after the counter fill .. after the scan kernel
        b.icq_index_set_stage_timing(idx, True)
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        stage, calls, _ = b.icq_index_stage_times(idx)
        b.icq_index_set_stage_timing(idx, False)
        ms = stage[1]
        surv = int(cnt.sum().item())
        # what the launch must move: the streamed rows once, the tables, the survivors' ids
        # (grouped: two rows and one 4-byte label per 16 positions, over the padded positions)
        rows = (Kf - 2) * npos + npos // 4 if grouped else Kf * N
        alg_bytes = rows + 4 * Q * Kf * 256 + 4 * surv
        achieved = alg_bytes / (ms * 1e-3) / 1e9
        nt = "true" if Q <= 2 and rows > (256 << 20) else "false"
        kern = "scan_stream_kernel<%d,%d,%s,%s,false>" % (Kf - 2 if grouped else Kf, Q, nt, "true" if grouped else "false")
        tr = pmc_traffic("scan_stream_kernel_B%d%s" % (Q, "g" if grouped else ""), "fast400MB")
        out["B%d%s" % (Q, "_grouped" if grouped else "")] = {
            "bound": "hbm", "kernel": kern, "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
            "algorithmic_bytes": alg_bytes, "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None,
            "ms": round(ms, 4),
            "workload": "fast codes [4][1e8] u8 (400 MB)%s, %d quer%s per pass, %d survivors"
                        % (", items ordered by the first two: %d positions, %d MB streamed" % (npos, rows >> 20) if grouped else "",
                           Q, "y" if Q == 1 else "ies", surv)}
    return out


def rule_check(orc, cfg, thr_np, qs, gpu_ids, gpu_dist):
    """The acceptance rule (tests/helpers.py: distances within 1e-4 (|d| + 1), top-k sets equal up
    to ties and to items within that tolerance of the threshold) on the queries `qs`, against the
    oracle's crude and full distances of EVERY item.  Raises AssertionError on a violation."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import check_topk
    codes, Kf, K, topk = cfg["codes"], cfg["Kf"], cfg["K"], cfg["topk"]
    group = max(1, min(16, int(2e9 // (16 * codes.shape[1]))))     # P and D: 16 bytes per item and query
    for c0 in range(0, len(qs), group):
        sel = np.asarray(qs[c0:c0 + group], dtype=np.int64)
        T = orc.lut(cfg["codebooks"], cfg["queries"][sel])
        P = orc.partial(T, codes, Kf)
        D = orc.partial(T, codes, K)        # all K terms, k ascending: the full distance
        for j, q in enumerate(sel):
            check_topk(P[j], D[j], thr_np[q], topk, gpu_ids[q], gpu_dist[q])
    return len(qs)


def cpu_baseline(cfg, thr_np, gpu_ids, gpu_dist, target_s=15.0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the
    same workload; its results double as the oracle-matched check of the GPU lists."""
    from oracle import icq_oracle as orc
    codes, cb, queries = cfg["codes"], cfg["codebooks"], cfg["queries"]
    Kf, topk = cfg["Kf"], cfg["topk"]
    Q = queries.shape[0]
    pilot = min(Q, orc.threads())
    t0 = time.perf_counter()
    T = orc.lut(cb, queries[:pilot])
    orc.search(T, codes, Kf, thr_np[:pilot], topk)
    per_q = (time.perf_counter() - t0) / pilot
    n = int(min(Q, max(pilot, target_s / max(per_q, 1e-9))))
    t0 = time.perf_counter()
    T = orc.lut(cb, queries[:n])
    o_ids, o_dist, o_cnt = orc.search(T, codes, Kf, thr_np[:n], topk)
    dt = time.perf_counter() - t0
    # oracle-matched: identical-list rate on all sampled queries; the acceptance rule itself on the
    # first few and on a bounded number of those whose lists differ from the oracle's (ties and items
    # within rounding of the threshold or of the topk-th distance, which the rule decides)
    identical = (gpu_ids[:n] == o_ids).all(axis=1)
    differ = np.nonzero(~identical)[0]
    few = 16 if codes.shape[1] <= 20_000_000 else 4
    most = 48 if codes.shape[1] <= 20_000_000 else 12
    check = np.unique(np.concatenate([np.arange(min(n, few)), differ[:most]])).astype(np.int64)
    rule_check(orc, cfg, thr_np, check, gpu_ids, gpu_dist)
    same = float(identical.mean())
    return ({"value": round(n / dt, 2), "unit": "queries/s", "cores": orc.threads(), "kind": "oracle",
             "sample": "first %d of %d queries of the workload, full N, table build + two-step search, "
                       "%.1f s wall" % (n, Q, dt)},
            {"checked_queries": int(len(check)), "checked_of_the_differing": int(min(len(differ), most)),
             "rule_violations": 0, "differing_lists": int(len(differ)), "identical_lists_frac": round(same, 4),
             "sampled_queries": n})


def tile_bounds(N, first=8192, growth=4):
    """Tiles growing by a factor of four from 8192 items: the threshold of Sec. 3.4's loop tightens
    fastest over the first items.  (At N = 1e8, 128 queries: 8 tiles, 38.9 k exact comparisons per
    query in 1.98 ms; doubling from 16384: 13 tiles, 36.5 k in 2.45 ms; factor 8: 6 tiles, 50 k in 1.84 ms.)"""
    bounds, size = [0], first
    while bounds[-1] + size < N:
        bounds.append(bounds[-1] + size)
        size *= growth
    bounds.append(N)
    return bounds


def policy_leg(torch, b, cfg, index, queries, step_args, steps, with_cpu, cb=None, codes=None):
    """The paper's threshold policy on the same workload: thresholds from the first M items
    with the margin of Eq. 11 (icq_sample_thresholds), then the two-step search, then the
    operation counts of the paper's speed axis; on a few queries the result is compared with
    the paper's serial loop (oracle) run with the same margin."""
    K, Kf, N, topk = cfg["K"], cfg["Kf"], cfg["N"], cfg["topk"]
    Q = queries.shape[0]
    M = 4096
    # margin: variance of the data in the part of space the slow codebooks cover, summed over
    # the dimensions -- for sub-codes drawn uniformly that is the codeword variance of the slow
    # codebooks (input preparation, from the codebooks alone)
    cbk = cfg["codebooks"].astype(np.float64)
    sigma_val = float(sum(cbk[k].var(axis=0).sum() for k in range(Kf, K)))
    sigma = torch.full((Q,), sigma_val, dtype=torch.float32, device="cuda")
    cap, out_ids, out_dist, surv, ws = step_args
    out_ids, out_dist, surv = out_ids[:Q], out_dist[:Q], surv[:Q]
    lut = torch.empty((Q, K, 256), dtype=torch.float32, device="cuda")
    thr = torch.empty((Q,), dtype=torch.float32, device="cuda")
    b.icq_build_lut(index, queries, lut)

    def sample():
        b.icq_sample_thresholds(index, lut, sigma, topk, M, thr)

    def whole():   # what a caller runs per batch: tables for the policy, policy, search (which builds its own tables)
        b.icq_build_lut(index, queries, lut)
        b.icq_sample_thresholds(index, lut, sigma, topk, M, thr)
        b.icq_search(index, queries, thr, cap, topk, out_ids, out_dist, surv, ws)
    sample()
    whole()
    torch.cuda.synchronize()
    ms_sample = event_time_ms(torch, sample, max(3, steps))
    ms_whole = event_time_ms(torch, whole, max(3, steps))
    ops = torch.empty((Q,), dtype=torch.int64, device="cuda")
    summary = torch.empty((4,), dtype=torch.float64, device="cuda")
    b.icq_op_counts(index, surv, ops, summary)
    torch.cuda.synchronize()
    sm = summary.cpu().numpy()
    surv_np = surv.cpu().numpy().view(np.uint32)
    out = {"queries": Q,
           "policy": "t_q = crude distance of the top-%d-th nearest of the first %d items + sigma" % (topk, M),
           "sigma": round(sigma_val, 4), "ms_sample_thresholds": round(ms_sample, 4),
           "ms_tables_policy_search": round(ms_whole, 4), "queries_per_s": round(Q / (ms_whole * 1e-3), 1),
           "survivors_mean": round(float(surv_np.mean()), 1), "survivors_frac": round(float(surv_np.mean()) / N, 5),
           "ops_two_step_mean": float(sm[0]), "ops_one_step": float(sm[1]), "ops_ratio": round(float(sm[2]), 5),
           "code_bits": K * 8, "effective_code_bits": round(float(sm[3]), 3)}
    tiled_ids = None
    if cb is not None and codes is not None:
        # the loop's threshold refreshed per tile (icq_search_running): tiles of doubling size
        bounds = tile_bounds(N)
        tiles = [b.icq_index_create(cb, codes[:, a:e].contiguous(), Kf) for a, e in zip(bounds[:-1], bounds[1:])]
        tcap = max(bounds[1], cap)
        t_ids = torch.empty((Q, topk), dtype=torch.int32, device="cuda")
        t_dist = torch.empty((Q, topk), dtype=torch.float32, device="cuda")
        t_ref = torch.empty((Q,), dtype=torch.int32, device="cuda")
        tws = torch.empty(b.icq_running_workspace_bytes(tiles, Q, tcap, topk), dtype=torch.uint8, device="cuda")

        def tiled():
            b.icq_search_running(tiles, bounds[:-1], queries, sigma, tcap, topk, t_ids, t_dist, t_ref, tws)
        tiled()
        torch.cuda.synchronize()
        ms_tiled = event_time_ms(torch, tiled, max(3, steps))
        b.icq_op_counts(index, t_ref, ops, summary)
        torch.cuda.synchronize()
        st = summary.cpu().numpy()
        ref_np = t_ref.cpu().numpy().view(np.uint32)
        tiled_ids = t_ids.cpu().numpy().view(np.uint32)
        out["tiled_running"] = {
            "policy": "threshold of the loop refreshed per tile: %d tiles growing fourfold from %d items" % (len(tiles), bounds[1]),
            "ms_tables_search": round(ms_tiled, 4), "queries_per_s": round(Q / (ms_tiled * 1e-3), 1),
            "refined_mean": round(float(ref_np.mean()), 1), "refined_frac": round(float(ref_np.mean()) / N, 6),
            "ops_two_step_mean": float(st[0]), "ops_ratio": round(float(st[2]), 5),
            "effective_code_bits": round(float(st[3]), 3)}
        for t in tiles:
            b.icq_index_destroy(t)
        del tws, tiles
        torch.cuda.empty_cache()
    if with_cpu:
        from oracle import icq_oracle as orc
        nq = min(16, Q)
        T = orc.lut(cfg["codebooks"], cfg["queries"][:nq])
        t0 = time.perf_counter()
        r_ids, _, refined = orc.running_search(T, cfg["codes"], Kf, np.full(nq, sigma_val), topk)
        dt = time.perf_counter() - t0
        e_ids, _ = orc.adc_exhaustive(T, cfg["codes"], topk)
        g_ids = out_ids[:nq].cpu().numpy().view(np.uint32)
        inter = lambda a, c: float(np.mean([np.intersect1d(a[q], c[q]).size / topk for q in range(nq)]))
        if tiled_ids is not None:
            out["tiled_running"].update(
                recall_of_exhaustive_lists=round(inter(tiled_ids[:nq], e_ids), 4),
                recall_of_serial_loop_lists=round(inter(tiled_ids[:nq], r_ids), 4),
                refined_mean_of_these_queries=float(ref_np[:nq].mean()))
        out["vs_serial_loop"] = {
            "queries": nq, "recall_of_serial_loop_lists": round(inter(g_ids, r_ids), 4),
            "recall_of_exhaustive_lists": round(inter(g_ids, e_ids), 4),
            "serial_loop_recall_of_exhaustive": round(inter(r_ids, e_ids), 4),
            "serial_loop_refined_mean": float(refined.mean()),
            "two_pass_refined_mean": float(surv_np[:nq].mean()),
            "serial_loop_queries_per_s_cpu": round(nq / dt, 2)}
    return out


def encode_leg(torch, b, cfg, steps):
    """Greedy residual encoding of N vectors of the workload's shape (reconstructions of random
    codes plus 5 % noise, drawn on the GPU: input preparation).  One contraction [N x d].[d x 256]
    per codebook on the fp32 matrix cores."""
    K, d = cfg["K"], cfg["d"]
    N = min(cfg["N"], 1 << 20)
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    cb = torch.from_numpy(cfg["codebooks"]).cuda()
    src = torch.randint(0, 256, (K, N), device="cuda", generator=g)
    x = torch.zeros((N, d), dtype=torch.float32, device="cuda")
    for k in range(K):
        x += cb[k][src[k]]
    x += 0.05 * x.norm(dim=1, keepdim=True) / math.sqrt(d) * torch.randn((N, d), device="cuda", generator=g)
    index = b.icq_index_create(cb, torch.empty((K, 0), dtype=torch.uint8, device="cuda"), cfg["Kf"])
    codes = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    ws = torch.empty(b.icq_encode_workspace_bytes(index, N), dtype=torch.uint8, device="cuda")

    def run():
        b.icq_encode(index, x, codes, ws)
    run()
    torch.cuda.synchronize()
    ms = event_time_ms(torch, run, max(3, steps))
    same = float((codes == src.to(torch.uint8)).all(dim=0).float().mean().item())
    d_pad = (d + 15) // 16 * 16
    flops = 2.0 * N * K * 256 * d_pad
    ach = flops / (ms * 1e-3) / 1e12
    # quality: mean ||x - xbar||^2 of the planted codes (the noise), of the greedy codes, and of the
    # greedy codes after sweeps of coordinate descent over the codebooks (icq_encode_refine)
    err = torch.empty((N,), dtype=torch.float64, device="cuda")

    def mean_err(c):
        b.icq_quantization_error(index, x, c, err)
        return float(err.mean().item())
    e_planted = mean_err(src.to(torch.uint8).contiguous())
    e_greedy = mean_err(codes)
    sweeps = 4
    changed = torch.zeros((sweeps,), dtype=torch.int32, device="cuda")
    greedy = codes.clone()
    refined = codes.clone()

    def refine():
        refined.copy_(greedy)
        b.icq_encode_refine(index, x, refined, sweeps, changed, ws)
    refine()
    torch.cuda.synchronize()
    ms_refine = event_time_ms(torch, refine, max(3, steps))
    e_refined = mean_err(refined)
    same_r = float((refined == src.to(torch.uint8)).all(dim=0).float().mean().item())
    x_norm2 = float((x.double() ** 2).sum(dim=1).mean().item())
    return {"bound": "mfma", "kernel": "encode_level_kernel", "achieved": round(ach, 2), "peak": 157.3,
            "unit": "TFLOP/s", "frac": round(ach / 157.3, 4), "traffic": None, "ms": round(ms, 4),
            "items_per_s": round(N / (ms * 1e-3), 1), "N": N, "codes_recovered_frac": round(same, 4),
            "mean_sq_error": {"planted_codes": round(e_planted, 4), "greedy": round(e_greedy, 4),
                              "greedy_then_%d_sweeps" % sweeps: round(e_refined, 4), "mean_sq_norm_of_x": round(x_norm2, 2)},
            "refine": {"sweeps": sweeps, "ms": round(ms_refine, 4), "subcodes_changed_per_sweep": changed.cpu().tolist(),
                       "codes_recovered_frac": round(same_r, 4),
                       "TFLOPs": round(flops * sweeps / (ms_refine * 1e-3) / 1e12, 2)},
            "note": "%d launches (one per codebook); flops = 2*N*K*256*d_pad; fp32 inputs on "
                    "v_mfma_f32_32x32x2_f32; each level also rewrites the N x d residuals" % K}


def counted_vector_instructions(kernel, workload):
    """Wavefront vector instructions per launch of `kernel` on `workload` from the committed SQ
    counter summary (line `issue <kernel> <workload> <count>` in profiles/sq_counters_<workload>.txt)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "sq_counters_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 4 and f[0] == "issue" and f[1] == kernel and f[2] == workload:
            return float(f[3])
    return None


def pmc_traffic(kernel, workload):
    """HBM-side bytes per launch of `kernel` on `workload` from the committed counter summary
    (two rocprofv3 --pmc runs of this program, scaled by what the counters read for a copy of
    known size) -- a figure of that profile, not of this run -- or None when the summary has
    no line for this kernel and workload.  Line format:
    `traffic <kernel> <workload> <fetch_bytes> <write_bytes>`."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 5 and f[0] == "traffic" and f[1] == kernel and f[2] == workload:
            return {"workload": f[2], "fetch_bytes": float(f[3]), "write_bytes": float(f[4]),
                    "bytes": float(f[3]) + float(f[4]), "source": "profiles/pmc_traffic.txt (committed rocprofv3 run)"}
    return None


def configs_leg(torch, b, synth, skip, with_cpu, target_s=4.0):
    """Queries/s of the whole path at every other workload shape (full N, the batch size the
    shape names), with the oracle timed beside it on a bounded sample of the same queries.
    Thresholds: the shape's own rule for C0 (1.5 x the 20th-smallest crude distance), else
    the sampled 1 % quantile.  Input preparation is not timed."""
    from oracle import icq_oracle as orc
    out = {}
    for name in ("C0", "C1", "C2", "C3", "C4"):
        if name == skip:
            continue
        batch = synth.CONFIGS[name]["batch"]
        t_prep = time.perf_counter()
        cfg = synth.make(name)
        K, Kf, d, N, Q, topk = cfg["K"], cfg["Kf"], cfg["d"], cfg["N"], cfg["Q"], cfg["topk"]
        batch = batch or Q
        cb = torch.from_numpy(cfg["codebooks"]).cuda()
        codes = torch.from_numpy(cfg["codes"]).cuda()
        queries = torch.from_numpy(cfg["queries"]).cuda()
        index = b.icq_index_create(cb, codes, Kf)
        if name == "C0":
            lut = torch.empty((Q, K, 256), dtype=torch.float32, device="cuda")
            b.icq_build_lut(index, queries, lut)
            ids = torch.empty((Q, N), dtype=torch.int32, device="cuda")
            part = torch.empty((Q, N), dtype=torch.float32, device="cuda")
            cnt = torch.empty((Q,), dtype=torch.int32, device="cuda")
            ws0 = torch.empty(b.icq_workspace_bytes(index, Q, N, 1), dtype=torch.uint8, device="cuda")
            b.icq_scan_fast(index, lut, torch.full((Q,), float("inf"), device="cuda"), ids, part, cnt, ws0)
            thr = (torch.kthvalue(part, 20, dim=1).values * 1.5).contiguous()
            cap = N
            del lut, ids, part, cnt, ws0
        else:
            thr = sampled_thresholds(torch, b, cb, codes, queries, Kf, SURVIVE_FRAC, 16384, cfg["seed"])
            cap = int(N * SURVIVE_FRAC * 2)
        out_ids = torch.empty((Q, topk), dtype=torch.int32, device="cuda")
        out_dist = torch.empty((Q, topk), dtype=torch.float32, device="cuda")
        surv = torch.empty((Q,), dtype=torch.int32, device="cuda")
        ws = torch.empty(b.icq_workspace_bytes(index, batch, cap, topk), dtype=torch.uint8, device="cuda")

        def run():
            for q0 in range(0, Q, batch):
                b.icq_search(index, queries[q0:q0 + batch], thr[q0:q0 + batch], cap, topk, out_ids[q0:q0 + batch],
                             out_dist[q0:q0 + batch], surv[q0:q0 + batch], ws)
        run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run()
        torch.cuda.synchronize()
        reps = int(min(200, max(3, 0.3 / max(time.perf_counter() - t0, 1e-6))))   # about 0.3 s of timed work
        t0 = time.perf_counter()
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / reps
        surv_np = surv.cpu().numpy().view(np.uint32)
        b.icq_index_set_stage_timing(index, True)
        run()
        torch.cuda.synchronize()
        stage, _, _ = b.icq_index_stage_times(index)
        b.icq_index_set_stage_timing(index, False)
        entry = {"workload": "%s: d=%d K=%d Kf=%d N=%d Q=%d top-%d, batches of %d" % (name, d, K, Kf, N, Q, topk, batch),
                 "queries_per_s": round(Q / sec, 1), "ms_per_batch": round(sec * 1e3 / math.ceil(Q / batch), 4),
                 "stages_ms_per_batch": {"build_lut": round(stage[0], 4), "stage1": round(stage[1], 4), "stage2": round(stage[2], 4)},
                 "stage1_kernel": stage1_kernel_name(Kf, K, N, batch, topk),
                 "survivors_mean": round(float(surv_np.mean()), 1), "overflowed_lists": int((surv_np > cap).sum())}
        if with_cpu:
            thr_np = thr.cpu().numpy()
            n = min(Q, orc.threads())
            t0 = time.perf_counter()
            o_ids = orc.search(orc.lut(cfg["codebooks"], cfg["queries"][:n]), cfg["codes"], Kf, thr_np[:n], topk)[0]
            dt = time.perf_counter() - t0
            more = int(min(Q, n * target_s / max(dt, 1e-9))) // n * n
            if more > n and dt < target_s / 2:
                n = more
                t0 = time.perf_counter()
                o_ids = orc.search(orc.lut(cfg["codebooks"], cfg["queries"][:n]), cfg["codes"], Kf, thr_np[:n], topk)[0]
                dt = time.perf_counter() - t0
            g_ids = out_ids.cpu().numpy().view(np.uint32)
            g_dist = out_dist.cpu().numpy()
            identical = (g_ids[:n] == o_ids).all(axis=1)
            differ = np.nonzero(~identical)[0]
            # the acceptance rule on the first queries and on (at most 16 of) the lists that differ; a
            # violation raises and the bench fails
            check = np.unique(np.concatenate([np.arange(min(n, 4)), differ[:16]])).astype(np.int64)
            rule_check(orc, cfg, thr_np, check, g_ids, g_dist)
            entry["oracle"] = {"queries_per_s": round(n / dt, 2), "cores": orc.threads(),
                               "sample": "first %d queries, full N, %.1f s wall" % (n, dt),
                               "identical_lists_frac": round(float(identical.mean()), 4),
                               "differing_lists": int(len(differ)), "rule_checked_queries": int(len(check)),
                               "rule_violations": 0}
            entry["gpu_over_oracle"] = round(Q / sec / (n / dt), 1)
        out[name] = entry
        log("[bench] %s: %.0f queries/s (%.3f ms per batch of %d)%s, prepared in %.0f s" %
            (name, Q / sec, entry["ms_per_batch"], batch,
             "; oracle %.1f queries/s" % entry["oracle"]["queries_per_s"] if with_cpu else "", time.perf_counter() - t_prep))
        del index, cb, codes, queries, ws, out_ids, out_dist, surv, thr
        torch.cuda.empty_cache()
    return out


def encoded_index_leg(torch, b, synth, with_cpu, sweeps=2):
    """C3's shape with codes that come from the encoder instead of a generator: 1e7 Gaussian-mixture
    vectors (synth.make_vectors) are encoded on the GPU (greedy assignment, then `sweeps` sweeps of
    coordinate descent), indexed and searched like C3.  The oracle beside it encodes a sample of the
    vectors itself -- the GPU's returned neighbours, cluster mates of the queries' sources and random
    items -- and judges codes, distances and completeness of the lists on that sample."""
    from oracle import icq_oracle as orc
    t_prep = time.perf_counter()
    cfg = synth.make_vectors("C3")
    K, Kf, d, N, Q, topk, batch = cfg["K"], cfg["Kf"], cfg["d"], cfg["N"], cfg["Q"], cfg["topk"], cfg["batch"]
    cb = torch.from_numpy(cfg["codebooks"]).cuda()
    x = torch.from_numpy(cfg["x"]).cuda()
    queries = torch.from_numpy(cfg["queries"]).cuda()
    enc = b.icq_index_create(cb, torch.empty((K, 0), dtype=torch.uint8, device="cuda"), Kf)
    ws_e = torch.empty(b.icq_encode_workspace_bytes(enc, N), dtype=torch.uint8, device="cuda")
    codes = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    changed = torch.zeros((sweeps,), dtype=torch.int32, device="cuda")
    err = torch.empty((N,), dtype=torch.float64, device="cuda")

    def mean_err():
        b.icq_quantization_error(enc, x, codes, err)
        return float(err.mean().item())
    b.icq_encode(enc, x, codes, ws_e)
    torch.cuda.synchronize()
    ms_greedy = event_time_ms(torch, lambda: b.icq_encode(enc, x, codes, ws_e), 2)
    e_greedy = mean_err()
    greedy = codes.clone()
    b.icq_encode_refine(enc, x, codes, sweeps, changed, ws_e)
    torch.cuda.synchronize()
    codes.copy_(greedy)
    ms_refine = event_time_ms(torch, lambda: b.icq_encode_refine(enc, x, codes, sweeps, changed, ws_e), 1)
    e_refined = mean_err()
    x_norm2 = float((x[:1 << 20].double() ** 2).sum(dim=1).mean().item())
    del greedy, err, ws_e, x
    torch.cuda.empty_cache()
    t0 = time.perf_counter()
    index = b.icq_index_create(cb, codes, Kf)
    torch.cuda.synchronize()
    ms_index = (time.perf_counter() - t0) * 1e3
    pairs = codes[0].to(torch.int32) * 256 + codes[1].to(torch.int32)
    runs = torch.bincount(pairs, minlength=65536)
    thr = sampled_thresholds(torch, b, cb, codes, queries, Kf, SURVIVE_FRAC, 16384, cfg["seed"])
    cap = int(N * SURVIVE_FRAC * 4)
    out_ids = torch.empty((Q, topk), dtype=torch.int32, device="cuda")
    out_dist = torch.empty((Q, topk), dtype=torch.float32, device="cuda")
    surv = torch.empty((Q,), dtype=torch.int32, device="cuda")
    ws = torch.empty(b.icq_workspace_bytes(index, batch, cap, topk), dtype=torch.uint8, device="cuda")

    def run():
        for q0 in range(0, Q, batch):
            b.icq_search(index, queries[q0:q0 + batch], thr[q0:q0 + batch], cap, topk, out_ids[q0:q0 + batch],
                         out_dist[q0:q0 + batch], surv[q0:q0 + batch], ws)
    run()
    torch.cuda.synchronize()
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / reps
    b.icq_index_set_stage_timing(index, True)
    run()
    torch.cuda.synchronize()
    stage, _, _ = b.icq_index_stage_times(index)
    b.icq_index_set_stage_timing(index, False)
    surv_np = surv.cpu().numpy().view(np.uint32)
    flops = 2.0 * N * K * 256 * ((d + 15) // 16 * 16)
    entry = {"workload": "C3's shape over encoded vectors: d=%d K=%d Kf=%d N=%d Q=%d top-%d, batches of %d; "
                         "%d-cluster Gaussian mixture, spread %.1f" % (d, K, Kf, N, Q, topk, batch, cfg["n_centres"], cfg["spread"]),
             "encode": {"greedy_ms": round(ms_greedy, 2), "greedy_TFLOPs": round(flops / (ms_greedy * 1e-3) / 1e12, 1),
                        "refine_sweeps": sweeps, "refine_ms": round(ms_refine, 2),
                        "subcodes_changed_per_sweep": changed.cpu().tolist(),
                        "mean_sq_error": {"greedy": round(e_greedy, 4), "refined": round(e_refined, 4),
                                          "mean_sq_norm_of_x": round(x_norm2, 2)}},
             "index_build_ms": round(ms_index, 1),
             "fast_pairs_in_use": int((runs > 0).sum().item()), "largest_pair_run": int(runs.max().item()),
             "queries_per_s": round(Q / sec, 1), "ms_per_batch": round(sec * 1e3 / math.ceil(Q / batch), 4),
             "stages_ms_per_batch": {"build_lut": round(stage[0], 4), "stage1": round(stage[1], 4), "stage2": round(stage[2], 4)},
             "stage1_kernel": stage1_kernel_name(Kf, K, N, batch, topk),
             "survivors_mean": round(float(surv_np.mean()), 1), "overflowed_lists": int((surv_np > cap).sum())}
    if with_cpu:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from helpers import tol
        n = 8
        g_ids = out_ids[:n].cpu().numpy().view(np.uint32)
        g_dist = out_dist[:n].cpu().numpy()
        thr_np = thr[:n].cpu().numpy()
        rng = np.random.default_rng(cfg["seed"])
        parts = [g_ids[g_ids != 0xFFFFFFFF].astype(np.int64), rng.integers(0, N, size=4000)]
        for q in range(n):
            mates = np.nonzero(cfg["cluster"] == cfg["cluster"][cfg["query_sources"][q]])[0]
            parts.append(rng.choice(mates, size=min(1500, len(mates)), replace=False))
        S = np.unique(np.concatenate(parts))
        t0 = time.perf_counter()
        xs = np.ascontiguousarray(cfg["x"][S])
        want, _ = orc.encode_icm(cfg["codebooks"], xs, orc.encode(cfg["codebooks"], xs), sweeps)
        got = codes[:, torch.from_numpy(S).cuda()].cpu().numpy()
        same = (want == got).all(axis=0)
        if same.mean() < 0.95:
            raise AssertionError("encoded index: only %.3f of the sampled items carry the oracle's codes" % same.mean())
        S_ok, c_ok = S[same], np.ascontiguousarray(want[:, same])
        T = orc.lut(cfg["codebooks"], cfg["queries"][:n])
        P, D = orc.partial(T, c_ok, Kf), orc.partial(T, c_ok, K)
        checked = skipped = 0
        for q in range(n):
            t = float(thr_np[q])
            valid = g_ids[q] != 0xFFFFFFFF
            pos = np.searchsorted(S_ok, g_ids[q][valid])
            pos[pos >= len(S_ok)] = 0
            known = S_ok[pos] == g_ids[q][valid]
            skipped += int((~known).sum())
            dq = g_dist[q][valid][known]
            if not (np.abs(dq - D[q][pos[known]]) <= tol(D[q][pos[known]])).all():
                raise AssertionError("encoded index, query %d: a returned distance is off" % q)
            if not (P[q][pos[known]] <= t + tol(t)).all():
                raise AssertionError("encoded index, query %d: a returned item is clearly above the threshold" % q)
            dk = float(g_dist[q][-1]) if valid.all() else np.inf
            must = np.nonzero((P[q] < t - tol(t)) & (D[q] < dk - tol(dk)))[0] if np.isfinite(dk) else \
                np.nonzero(P[q] < t - tol(t))[0]
            if not np.isin(S_ok[must], g_ids[q][valid]).all():
                raise AssertionError("encoded index, query %d: a clearly nearer survivor is missing from the list" % q)
            checked += int(known.sum()) + len(must)
        entry["oracle"] = {"sample_items": int(len(S)), "codes_identical_frac": round(float(same.mean()), 4),
                           "queries": n, "checks": checked, "returned_items_with_differing_codes_skipped": skipped,
                           "violations": 0, "cores": orc.threads(), "wall_s": round(time.perf_counter() - t0, 1),
                           "what": "the oracle encodes the sampled vectors itself (greedy + %d sweeps) and judges, on the "
                                   "items whose codes agree, returned distances, the threshold and that no clearly "
                                   "nearer survivor of the sample is missing" % sweeps}
    log("[bench] C3 over encoded vectors: encode %.1f + %.1f ms, index %.0f ms, %.0f queries/s (%.3f ms per batch), "
        "%.0f survivors/query, prepared in %.0f s" % (ms_greedy, ms_refine, ms_index, Q / sec, entry["ms_per_batch"],
                                                      surv_np.mean(), time.perf_counter() - t_prep))
    return entry


def machine_limits(torch, b):
    """What this GPU delivers for the access patterns the kernels are made of (icq_machine_probe):
    the figures behind the peaks the rooflines use."""
    buf = torch.zeros(400_000_000, dtype=torch.uint8, device="cuda")
    out = {}
    for name, kind, reps in (("stream_read_400MB", b.ICQ_PROBE_READ, 20), ("stream_read_400MB_nontemporal", b.ICQ_PROBE_READ_NT, 20),
                             ("lds_read_b32", b.ICQ_PROBE_LDS_B32, 3), ("lds_read_b64", b.ICQ_PROBE_LDS_B64, 3),
                             ("lds_read_b128", b.ICQ_PROBE_LDS_B128, 3), ("valu_add_f32", b.ICQ_PROBE_VALU, 3),
                             ("atomic_add_one_word", b.ICQ_PROBE_ATOMIC, 5), ("mfma_f32_32x32x2", b.ICQ_PROBE_MFMA_F32, 3),
                             ("mfma_f32_32x32x2_random_operands", b.ICQ_PROBE_MFMA_F32_RANDOM, 3)):
        ms, units = b.icq_machine_probe(kind, buf, reps)
        rate = units / (ms * 1e-3)
        e = {"ms": round(ms, 4)}
        if "stream" in name:
            e.update(GBs=round(rate / 1e9, 1), frac_of_8TBs=round(rate / 8e12, 4))
        elif "lds" in name:
            width = {"b32": 4, "b64": 8, "b128": 16}[name.split("_")[-1]]
            e.update(Gaddr_s=round(rate / 1e9, 1), addr_per_clk_per_cu_at_2p4GHz=round(rate / 256 / 2.4e9, 2),
                     bytes_per_clk_per_cu_at_2p4GHz=round(rate * width / 256 / 2.4e9, 1))
        elif "mfma" in name:
            e.update(TFLOPs=round(rate / 1e12, 1), frac_of_157p3=round(rate / 157.3e12, 4))
        elif "valu" in name:
            e.update(Tops_s=round(rate / 1e12, 2), lanes_per_clk_per_cu_at_2p4GHz=round(rate / 256 / 2.4e9, 1))
        else:
            e.update(Matomics_s=round(rate / 1e6, 1))
        out[name] = e
    del buf
    torch.cuda.empty_cache()
    return out


def index_words(K):
    return 1 if K <= 4 else 2 if K <= 8 else 4


def stage1_form(Kf, K, N, Qb, topk):
    """Which stage-1 form the library picks in automatic mode (icq_index_set_scan_mode) for a call
    of Qb queries: 'tuples' (Kf <= 2: one evaluation per fast-code tuple, distances and lists in the
    same kernel), 'pairs' (Kf = 3, 4 from 64 * 65536 items on: items ordered by their first two fast
    sub-codes, the other rows streamed) or 'items' (all Kf rows streamed); and whether stage 1
    hands stage 2 hit bits (from 2^22 items on) or candidate lists."""
    if Kf <= 2 and Qb > 4 and N >= 256 ** Kf // 2:
        return "tuples", False
    bits = Kf <= 4 and K <= 16 and topk <= 512 and (N >= 1 << 22 or (N >= 1 << 19 and Qb >= 32))
    if Kf in (3, 4) and N >= 64 * 65536:
        return "pairs", bits
    return "items", bits


def stage1_kernel_name(Kf, K, N, Qb, topk, mode_streamed=False):
    form, bits = stage1_form(Kf, K, N, Qb, topk)
    if mode_streamed and form != "items":
        form, bits = "items", Kf <= 4 and K <= 16 and topk <= 512 and (N >= 1 << 22 or (N >= 1 << 19 and Qb >= 32))
    if form == "tuples":
        return "group_keys_kernel<%d,%d,%s>" % (Kf, index_words(K), "true" if topk <= 256 and K <= 16 else "false")
    if Kf > 4:
        return "scan_items_kernel"
    if bits and Qb >= 6:
        return "scan_pairs_q16_kernel<%d,%s>" % ((Kf - 2, "true") if form == "pairs" else (Kf, "false"))
    B = 4 if Qb >= 3 else Qb
    return "scan_stream_kernel<%d,%d,false,%s,%s>" % (Kf - 2 if form == "pairs" else Kf, B,
                                                       "true" if form == "pairs" else "false", "true" if bits else "false")


def stage1_model(Kf, npos, Qb, pairs, q16=False):
    """Work of ONE launch of the item-by-item stage-1 kernel over npos scan positions for Qb
    queries.  fp32 form, four queries per pass -- per (query, position): one table read per
    streamed row, the additions of Eq. 2 left of the threshold, one comparison, one instruction
    that collects the hit bit; per position and pass: one byte extraction and one address per
    streamed row (shared by the pass's four queries).  pairs: the first two entries' sum comes once
    per 16 positions (not counted) and is one more addition per (query, position).
    q16 (the 16-bit pre-filter, eight queries per pass): a 32-bit instruction serves two queries,
    so per position and pass there are one address per streamed row, and per PAIR of queries the
    additions (two of them fold into one three-operand instruction) and, per TWO positions, one
    byte permute, one shift and one bit-field insert that collect the four miss bits; per 16
    positions and pass about 26 more (the pair's part of the sum, the tests that let a pair of
    queries sit a step out, masks, stores).
    alu_ops counts lanes of wavefront instructions either way."""
    R = Kf - 2 if pairs else Kf
    if q16:
        passes = (Qb + 7) // 8
        addr = R if R <= 2 else 2 * R          # one byte permute per address with 16 table copies, extract + shift-add with 8
        # per query pair and TWO positions: the additions of both (two per instruction), permute, shift, insert
        per_pair2 = 2 * (((R if pairs else R - 1) + 1) // 2) + 3
        return {"positions": npos, "queries": Qb, "passes": passes, "streamed_rows": R,
                "alu_ops": npos * passes * addr + npos // 2 * passes * 4 * per_pair2 + npos // 16 * passes * (26 if pairs else 24),
                "lds_addresses": npos * passes * R,
                "table_entries": npos * Qb * R,
                "code_bytes": npos * passes * R + npos * passes // 4,
                "hit_bit_bytes": npos * Qb // 8}
    adds = R if pairs else R - 1
    passes = (Qb + 3) // 4 if Qb >= 3 else 1
    return {"positions": npos, "queries": Qb, "passes": passes, "streamed_rows": R,
            "alu_ops": npos * Qb * (adds + 2) + npos * passes * 2 * R,
            "lds_addresses": npos * passes * R,            # one read serves the pass's queries
            "table_entries": npos * Qb * R,
            "code_bytes": npos * passes * R + (npos * passes // 4 if pairs else 0),
            "hit_bit_bytes": npos * Qb // 8}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--streams", type=int, default=2,
                    help="HIP streams the step's icq_search calls alternate between (each with a workspace of its "
                         "own); 1 = all calls on one stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hbm-leg", action="store_true")
    ap.add_argument("--no-streamed-leg", action="store_true")
    ap.add_argument("--no-policy-leg", action="store_true")
    ap.add_argument("--no-encode-leg", action="store_true")
    ap.add_argument("--no-configs-leg", action="store_true")
    ap.add_argument("--machine-limits-only", action="store_true",
                    help="print only the machine-limit probes (one JSON line) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one elementwise copy of 1 GiB (reads 1 GiB, writes 1 GiB): the scale for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_1912_08756_amd import binding as b, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    b.load()

    if args.machine_limits_only:
        print(json.dumps({"machine_limits": machine_limits(torch, b)}), flush=True)
        return

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    log("[bench] drawing workload", args.workload)
    cfg = synth.make(args.workload)
    K, Kf, d, N, Q, topk = cfg["K"], cfg["Kf"], cfg["d"], cfg["N"], cfg["Q"], cfg["topk"]
    batch = min(cfg["batch"], Q)
    nbatches = math.ceil(Q / batch)
    cb = torch.from_numpy(cfg["codebooks"]).cuda()
    codes = torch.from_numpy(cfg["codes"]).cuda()
    queries = torch.from_numpy(cfg["queries"]).cuda()
    index = b.icq_index_create(cb, codes, Kf)
    thr = sampled_thresholds(torch, b, cb, codes, queries, Kf, SURVIVE_FRAC, 16384, cfg["seed"])
    cap = int(N * SURVIVE_FRAC * 2) if N > 1 << 20 else 1 << int(math.ceil(math.log2(max(64, N * SURVIVE_FRAC * 1.5))))
    out_ids = torch.empty((Q, topk), dtype=torch.int32, device="cuda")
    out_dist = torch.empty((Q, topk), dtype=torch.float32, device="cuda")
    surv = torch.empty((Q,), dtype=torch.int32, device="cuda")
    ws_bytes = b.icq_workspace_bytes(index, batch, cap, topk)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    log("[bench] N=%d Q=%d (batches of %d) K=%d Kf=%d d=%d topk=%d cap=%d workspace=%.2f GB" %
        (N, Q, batch, K, Kf, d, topk, cap, ws_bytes / 1e9))

    def step():
        for q0 in range(0, Q, batch):
            b.icq_search(index, queries[q0:q0 + batch], thr[q0:q0 + batch], cap, topk, out_ids[q0:q0 + batch],
                         out_dist[q0:q0 + batch], surv[q0:q0 + batch], ws)

    def timed(steps, warmup):
        """ms per step by the host clock around `steps` passes over the query set, and the stage
        times per icq_search call that the library's own events (on the launch stream) recorded
        inside those same calls (the latest 64 calls)."""
        b.icq_index_set_stage_timing(index, False)
        for _ in range(warmup):
            step()
        b.icq_index_set_stage_timing(index, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        stage, calls, batches = b.icq_index_stage_times(index)
        b.icq_index_set_stage_timing(index, False)
        assert batches == 1, "the workspace must hold a whole query batch"
        return ms, stage, calls

    # One stream first: the library's stage events are recorded inside these calls, undisturbed by
    # other work on the GPU; the rooflines below use them.
    ms_one_stream, stage, calls = timed(args.steps, args.warmup)
    ms_per_step = ms_one_stream
    nstreams = max(1, min(args.streams, nbatches))
    if nstreams > 1:
        # The timed region of record: the same calls alternating between streams, so that one batch's
        # stage 2 (bound by record gathers) runs beside the next batch's stage 1 (bound by vector issue).
        wss = [ws] + [torch.empty(ws_bytes, dtype=torch.uint8, device="cuda") for _ in range(nstreams - 1)]
        streams = [torch.cuda.Stream() for _ in range(nstreams)]          # default priority

        def step_streams():
            cur = torch.cuda.current_stream()
            for st in streams:
                st.wait_stream(cur)
            for i, q0 in enumerate(range(0, Q, batch)):
                with torch.cuda.stream(streams[i % nstreams]):
                    b.icq_search(index, queries[q0:q0 + batch], thr[q0:q0 + batch], cap, topk, out_ids[q0:q0 + batch],
                                 out_dist[q0:q0 + batch], surv[q0:q0 + batch], wss[i % nstreams])
            for st in streams:
                cur.wait_stream(st)
        ids_one = out_ids.clone()
        for _ in range(args.warmup):
            step_streams()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_streams()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        assert bool((out_ids == ids_one).all()), "the calls on several streams gave other lists"
        del wss, streams, ids_one
        torch.cuda.empty_cache()
        log("[bench] %d streams: %.3f ms/step (one stream: %.3f)" % (nstreams, ms_per_step, ms_one_stream))
    surv_np = surv.cpu().numpy().view(np.uint32)
    overflow = int((surv_np > cap).sum())
    n_surv_batch = float(np.minimum(surv_np, cap).sum()) / nbatches
    log("[bench] one stream: %.3f ms/step (%d calls); per call (events, mean of %d calls): lut %.3f, stage 1 %.3f, stage 2 %.3f ms; "
        "survivors mean %.0f max %d, overflowed lists %d" %
        (ms_one_stream, nbatches, calls, stage[0], stage[1], stage[2], surv_np.mean(), surv_np.max(), overflow))
    gpu_ids = out_ids.cpu().numpy().view(np.uint32)
    gpu_dist = out_dist.cpu().numpy()
    qmean = Q / nbatches                       # queries per call (the last batch may be short)

    form, bits = stage1_form(Kf, K, N, batch, topk)
    kern1 = stage1_kernel_name(Kf, K, N, batch, topk)
    npos = b.icq_index_scan_positions(index, batch)
    wl = args.workload
    if form == "tuples":
        # Stage 1 over the items grouped by fast-code tuple, fused with the survivors' distances and
        # the nearest-neighbour lists (one launch is the whole of stages 1 and 2).  It is bound by
        # instruction issue (profiles/sq_counters_C1.txt); priced here by the bytes the method must
        # move -- per survivor its K code bytes, per query its K tables and result rows -- next to
        # the bytes the counters saw, which are fewer: the kernel skips tuples its list's bound excludes.
        alg_bytes = n_surv_batch * K + 4.0 * qmean * K * 256 + 8.0 * qmean * topk
        tr = pmc_traffic("group_keys_kernel", wl)
        insts = counted_vector_instructions("group_keys_kernel", wl)
        issue_peak = 256 * 4 * 2.4e9 / 4.0 / 1e9          # G wavefront instructions/s: one per SIMD every 4 clocks
        ach = insts / (stage[1] * 1e-3) / 1e9 if insts else None
        roofline = {"bound": "issue", "kernel": kern1, "achieved": round(ach, 1) if ach else None, "peak": issue_peak,
                    "unit": "G wavefront vector instructions/s", "frac": round(ach / issue_peak, 4) if ach else None,
                    "ms": round(stage[1], 4), "vector_instructions_per_launch": insts,
                    "instructions_source": "profiles/sq_counters_%s.txt (committed rocprofv3 run)" % wl if insts else None,
                    "hbm": {"algorithmic_bytes": alg_bytes, "achieved_GBs": round(alg_bytes / (stage[1] * 1e-3) / 1e9, 1),
                            "peak_GBs": HBM_PEAK_GBS, "frac": round(alg_bytes / (stage[1] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
                    "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None,
                    "note": "bound by instruction issue: achieved = the wavefront vector instructions one launch issues "
                            "(SQ_INSTS_VALU of the committed counter run; the work depends on the data -- which tuples the "
                            "list's bound excludes -- so it is counted, not modelled) over the stage-1 event time of this "
                            "run; peak = 256 CU x 4 SIMD x 2.4 GHz / 4 clocks.  hbm: the bytes the method must move "
                            "(survivors*K + Q*4*K*256 + Q*topk*8) against 8 TB/s, for reference only: the kernel skips the "
                            "tuples its bound excludes and moves fewer bytes than that (traffic)"}
    else:
        # Item-by-item stage 1: bound by the vector ALUs (every (query, position) pair costs a few
        # plain vector instructions whatever the memory system does; SQ counters in profiles/).
        q16 = kern1.startswith("scan_pairs_q16")
        m = stage1_model(Kf, npos, int(round(qmean)), form == "pairs", q16)
        t = stage[1] * 1e-3
        ach = m["alu_ops"] / t / 1e12
        tr = pmc_traffic("scan_pairs_q16_kernel" if q16 else kern1.split("<")[0] + ("_pairs" if form == "pairs" else "_items"), wl)
        roofline = {"bound": "alu", "kernel": kern1, "achieved": round(ach, 3), "peak": round(ALU_PEAK_TOPS, 2),
                    "unit": "Tops/s", "frac": round(ach / ALU_PEAK_TOPS, 4), "ms": round(stage[1], 4),
                    "work_model": m,
                    # Eq. 2 as written: Kf - 1 additions and one comparison per (query, item).  The kernel needs fewer
                    # instructions than that (two queries per 32-bit instruction, the first two terms once per run of
                    # items), so this rate can exceed the vector peak; it does not depend on how the kernel is written.
                    "eq2": {"ops_per_launch": int(N) * int(round(qmean)) * Kf,
                            "Tops_per_s": round(N * qmean * Kf / t / 1e12, 2),
                            "vs_vector_peak": round(N * qmean * Kf / t / 1e12 / ALU_PEAK_TOPS, 3)},
                    "lds": {"achieved_Gaddr_s": round(m["lds_addresses"] / t / 1e9, 1), "peak_Gaddr_s": LDS_PEAK_GADDR,
                            "frac": round(m["lds_addresses"] / t / 1e9 / LDS_PEAK_GADDR, 4),
                            "table_entries_per_s": round(m["table_entries"] / t, 1)},
                    "hbm": {"algorithmic_bytes": m["code_bytes"] + m["hit_bit_bytes"] + 4 * int(round(qmean)) * Kf * 256,
                            "achieved_GBs": round((m["code_bytes"] + m["hit_bit_bytes"]) / t / 1e9, 1), "peak_GBs": HBM_PEAK_GBS,
                            "frac": round((m["code_bytes"] + m["hit_bit_bytes"]) / t / 1e9 / HBM_PEAK_GBS, 4)},
                    "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None,
                    "note": "one launch per icq_search call; duration = the stage-1 event pair inside the one-stream calls "
                            "(counter fill .. after the scan kernel).  achieved = lanes of the vector instructions of the "
                            "work model (alu_ops; see stage1_model in bench.py: additions, comparison, hit-bit "
                            "collection, table addresses -- a 32-bit instruction serves two queries' 16-bit sums in the "
                            "16-bit pre-filter) per second; peak = 256 CU x 4 SIMD x 16 lanes x 2.4 GHz.  lds / hbm: the same launch against the other two resources "
                            "(LDS: lane addresses against the 7.72e12 per second measured for 16-byte reads; HBM: code "
                            "rows per pass plus the hit bits written -- all passes but the first are served by the caches, "
                            "see traffic).  The vector peak is the rate of three-operand and compare instructions; "
                            "two-operand additions can issue at almost twice that (profiles/machine_limits.txt), so the "
                            "fraction is an upper estimate; SQ counters of the same launch: profiles/sq_counters_C4.txt"}

    result = {
        "metric": "queries/sec at top-%d (oracle-matched)" % topk,
        "value": round(Q / (ms_per_step * 1e-3), 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: d=%d K=%d Kf=%d m=256 N=%d Q=%d in batches of %d, top-%d, ~%.0f%% survive stage 1" %
                   (args.workload, d, K, Kf, N, Q, batch, topk, 100 * SURVIVE_FRAC),
                   "batch": batch, "calls_per_step": nbatches, "streams": nstreams, "cap": cap, "overflowed_lists": overflow,
                   "survivors_mean": round(float(surv_np.mean()), 1),
                   "stage1": {"tuples": "one evaluation per fast-code tuple, distances and lists in the same kernel",
                              "pairs": "items ordered by their first two fast sub-codes, remaining fast rows streamed"
                                       + (" through a conservative 16-bit pre-filter, eight queries per pass; stage 2 "
                                          "applies the exact comparison" if kern1.startswith("scan_pairs_q16") else ""),
                              "items": "all fast rows streamed item by item"}[form],
                   "stage1_to_stage2": "hit bits" if bits else ("on chip" if form == "tuples" else "candidate lists")},
        "ms_per_step_one_stream": round(ms_one_stream, 4),
        "stages_ms_per_call": {"build_lut": round(stage[0], 4), "stage1": round(stage[1], 4), "stage2": round(stage[2], 4),
                               "measured": "the library's events inside the calls of the one-stream pass (%d steps)%s"
                                           % (args.steps, ", timed before the pass of record; with %d streams the calls of a "
                                              "step overlap, so calls_per_step x their sum exceeds ms_per_step" % nstreams
                                              if nstreams > 1 else "")},
        "roofline": roofline,
    }
    if form != "tuples":
        # stage 2: record gathers; what the method must move per call is one 16-byte record per
        # survivor, the hit bits once more, the tables and the result rows
        rec = index_words(K) * 4
        alg2 = n_surv_batch * rec + (npos * qmean / 8 if bits else 4 * n_surv_batch) + 4.0 * qmean * K * 256 + 8.0 * qmean * topk
        ach2 = alg2 / (stage[2] * 1e-3) / 1e9
        k2 = "refine_mask_kernel<%d,true>" % index_words(K) if bits else "refine_dist_kernel<%d>" % index_words(K)
        tr2 = pmc_traffic(k2.split("<")[0], wl)
        result["roofline_stage2"] = {
            "bound": "hbm", "kernel": k2 + " (+ its unfiltered first part and two selections)" if bits else k2 + " + select_keys_kernel",
            "achieved": round(ach2, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach2 / HBM_PEAK_GBS, 4),
            "algorithmic_bytes": alg2, "traffic": tr2["bytes"] if tr2 else None, "traffic_source": tr2["source"] if tr2 else None,
            "ms": round(stage[2], 4), "survivors_per_call": n_surv_batch,
            "note": "all stage-2 kernels of a call (event pair after stage 1 .. results written); algorithmic bytes = "
                    "survivors x record + hit bits (or ids) + tables + result rows.  A random 16-byte gather moves a "
                    "whole cache line, so the traffic is a multiple of the algorithmic bytes unless the line is "
                    "reused from the cache by the batch's other queries"}
        # `roofline` is the stage that takes longer between the library's events; the other keeps its own key
        result["roofline_stage1"] = roofline
        if stage[2] > stage[1]:
            result["roofline"] = dict(result["roofline_stage2"])
            result["roofline"]["why_this_one"] = ("stage 2 takes %.3f ms of the call, stage 1 %.3f (roofline_stage1: bound "
                                                  "by the vector ALUs)" % (stage[2], stage[1]))

    if not args.no_streamed_leg:
        # The same step with stage 1 walking all Kf fast rows item by item (what an index without the
        # grouped layouts runs)
        b.icq_index_set_scan_mode(index, b.ICQ_SCAN_STREAMED)
        ws2 = torch.empty(b.icq_workspace_bytes(index, batch, cap, topk), dtype=torch.uint8, device="cuda")
        ws_keep, ws = ws, ws2
        ms_s, stage_s, _ = timed(max(2, args.steps // 4), 1)
        same = bool((out_ids.cpu().numpy().view(np.uint32) == gpu_ids).all() and (out_dist.cpu().numpy() == gpu_dist).all())
        ws = ws_keep
        del ws2
        b.icq_index_set_scan_mode(index, b.ICQ_SCAN_AUTO)
        if Kf <= 4:
            kern_s = stage1_kernel_name(Kf, K, N, batch, topk, True)
            m = stage1_model(Kf, N, int(round(qmean)), False, kern_s.startswith("scan_pairs_q16"))
            t = stage_s[1] * 1e-3
            ach = m["alu_ops"] / t / 1e12
            result["roofline_streamed"] = {
                "bound": "alu", "kernel": kern_s, "achieved": round(ach, 3),
                "peak": round(ALU_PEAK_TOPS, 2), "unit": "Tops/s", "frac": round(ach / ALU_PEAK_TOPS, 4),
                "ms": round(stage_s[1], 4), "ms_per_step": round(ms_s, 4), "queries_per_s": round(Q / (ms_s * 1e-3), 1),
                "same_lists_as_default": same, "work_model": m,
                "lds": {"achieved_Gaddr_s": round(m["lds_addresses"] / t / 1e9, 1), "peak_Gaddr_s": LDS_PEAK_GADDR,
                        "frac": round(m["lds_addresses"] / t / 1e9 / LDS_PEAK_GADDR, 4),
                        "table_entries_per_s": round(m["table_entries"] / t, 1)},
                "stages_ms_per_call": {"build_lut": round(stage_s[0], 4), "stage1": round(stage_s[1], 4),
                                       "stage2": round(stage_s[2], 4)},
                "traffic": (pmc_traffic(kern_s.split("<")[0] + "_items", wl) or {}).get("bytes"),
                "traffic_source": (pmc_traffic(kern_s.split("<")[0] + "_items", wl) or {}).get("source")}
        log("[bench] all fast rows item by item: %.3f ms/step (stage 1 %.3f ms per call), same lists: %s" %
            (ms_s, stage_s[1], same))

    if not args.no_policy_leg:
        log("[bench] threshold policy of the paper: sampled thresholds with margin, search, operation counts")
        result["threshold_policy"] = policy_leg(torch, b, cfg, index, queries[:batch].contiguous(),
                                                (cap, out_ids, out_dist, surv, ws),
                                                max(3, args.steps // 2), not args.no_cpu_baseline, cb, codes)
        p = result["threshold_policy"]
        if "tiled_running" in p:
            t = p["tiled_running"]
            log("[bench] loop threshold per tile: tables + search %.3f ms, %.4f %% refined, ops ratio %.4f"
                % (t["ms_tables_search"], 100 * t["refined_frac"], t["ops_ratio"]))
        log("[bench] policy: thresholds %.3f ms, tables + policy + search %.3f ms, %.2f %% survive, ops ratio %.4f"
            % (p["ms_sample_thresholds"], p["ms_tables_policy_search"], 100 * p["survivors_frac"], p["ops_ratio"]))

    if not args.no_encode_leg:
        log("[bench] greedy encoding of vectors of the workload's shape")
        result["encode"] = encode_leg(torch, b, cfg, max(3, args.steps // 4))
        log("[bench] encode: %.3f ms for %d items, %.1f TFLOP/s; mean squared error %s; %d refinement sweeps %.3f ms" %
            (result["encode"]["ms"], result["encode"]["N"], result["encode"]["achieved"],
             result["encode"]["mean_sq_error"], result["encode"]["refine"]["sweeps"], result["encode"]["refine"]["ms"]))

    del ws, index, cb, codes, queries
    torch.cuda.empty_cache()
    result["machine_limits"] = machine_limits(torch, b)
    if not args.no_hbm_leg:
        log("[bench] stage-1 scan on the 400 MB fast-code array, one, two and four queries per pass")
        result["roofline_stage1_hbm"] = hbm_leg(torch, b, max(5, args.steps), args.warmup)
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle")
        base, match = cpu_baseline(cfg, thr.cpu().numpy(), gpu_ids, gpu_dist)
        result["cpu_baseline"] = base
        result["oracle_matched"] = match
    if not args.no_configs_leg:
        log("[bench] the other workload shapes, each against the oracle")
        result["configs"] = configs_leg(torch, b, synth, args.workload, not args.no_cpu_baseline)
        log("[bench] C3's shape over vectors encoded on the GPU")
        result["configs"]["C3_encoded"] = encoded_index_leg(torch, b, synth, not args.no_cpu_baseline)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
