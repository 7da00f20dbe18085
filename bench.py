#!/usr/bin/env python3
"""Benchmark of the filtered int8 top-K hot path on one MI355X.

One "step" is one pass of the whole path -- Bloom test, compaction, int8 scoring, rescale,
(multi-task aggregation,) per-workgroup candidate admission, selection/merge -- over one batch
of synthetic queries against the resident corpus.  Inputs are generated on the GPU and are
resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large|mid|tiny|multi|mfma]

The headline record is the Large workload (10 M items x d = 256, batch 256: the largest
memory-bound configuration).  Unless --no-others is given the same line also carries the Large
selectivity sweep, the all-distinct-filters variant and a compact record for each other workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_MFMA_PEAK_TOPS = 5000.0  # dense int8 MFMA, published


def union_and_rows(st, bloom, w):
    """Algorithmic-byte ingredients: signature rows each distinct filter touches, fraction of
    items passing at least one filter of the batch, passing pairs per query."""
    import torch
    fo = w.filt_offsets
    seen, filt = {}, []
    for b in range(w.cfg.batch):
        key = tuple(sorted(set(int(x) for x in w.filt_ids[fo[b]:fo[b + 1]])))
        if key not in seen:
            seen[key] = len(filt)
            filt.append(key)
    fid = np.array([x for f in filt for x in f], dtype=np.uint64)
    foff = np.concatenate([[0], np.cumsum([len(f) for f in filt])]).astype(np.int64)
    masks = st.st_bloom_mask(bloom, fid, foff)
    torch.cuda.synchronize()

    def popcount(t):
        return int(torch.from_numpy(np.unpackbits(t.cpu().numpy().view(np.uint8))).sum())

    union = masks[0].clone()
    for j in range(1, masks.shape[0]):
        union |= masks[j]
    per_filter = [popcount(masks[j]) for j in range(masks.shape[0])]
    rows = 0
    m, k = w.cfg.m_bits, w.cfg.k_hashes
    # signature rows a filter touches: k per term (an upper bound that is exact unless two of
    # a filter's k * terms hashes collide, which costs at most one 128-byte line per tile)
    for f in filt:
        rows += k * len(f)
    passing_pairs = 0
    for b in range(w.cfg.batch):
        key = tuple(sorted(set(int(x) for x in w.filt_ids[fo[b]:fo[b + 1]])))
        passing_pairs += per_filter[seen[key]]
    return {"distinct_filters": len(filt), "rows_touched": rows, "union_items": popcount(union),
            "passing_pairs": passing_pairs, "per_filter_sel": [p / max(w.cfg.n_items, 1) for p in per_filter]}


def union_and_rows_programs(st, bloom, w, prog):
    """The same ingredients for a batch whose filters are programs (ops, ids, offsets): signature
    rows read by the leaves of each distinct program, plus one mask row written and read per
    distinct program (counted as 2 rows each)."""
    import torch
    ops, ids, off = prog
    seen, progs, q2p = {}, [], []
    for b in range(w.cfg.batch):
        key = (tuple(ops[off[b]:off[b + 1]].tolist()), tuple(ids[off[b]:off[b + 1]].tolist()))
        if key not in seen:
            seen[key] = len(progs)
            progs.append(key)
        q2p.append(seen[key])
    p_ops = np.array([o for p in progs for o in p[0]], dtype=np.int32)
    p_ids = np.array([i for p in progs for i in p[1]], dtype=np.uint64)
    p_off = np.concatenate([[0], np.cumsum([len(p[0]) for p in progs])]).astype(np.int64)
    masks = st.st_bloom_mask_expr(bloom, p_ops, p_ids, p_off)
    torch.cuda.synchronize()

    def popcount(t):
        return int(torch.from_numpy(np.unpackbits(t.cpu().numpy().view(np.uint8))).sum())

    union = masks[0].clone()
    for j in range(1, masks.shape[0]):
        union |= masks[j]
    per = [popcount(masks[j]) for j in range(masks.shape[0])]
    rows = sum(w.cfg.k_hashes * sum(1 for o in p[0] if o == 0) + 2 for p in progs)
    return {"distinct_filters": len(progs), "rows_touched": rows, "union_items": popcount(union),
            "passing_pairs": sum(per[j] for j in q2p), "per_filter_sel": [p / max(w.cfg.n_items, 1) for p in per]}


def stats_ivf(st, bloom, w, prog, coff, probes, n_clusters):
    """Ingredients for the probing search: passing items per query = program mask AND probed
    ranges; bytes of phases 1-2 = centroid table and keys, signature rows over the probed words
    only, and the per-query mask rows (zeroed, then read by the scan)."""
    import torch
    cfg = w.cfg
    base = union_and_rows_programs(st, bloom, w, prog)  # per-program masks are recomputed below, cheaply
    ops, ids, off = prog
    seen, progs, q2p = {}, [], []
    for b in range(cfg.batch):
        key = (tuple(ops[off[b]:off[b + 1]].tolist()), tuple(ids[off[b]:off[b + 1]].tolist()))
        if key not in seen:
            seen[key] = len(progs)
            progs.append(key)
        q2p.append(seen[key])
    p_ops = np.array([o for p in progs for o in p[0]], dtype=np.int32)
    p_ids = np.array([i for p in progs for i in p[1]], dtype=np.uint64)
    p_off = np.concatenate([[0], np.cumsum([len(p[0]) for p in progs])]).astype(np.int64)
    masks = st.st_bloom_mask_expr(bloom, p_ops, p_ids, p_off)  # [E][n_words] int64
    shifts = torch.arange(64, device="cuda", dtype=torch.int64)
    cluster_of = torch.bucketize(torch.arange(cfg.n_items, device="cuda"), coff[1:], right=True).clamp_(max=n_clusters - 1)
    union = torch.zeros(cfg.n_items, dtype=torch.bool, device="cuda")
    passing_pairs, probed_words, leaf_row_words = 0, 0, 0
    sizes = (coff[1:] - coff[:-1])
    for b in range(cfg.batch):
        pr = probes[b][probes[b] >= 0].long()
        probed = torch.zeros(n_clusters, dtype=torch.bool, device="cuda")
        probed[pr] = True
        in_probe = probed[cluster_of]
        bits = ((masks[q2p[b]].unsqueeze(1) >> shifts) & 1).reshape(-1)[: cfg.n_items].bool()
        pb = bits & in_probe
        union |= pb
        passing_pairs += int(pb.sum())
        words_b = int(((sizes[pr] + 63) // 64 + 1).sum())
        probed_words += words_b
        leaf_row_words += words_b * cfg.k_hashes * sum(1 for o in progs[q2p[b]][0] if o == 0)
    n_words = (cfg.n_items + 63) // 64
    extra = n_clusters * (cfg.d + 4) + 2 * cfg.batch * n_clusters * 8 + leaf_row_words * 8 + 2 * cfg.batch * n_words * 8
    # Scratch memory of the filter stage per batch (the comparison of Sec. 6.2.3, Fig. 9): a full
    # filter pass first materialises one bit per item and query (filter-then-probe); filtering only
    # inside the probed clusters needs the probed words alone (probe-then-filter), and the
    # per-query kernel of this library keeps even those in LDS: what it touches in HBM beside the
    # index is the centroid keys, the probed ids and the keys of the passing items.
    scratch = {
        "filter_then_probe_mask_bytes": cfg.batch * n_words * 8,
        "probe_then_filter_mask_bytes": probed_words * 8,
        "per_query_kernel_hbm_scratch_bytes": cfg.batch * n_clusters * 8 + cfg.batch * len(probes[0]) * 4 + passing_pairs * 8,
        "mask_row_route_hbm_scratch_bytes": 2 * cfg.batch * ((cfg.n_items + 1023) // 1024) * 128 + cfg.batch * n_clusters * 8,
    }
    return {"distinct_filters": cfg.batch, "rows_touched": 0, "extra_bytes": extra, "union_items": int(union.sum()),
            "passing_pairs": passing_pairs, "per_filter_sel": base["per_filter_sel"],
            "probed_item_fraction": float(probed_words * 64) / max(cfg.n_items * cfg.batch, 1), "filter_scratch": scratch}


def quantize_bench(args, cfg, torch, st):
    """Publish-time quantisation of an fp32 [n_items, d] table: two passes (min / max, then codes),
    9 bytes per value of algorithmic traffic."""
    n, d = cfg.n_items, cfg.d
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20251114)
    x = torch.randn((n, d), generator=gen, device="cuda", dtype=torch.float32)
    q = torch.empty((n, d), dtype=torch.int8, device="cuda")
    rs = torch.empty(n, dtype=torch.float32, device="cuda")
    mm = torch.empty(2, dtype=torch.float32, device="cuda")
    scratch = torch.empty(2, dtype=torch.int32, device="cuda")
    import ctypes as C
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def step():
        rc = st.lib().st_quantize_global(C.c_void_p(x.data_ptr()), n, d, C.c_void_p(q.data_ptr()), C.c_void_p(rs.data_ptr()),
                                         C.c_void_p(mm.data_ptr()), C.c_void_p(scratch.data_ptr()), stream)
        if rc != 0:
            raise RuntimeError(st.last_error())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    st.st_timing_begin(args.steps * 2 + 8)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    k_ms = st.st_timing_end()["scan"][0] / args.steps
    a_bytes = 9 * n * d + 4 * n
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import st_oracle as O
        n_s = min(n, 2_000_000)
        xs = x[:n_s].cpu().numpy()
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 100:
            t0 = time.perf_counter()
            O.quantize_global(xs)
            spent += time.perf_counter() - t0
            reps += 1
        cpu = {"value": n_s / (spent / reps), "unit": "items/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n_s} rows, {reps} repetitions, {spent:.1f} s"}
    print(json.dumps({
        "metric": "int8 quantisation items/sec", "value": n / (ms * 1e-3), "unit": "items/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name + "+quantize", "n_items": n, "d": d},
        "roofline": {"bound": "hbm", "achieved": a_bytes / (k_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": a_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "quant_minmax + quant_apply", "kernel_ms_per_step": k_ms,
                     "algorithmic_bytes_per_step": a_bytes},
        "cpu_baseline": cpu}))


def value_model_bench(args, cfg, torch, st):
    """A formula with a condition over four task scores per item: if s2 > 0.5 then
    0.4*s0 + 0.3*s1 + 0.2*s2 + 0.1*s3 else min(s0, s1) * 0.5.  20 bytes per item."""
    n, T = cfg.n_items, 4
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20251114)
    scores = torch.rand((n, T), generator=gen, device="cuda", dtype=torch.float32)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    TASK = lambda t: 0 | (t << 8)
    prog = [(TASK(2), 0), (1, 0.5), (7, 0),
            (1, 0.4), (TASK(0), 0), (4, 0), (1, 0.3), (TASK(1), 0), (4, 0), (2, 0), (1, 0.2), (TASK(2), 0), (4, 0), (2, 0),
            (1, 0.1), (TASK(3), 0), (4, 0), (2, 0),
            (TASK(0), 0), (TASK(1), 0), (5, 0), (1, 0.5), (4, 0), (8, 0)]
    ops = [p[0] for p in prog]
    consts = [float(p[1]) for p in prog]

    def step():
        st.st_value_model(scores, ops, consts, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    st.st_timing_begin(args.steps + 8)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    k_ms = st.st_timing_end()["scan"][0] / args.steps
    a_bytes = n * (4 * T + 4)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import st_oracle as O
        n_s = min(n, 2_000_000)
        xs = scores[:n_s].cpu().numpy()
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 100:
            t0 = time.perf_counter()
            O.value_model(xs, ops, consts)
            spent += time.perf_counter() - t0
            reps += 1
        cpu = {"value": n_s / (spent / reps), "unit": "items/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n_s} items, {reps} repetitions, {spent:.1f} s"}
    print(json.dumps({
        "metric": "value model items/sec", "value": n / (ms * 1e-3), "unit": "items/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name + "+value-model", "n_items": n, "n_tasks": T, "formula_entries": len(ops)},
        "roofline": {"bound": "hbm", "achieved": a_bytes / (k_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": a_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "value_model", "kernel_ms_per_step": k_ms, "algorithmic_bytes_per_step": a_bytes},
        "cpu_baseline": cpu}))


def measured_read_peak(torch, st, gib: float = 4.0, reps: int = 10):
    """Practical HBM read ceiling: the library's streaming-read kernel over a buffer far larger
    than the caches, best of `reps` launches at the best of three launch shapes (two workgroups
    per compute unit measured fastest: 6.3 TB/s; HIP events on the launch stream)."""
    n = int(gib * (1 << 30))
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    best = None
    for wgs in (256, 512, 65536):
        sink = torch.empty(wgs, dtype=torch.int32, device="cuda")
        for _ in range(2):
            st.st_stream_read(src, sink, wgs)
        torch.cuda.synchronize()
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            st.st_stream_read(src, sink, wgs)
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
    del src, sink
    return n / (best * 1e-3) / 1e9


def measure_search(args, torch, st, w, bloom, buf=None, prog=None, ivf=None, ivf_tensors=None, mfma_bound=False,
                   traffic=None, read_peak=None):
    """Times one workload: W warm-up steps, K steps bracketed by synchronisations (the contract's
    ms_per_step), the same K steps again with a pair of HIP events around each (median / min) and
    once more with events around every kernel (per-kernel durations); then the algorithmic bytes
    and operations of a step.  Returns the record's pieces."""
    cfg = w.cfg
    T = max(cfg.n_tasks, 1)
    if buf is None:
        if ivf:
            buf = st.IvfBuffers(cfg.n_items, cfg.d, cfg.batch, cfg.top_k, ivf[0], ivf[1], int(prog[2][-1]))
        else:
            buf = st.SearchBuffers(cfg.n_items, cfg.d, cfg.batch, T, cfg.top_k,
                                   n_expr_entries=None if prog is None else int(prog[2][-1]))

    def step():
        if ivf:
            cent, cscale, coff = ivf_tensors
            st.st_search_ivf(bloom, w.items, w.item_scale, cent, cscale, coff, ivf[1], w.queries, w.query_scale,
                             prog[0], prog[1], prog[2], cfg.top_k, buffers=buf)
        elif prog is not None:
            st.st_search_expr(bloom, w.items, w.item_scale, w.queries, w.query_scale, prog[0], prog[1], prog[2],
                              cfg.top_k, task_weight=w.task_weight, buffers=buf)
        elif cfg.n_tasks > 0:
            st.st_search_multitask(bloom, w.items, w.item_scale, w.queries, w.query_scale, w.task_weight,
                                   w.filt_ids, w.filt_offsets, cfg.top_k, buffers=buf)
        else:
            st.st_search(bloom, w.items, w.item_scale, w.queries, w.query_scale, w.filt_ids,
                         w.filt_offsets, cfg.top_k, buffers=buf)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-step durations on the GPU's clock (events on the launch stream around each call)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per = np.array([e0.elapsed_time(e1) for e0, e1 in evs])

    # host time of one call with the GPU idle: what the calling thread spends before the call returns
    host = []
    for _ in range(min(args.steps, 20)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        host.append((time.perf_counter() - t0) * 1e6)
    torch.cuda.synchronize()

    # per-kernel durations, HIP events on the launch stream around every kernel of K more steps
    plan_levels, _, _ = st.st_search_plan(cfg.n_items, cfg.batch * T, cfg.top_k)
    st.st_timing_begin(args.steps * 3 * (len(plan_levels) + 6) + 8)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    timing = st.st_timing_end()
    scan_ms, scan_n = timing["scan"]
    scan_ms_per_step = scan_ms / args.steps
    n_levels = timing["select"][1] // args.steps  # one selection (or seed) launch per level

    if ivf:
        stats = stats_ivf(st, bloom, w, prog, ivf_tensors[2], buf.probes, ivf[0])
    else:
        stats = union_and_rows(st, bloom, w) if prog is None else union_and_rows_programs(st, bloom, w, prog)
    n_words = (cfg.n_items + 63) // 64
    a_bytes = (stats["rows_touched"] * n_words * 8 + stats["union_items"] * (cfg.d + 4)
               + cfg.batch * T * cfg.d + cfg.batch * cfg.top_k * 12 + stats.get("extra_bytes", 0))
    a_ops = 2.0 * cfg.d * T * stats["passing_pairs"]
    stream_all = cfg.n_items * (cfg.d + 4) + cfg.n_items * cfg.m_bits // 8
    kern_s = scan_ms_per_step * 1e-3
    step_s = ms_per_step * 1e-3
    if mfma_bound:
        ach, ach_step, peak, unit, bound = a_ops / kern_s / 1e12, a_ops / step_s / 1e12, INT8_MFMA_PEAK_TOPS, "TOP/s", "mfma"
    else:
        ach, ach_step, peak, unit, bound = a_bytes / kern_s / 1e9, a_bytes / step_s / 1e9, HBM_PEAK_GBS, "GB/s", "hbm"
    roofline = {
        "bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
        # the whole step (every launch and the gaps between them) against the same peak
        "achieved_step": ach_step, "frac_step": ach_step / peak,
        "traffic": traffic,
        "traffic_source": None if traffic is None else "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                                                       "earlier run of this command; not measured in this run)",
        "kernel": "scan (all of its launches of one step)", "kernel_ms_per_step": scan_ms_per_step,
        "kernel_launches_per_step": scan_n / args.steps,
        "algorithmic_bytes_per_step": a_bytes, "stream_all_bytes_per_step": stream_all,
        "stream_all_GBs": stream_all / kern_s / 1e9 if kern_s > 0 else 0.0,
        "algorithmic_ops_per_step": a_ops,
        "select_ms_per_step": timing["select"][0] / args.steps,
        "rescue_ms_per_step": timing["rescue"][0] / args.steps,
        "filter_expr_ms_per_step": timing["expr"][0] / args.steps,
    }
    if read_peak and not mfma_bound:
        roofline.update({"measured_peak": read_peak, "frac_of_measured": ach / read_peak,
                         "frac_step_of_measured": ach_step / read_peak})
    elif read_peak:
        roofline.update({"measured_peak": read_peak,
                         "hbm_frac_of_measured": a_bytes / kern_s / 1e9 / read_peak})
    rec = {
        "value": cfg.batch / step_s, "ms_per_step": ms_per_step,
        "step_ms": {"mean": float(per.mean()), "median": float(np.median(per)), "min": float(per.min())},
        "host_us_per_call": float(np.median(host)),
        "levels": n_levels, "stats": stats, "roofline": roofline,
    }
    return rec, buf


def config_block(cfg, rec, args, extra=None):
    stats = rec["stats"]
    out = {"workload": cfg.name, "n_items": cfg.n_items, "d": cfg.d, "batch": cfg.batch,
           "n_tasks": cfg.n_tasks, "m_bits": cfg.m_bits, "k_hashes": cfg.k_hashes,
           "filter_terms": cfg.n_terms, "top_k": cfg.top_k, "levels": rec["levels"],
           "scoring_path": args.path, "distinct_filters": stats["distinct_filters"],
           "union_selectivity": stats["union_items"] / max(cfg.n_items, 1),
           "mean_filter_selectivity": float(np.mean(stats["per_filter_sel"]))}
    if extra:
        out.update(extra)
    return out


def brief(cfg, rec, args):
    """Compact sub-record of a workload that is not the headline."""
    r = rec["roofline"]
    out = {"config": config_block(cfg, rec, args), "value": rec["value"], "unit": "queries/s",
           "ms_per_step": rec["ms_per_step"], "step_ms": rec["step_ms"], "host_us_per_call": rec["host_us_per_call"],
           "roofline": {k: r[k] for k in ("bound", "achieved", "peak", "unit", "frac", "achieved_step", "frac_step",
                                          "kernel_ms_per_step", "kernel_launches_per_step", "select_ms_per_step",
                                          "algorithmic_bytes_per_step", "algorithmic_ops_per_step", "traffic")}}
    for k in ("measured_peak", "frac_of_measured", "frac_step_of_measured", "hbm_frac_of_measured"):
        if k in r:
            out["roofline"][k] = r[k]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="large",
                    help="workload of the headline record: large (default: the largest memory-bound "
                         "configuration), mid, tiny, multi, mfma")
    ap.add_argument("--selectivity", type=float, default=0.0,
                    help="variant of the workload: filters chosen for this exact-set selectivity instead of the "
                         "recipe's (Large sweeps 0.001 .. the broadest available, 1.0); own workload name")
    ap.add_argument("--no-others", action="store_true",
                    help="only the headline workload: no sub-records for the other configurations, the Large "
                         "selectivity sweep and the all-distinct-filters variant")
    ap.add_argument("--path", type=int, default=0, help="0 auto, 1 wavefront dot, 2 MFMA")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--distinct-filters", action="store_true",
                    help="stress variant of the workload: the filter pool is as large as the batch, so "
                         "(almost) every query carries its own filter; reported as its own workload name")
    ap.add_argument("--filter-programs", action="store_true",
                    help="variant of the workload: every query's filter is a boolean program of the "
                         "paper's query form (a term AND an OR-group, every second one AND NOT a term), run "
                         "through st_search_expr; reported as its own workload name")
    ap.add_argument("--quantize", action="store_true",
                    help="time the publish-time int8 quantisation (st_quantize_global) of an fp32 table of the "
                         "workload's shape instead of the search; prints its own JSON line")
    ap.add_argument("--value-model", action="store_true",
                    help="time a Value Model formula (st_value_model) over n_items x 4 task scores instead of the "
                         "search; prints its own JSON line")
    ap.add_argument("--batch", type=int, default=0,
                    help="variant of the workload: another batch size (the paper's ANN runs use 16); "
                         "reported as its own workload name")
    ap.add_argument("--top-k", type=int, default=0,
                    help="variant of the workload: another K (the paper's pre-filter sizes are O(10,000)); "
                         "reported as its own workload name")
    ap.add_argument("--ivf", default="",
                    help="variant of the workload: N_CLUSTERS:N_PROBE, e.g. 1024:64 -- the corpus cut into "
                         "clusters, every query probes its N_PROBE best ones (st_search_ivf) with the filter "
                         "programs of --filter-programs; single-task workloads only")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy, as the known-size reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2511_14881_amd import binding as st
    from paper_2511_14881_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    st.lib()  # fail loudly if the HIP library is missing
    cfg = synth.CONFIGS[args.config]
    if args.quantize:
        quantize_bench(args, cfg, torch, st)
        return
    if args.value_model:
        value_model_bench(args, cfg, torch, st)
        return
    variant = bool(args.distinct_filters or args.filter_programs or args.top_k > 0 or args.batch > 0 or args.ivf
                   or args.selectivity > 0)
    if args.distinct_filters:
        cfg = synth.scaled(cfg, cfg.n_items, pool=cfg.batch, name=cfg.name + "+distinct-filters")
    if args.selectivity > 0:
        cfg = synth.scaled(cfg, cfg.n_items, target_sel=args.selectivity, name=cfg.name + "+sel%g" % args.selectivity)
    if args.top_k > 0:
        cfg = synth.scaled(cfg, cfg.n_items, top_k=args.top_k, name=cfg.name + "+K%d" % args.top_k)
    if args.batch > 0:
        cfg = synth.scaled(cfg, cfg.n_items, batch=args.batch, pool=min(cfg.pool, args.batch), name=cfg.name + "+B%d" % args.batch)
    ivf = None
    if args.ivf:
        ivf = tuple(int(x) for x in args.ivf.split(":"))
        if len(ivf) != 2:
            print("bench.py: --ivf takes N_CLUSTERS:N_PROBE", file=sys.stderr)
            sys.exit(2)
        args.filter_programs = True
        # a multi-task workload probes with every task embedding as a query of its own (Sec. 5.2:
        # the tasks of a request are batched against the one index and return task-specific lists)
        cfg = synth.scaled(cfg, cfg.n_items, name=cfg.name + "+ivf%d:%d" % ivf + ("+task-lists" if cfg.n_tasks > 0 else ""))
    elif args.filter_programs:
        cfg = synth.scaled(cfg, cfg.n_items, name=cfg.name + "+filter-programs")
    others = not (args.no_others or variant)

    read_peak = measured_read_peak(torch, st)

    t0 = time.time()
    w = synth.make_workload(cfg, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    T = max(cfg.n_tasks, 1)

    t0 = time.time()
    bloom = st.st_bloom_build(w.feat_offsets, w.feat_ids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
    torch.cuda.synchronize()
    build_first_s = time.time() - t0
    # steady state: the same build again (the first call also sets the library up on the device)
    build_s = build_first_s
    for _ in range(3):
        t0 = time.time()
        b2 = st.st_bloom_build(w.feat_offsets, w.feat_ids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
        torch.cuda.synchronize()
        build_s = min(build_s, time.time() - t0)
        b2.free()
        del b2
    prog = None
    if args.filter_programs:
        prog = synth.gen_filter_programs(cfg)[:3]
    if ivf and cfg.n_tasks > 0:
        w, prog = synth.flatten_tasks(w, prog)
        cfg = w.cfg
        T = 1
    ivf_tensors = synth.gen_clusters(cfg, ivf[0], device="cuda") if ivf else None
    st.st_set_scoring_path(args.path)

    if args.copy_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def traffic_of(name, is_variant):
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if is_variant or not os.path.exists(tpath):
            return None
        try:
            return json.load(open(tpath)).get(name)
        except Exception:
            return None

    rec, buf = measure_search(args, torch, st, w, bloom, prog=prog, ivf=ivf, ivf_tensors=ivf_tensors,
                              mfma_bound=args.config == "mfma", traffic=traffic_of(args.config, variant),
                              read_peak=read_peak)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import st_oracle as O
        # bounded sample of the same workload: a prefix of the corpus and of the batch
        n_s = min(cfg.n_items, 1_000_000)
        b_s = min(cfg.batch, 64)
        items = w.items[:n_s].cpu().numpy()
        isc = w.item_scale[:n_s].cpu().numpy()
        off = w.feat_offsets[: n_s + 1].cpu().numpy()
        ids = w.feat_ids[: int(off[-1])].cpu().numpy().view(np.uint64)
        q = w.queries[:b_s].cpu().numpy()
        qs = w.query_scale[:b_s].cpu().numpy()
        fo = w.filt_offsets[: b_s + 1]
        fi = w.filt_ids[: int(fo[-1])]
        sigs = O.bloom_build(off, ids, cfg.m_bits, cfg.k_hashes)
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 1000:
            t0 = time.perf_counter()
            if ivf:
                cent, cscale, coff = ivf_tensors
                po = prog[2][: b_s + 1]
                O.search_ivf(sigs, cfg.m_bits, cfg.k_hashes, items, isc, cent.cpu().numpy(), cscale.cpu().numpy(),
                             np.minimum(coff.cpu().numpy(), n_s), ivf[1], q, qs, prog[0][: int(po[-1])],
                             prog[1][: int(po[-1])], po, cfg.top_k)
            elif prog is not None:
                po = prog[2][: b_s + 1]
                O.search_expr(sigs, cfg.m_bits, cfg.k_hashes, items, isc, q, qs, prog[0][: int(po[-1])],
                              prog[1][: int(po[-1])], po, cfg.top_k, task_weight=w.task_weight)
            else:
                O.search(sigs, cfg.m_bits, cfg.k_hashes, items, isc, q, qs, fi, fo, cfg.top_k,
                         task_weight=w.task_weight)
            spent += time.perf_counter() - t0
            reps += 1
        per_batch = spent / reps
        # queries/s on the sample corpus, scaled to the full corpus size (work is linear in N)
        qps = b_s / per_batch * (n_s / cfg.n_items)
        cpu = {"value": qps, "unit": "queries/s", "cores": O.num_threads(), "kind": "oracle",
               "sample": f"{b_s} queries x first {n_s} items, {reps} repetitions, {spent:.1f} s; "
                         f"scaled by {n_s}/{cfg.n_items} to the full corpus"}
        del items, isc, off, ids, sigs

    out = {
        "metric": "filtered int8 top-K queries/sec", "value": rec["value"], "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": config_block(cfg, rec, args, {"probed_item_fraction": rec["stats"]["probed_item_fraction"],
                                                "filter_scratch": rec["stats"]["filter_scratch"]} if ivf else None),
        "step_ms": rec["step_ms"], "host_us_per_call": rec["host_us_per_call"],
        "items_scanned_per_s": cfg.n_items / (rec["ms_per_step"] * 1e-3),
        "item_query_pairs_per_s": cfg.n_items * cfg.batch / (rec["ms_per_step"] * 1e-3),
        "bloom_build_items_per_s": cfg.n_items / build_s if build_s > 0 else None,
        "bloom_build_first_call_items_per_s": cfg.n_items / build_first_s if build_first_s > 0 else None,
        "gen_seconds": gen_s,
        "roofline": rec["roofline"],
        "cpu_baseline": cpu,
    }

    if others:
        # the same corpus with every query carrying its own filter (no work shared between queries)
        cfg_d = synth.scaled(cfg, cfg.n_items, pool=cfg.batch, name=cfg.name + "+distinct-filters")
        sample = w.feat_ids[: min(cfg.n_items, 200_000) * cfg.feats_per_item].cpu().numpy()
        pool_d = synth.choose_filter_pool(cfg_d, sample)
        fid_d, foff_d = synth.gen_filters(cfg_d, pool_d)
        wd = synth.Workload(cfg_d, w.items, w.item_scale, w.feat_offsets, w.feat_ids, w.queries, w.query_scale,
                            w.task_weight, fid_d, foff_d, pool_d)
        rec_d, _ = measure_search(args, torch, st, wd, bloom, buf=buf, read_peak=read_peak)
        out["distinct_filters_variant"] = brief(cfg_d, rec_d, args)
        if args.config == "large":
            sweep = []
            for target in synth.LARGE_SWEEP:
                ws = synth.refilter(w, target)
                rec_s, _ = measure_search(args, torch, st, ws, bloom, buf=buf, read_peak=read_peak)
                b = brief(ws.cfg, rec_s, args)
                b["target_selectivity"] = target
                sweep.append(b)
            out["selectivity_sweep"] = sweep
        del w, bloom, buf, wd
        torch.cuda.empty_cache()
        subs = {}
        for name in ("tiny", "mid", "multi", "mfma", "large"):
            if name == args.config:
                continue
            c2 = synth.CONFIGS[name]
            w2 = synth.make_workload(c2, device="cuda")
            bl2 = st.st_bloom_build(w2.feat_offsets, w2.feat_ids, c2.n_items, c2.m_bits, c2.k_hashes)
            rec2, _ = measure_search(args, torch, st, w2, bl2, mfma_bound=name == "mfma",
                                     traffic=traffic_of(name, False), read_peak=read_peak)
            subs[name] = brief(c2, rec2, args)
            bl2.free()
            del w2, bl2
            torch.cuda.empty_cache()
        out["other_configs"] = subs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
