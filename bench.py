#!/usr/bin/env python3
"""Throughput of the Proximity-FLAT retrieval step on one MI355X.

A step is one proximity_search_batch call (cache probe, resolver, corpus scan
for the misses, top-k, routing) on one batch of the seeded synthetic stream.
The default workload is the 1 M x 768 float32 corpus with the Zipf(1.1) query
stream, capacity 300, LRU, k = 10, tau = 0.25, one query per call.

Prints one JSON line: whole-job queries/s, the roofline of the dominant kernel
(the streaming corpus-scan distance kernel, timed with HIP events inside the
library on the call's stream) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
F32_MFMA_PEAK_TFLOPS = 157.3   # MI355X dense float32 matrix, published
BF16_MFMA_PEAK_TFLOPS = 2500.0 # MI355X dense bfloat16 matrix, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed search_batch calls")
    ap.add_argument("--warmup", type=int, default=None, help="untimed calls before them")
    ap.add_argument("--workload", default="mid", choices=["tiny", "mid", "large", "lowreuse", "probe"],
                    help="mid is the headline workload; the others are the remaining benchmark configurations")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--rho", type=int, default=1,
                    help="re-ranking factor (Section 3.3.4): rho*k neighbours stored per key, hits re-ranked")
    ap.add_argument("--metric", default="l2", choices=["l2", "ip", "cosine"],
                    help="the index's distance function (Section 2.2).  The workloads' tolerances are Euclidean; "
                         "for cosine the run uses tau^2/2, the cosine distance of unit vectors that far apart")
    ap.add_argument("--lsh-bits", type=int, default=0,
                    help="bucketed cache (Section 3.2): 2^L buckets; 0 = the flat cache")
    ap.add_argument("--bucket-capacity", type=int, default=20, help="entries per bucket when --lsh-bits > 0")
    ap.add_argument("--n-docs", type=int, default=None, help="override corpus rows (debugging only)")
    ap.add_argument("--exact-scan", action="store_true",
                    help="never pre-rank on rounded operands (PROXIMITY_FLAG_NO_ROUNDED_SCAN): the scan that "
                         "multiplies the corpus as it is stored")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=24, help="queries the oracle is timed on")
    ap.add_argument("--recall-sweep", action="store_true",
                    help="hit rate and database k-recall (Section 4) over tau, flat and bucketed cache, then exit")
    ap.add_argument("--probe-scaling", action="store_true",
                    help="cache lookup time against the number of cached keys, flat and bucketed (Section 4.4), then exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for HBM byte counters)")
    return ap.parse_args()


def run_region(px, q_dev, tau, batch, first, n_calls, outs):
    """Issue n_calls calls on consecutive batches starting at row `first`."""
    ids, dists, hit = outs
    for c in range(n_calls):
        r0 = first + c * batch
        px.search_batch(q_dev[r0:r0 + batch], tau, ids[r0:r0 + batch], dists[r0:r0 + batch], hit[r0:r0 + batch])


PREROLL_BATCH = 64


def preroll(px, q_dev, tau, rows, outs):
    """Untimed: the first `rows` rows of the stream (a multiple of 64) go through the cache in calls of 64, so
    that the timed calls meet the cache in the state the workload keeps it in (capacity full, steady hit
    rate) however few of them there are.  Any split of a stream into calls leaves the same cache."""
    run_region(px, q_dev, tau, PREROLL_BATCH, 0, rows // PREROLL_BATCH, outs)


def timed_run(torch, px, q_dev, tau, batch, warmup, steps, outs, device, preroll_rows=0):
    """Clears the cache, replays preroll_rows untimed, then `warmup` untimed and `steps` timed calls of `batch`
    rows on the rows that follow.  Returns seconds, hit rate of the timed rows, first timed row."""
    px.clear()
    preroll(px, q_dev, tau, preroll_rows, outs)
    first = preroll_rows // batch          # in calls of `batch` rows
    run_region(px, q_dev, tau, batch, first * batch, warmup, outs)
    torch.cuda.synchronize(device)
    t0 = time.perf_counter()
    run_region(px, q_dev, tau, batch, (first + warmup) * batch, steps, outs)
    torch.cuda.synchronize(device)
    dt = time.perf_counter() - t0
    r0 = (first + warmup) * batch
    hit = outs[2][r0:r0 + steps * batch]
    return dt, float(hit.float().mean().item()), r0


def profiled_scan(torch, px, q_dev, tau, batch, first_call, n_calls, outs, device):
    """Re-run a stretch with per-launch HIP-event timing of the scan distance kernel."""
    px.profile_start()
    run_region(px, q_dev, tau, batch, first_call * batch, n_calls, outs)
    rec = px.profile_stop()
    hit = outs[2].cpu().numpy()
    busy = []
    for call, first_query, n_q, ms in rec:
        r0 = (first_call + call) * batch
        misses = int((hit[r0:r0 + batch] == 0).sum())
        if misses > first_query:
            busy.append((ms, min(n_q, misses - first_query)))
    return busy


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/*.md), scaled by what the
# same counters read for a 1 GiB copy (FETCH_SIZE: 2 KiB per count, WRITE_SIZE: 1 KiB per count).
# Keyed by (kernel, query-tile shape, corpus rows, dim, element bytes); anything else reports null.
COUNTER_TRAFFIC = {
    ("scan_regq_kernel (scores only)", 0, 1_000_000, 768, 4):
        {"fetch_bytes": 1_512_366 * 2048, "write_bytes": 3_906 * 1024, "source": "profiles/scan_regq_mid_b1.md"},
    ("scan_regq_kernel (rounded operands)", 64, 1_000_000, 768, 4):
        {"fetch_bytes": 1_513_890 * 2048, "write_bytes": 8_473 * 1024, "source": "profiles/scan_regq_mid_b64.md"},
    ("scan_regq_kernel", 64, 1_000_000, 768, 4):
        {"fetch_bytes": 1_514_328 * 2048, "write_bytes": 4_203 * 1024,
         "source": "profiles/scan_regq_mid_b64_exact.md"},
    ("scan_regq_kernel (one plane)", 128, 8_000_000, 384, 2):
        {"fetch_bytes": 3_029_002 * 2048, "write_bytes": 52_286 * 1024,
         "source": "profiles/scan_regq_lowreuse_b128.md"},
    ("scan_regq_kernel (rounded operands)", 64, 24_000_000, 768, 4):
        {"fetch_bytes": 36_058_895 * 2048, "write_bytes": 16_415 * 1024,
         "source": "profiles/scan_regq_large_b256.md"},
}


def scan_roofline(busy, n_docs, dim, batch, elem_bytes=4, one_plane=False):
    """Roofline entry from (duration ms, queries served) of the launches that streamed the corpus.
    `one_plane`: the instance's batched scans ran on rounded operands -- the first bfloat16 plane of the queries,
    and float32 rows rounded to bfloat16 on their way into the matrix instruction (its stats say so)."""
    if not busy:
        return None
    bytes_per_launch = n_docs * dim * elem_bytes + n_docs * 4      # corpus rows + their norms, read once
    avg_ms = sum(ms for ms, _ in busy) / len(busy)
    avg_q = sum(q for _, q in busy) / len(busy)
    gbs = bytes_per_launch / (avg_ms * 1e-3) / 1e9
    tflops = sum(2.0 * q * n_docs * dim for _, q in busy) / (sum(ms for ms, _ in busy) * 1e-3) / 1e12
    # A bfloat16 corpus is scanned on the bfloat16 matrix cores with the float32 queries split into bfloat16
    # terms: one multiply-add of that type per term of the split and of the inner product.  The scan with the
    # queries resident in registers (the dimensions it is built for) multiplies two terms -- one while its
    # exactness checks keep passing with the rounded queries --, the general one three.
    regq = batch > 4 and ((elem_bytes == 4 and dim in (768, 384)) or (elem_bytes == 2 and dim in (384, 256)))
    one_plane = one_plane and regq
    bf16_split = (elem_bytes == 2 and dim >= 64 and batch > 4) or one_plane     # multiplied on the bfloat16 matrix cores
    mfma_peak = BF16_MFMA_PEAK_TFLOPS if bf16_split else F32_MFMA_PEAK_TFLOPS
    per_term = (1.0 if one_plane else 2.0 if regq else 3.0) if bf16_split else 1.0
    ridge_q = mfma_peak * 1e12 / (HBM_PEAK_GBS * 1e9) * elem_bytes / (2 * per_term)  # queries per launch at the ridge
    if batch <= 4:
        # single-query calls: the register-resident kernel in its scores-only form on long float32 corpora of the
        # dimensions it is built for, the register-load streaming kernel otherwise
        dump = elem_bytes == 4 and dim in (768, 384) and n_docs >= 500_000
        kernel = "scan_regq_kernel (scores only)" if dump else "scores_stream_kernel"
    elif regq:
        kernel = "scan_regq_kernel" if not one_plane else \
            "scan_regq_kernel (one plane)" if elem_bytes == 2 else "scan_regq_kernel (rounded operands)"
    elif bf16_split:
        kernel = "scan_bf16x3_kernel"
    else:
        kernel = "scan_mfma_dma_kernel" if elem_bytes == 4 and dim >= 64 else "scan_mfma_topk_kernel"
    tile = 0 if batch <= 4 else (32 if avg_q <= 32 else 64 if avg_q <= 64 else 128)
    if one_plane and elem_bytes == 4:
        tile = 128 if avg_q > 64 else 64        # (the counters were taken on launches of these shapes)
    counted = COUNTER_TRAFFIC.get((kernel, tile, n_docs, dim, elem_bytes))
    if counted is not None:
        counted = dict(counted, measured_in_this_run=False,
                       note="HBM bytes per launch from the rocprofv3 --pmc runs summarised in `source`; not re-measured here")
    common = {"traffic": None if counted is None else counted["fetch_bytes"] + counted["write_bytes"],
              "traffic_counters": counted, "kernel": kernel,
              "launches_timed": len(busy), "avg_launch_ms": round(avg_ms, 5),
              "queries_per_launch_avg": round(avg_q, 3), "achieved_GBps": round(gbs, 1),
              "achieved_TFLOPs": round(tflops * per_term, 2), "algorithmic_bytes_per_launch": bytes_per_launch,
              "algorithmic_flops_per_launch_avg": 2.0 * per_term * avg_q * n_docs * dim,
              "float32_equivalent_TFLOPs": round(tflops, 2)}
    if avg_q < ridge_q:
        return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), **common}
    return {"bound": "mfma", "achieved": round(tflops * per_term, 2), "peak": mfma_peak, "unit": "TFLOP/s",
            "frac": round(tflops * per_term / mfma_peak, 4),
            "mfma_dtype": (f"bf16, {int(per_term)} term(s) of the query split, f32 accumulate") if bf16_split else "f32", **common}


def k_recall_per_query(ids, truth):
    """Database k-recall of Section 4, per query: the fraction of the k documents handed out (`ids`, [n][k]) that
    are among the k the index itself returns for that query (`truth`, [n][k]).  Padding ids (-1) count as
    documents that were not found.  Tensor arithmetic on whatever device the arguments live on."""
    found = (ids[:, :, None] == truth[:, None, :]) & (ids[:, :, None] >= 0)
    return found.any(dim=2).float().mean(dim=1)


def recall_sweep_rows(torch, W, Proximity, device, w, corpus_dev, q_dev, batch, rho, lsh_bits, bucket_capacity, taus):
    """Hit rate and database k-recall for every tolerance in `taus`, flat and bucketed cache, re-ranking factor 1
    and `rho`.  The index's own answers come from the library's plain search (proximity_knn_batch); the overlap
    is counted here, outside the method."""
    n_q = q_dev.shape[0]
    truth = torch.empty((n_q, w.k), dtype=torch.int64, device=device)
    plain = Proximity(corpus_dev, w.dim, 0, w.k, w.policy, batch)
    for r0 in range(0, n_q, batch):
        plain.knn_batch(q_dev[r0:r0 + batch], out_ids=truth[r0:r0 + batch])
    plain.close()
    rows = []
    planes = torch.from_numpy(W.lsh_planes(lsh_bits, w.dim, w.seed)).to(device)
    caches = (("flat", w.capacity, None), (f"bucketed {1 << lsh_bits}x{bucket_capacity}", bucket_capacity, planes))
    for name, cap, pl in caches:
        for r in sorted({1, rho}):
            px = Proximity(corpus_dev, w.dim, cap, w.k, w.policy, batch, rerank_factor=r, lsh_planes=pl)
            for tau in taus:
                px.clear()
                ids = torch.empty((n_q, w.k), dtype=torch.int64, device=device)
                hit = torch.empty((n_q,), dtype=torch.uint8, device=device)
                torch.cuda.synchronize(device)
                t0 = time.perf_counter()
                for r0 in range(0, n_q, batch):
                    px.search_batch(q_dev[r0:r0 + batch], tau, out_ids=ids[r0:r0 + batch], out_hit=hit[r0:r0 + batch],
                                    want_dists=False)
                torch.cuda.synchronize(device)
                dt = time.perf_counter() - t0
                same = k_recall_per_query(ids, truth)
                hits = hit.bool()
                rows.append({"cache": name, "rerank_factor": r, "tau": tau,
                             "hit_rate": round(float(hits.float().mean()), 4),
                             "k_recall": round(float(same.mean()), 4),
                             "k_recall_on_hits": round(float(same[hits].mean()), 4) if bool(hits.any()) else None,
                             "queries_per_s": round(n_q / dt, 1)})
            px.close()
    return rows


def recall_sweep(args, torch, np, W, Proximity, device):
    """Hit rate and database k-recall as Section 4 defines it: the fraction of the k documents the cache
    hands out that are among the k the index returns for the same query."""
    w = W.WORKLOADS[args.workload]
    batch = 64 if args.batch is None else args.batch
    n_q = (args.steps if args.steps is not None else 200) * batch
    corpus_dev = torch.from_numpy(W.corpus_for(w, args.n_docs)).to(device)
    q_dev = torch.from_numpy(W.stream_for(w, n_q)).to(device)
    bits = args.lsh_bits if args.lsh_bits > 0 else 4
    rows = recall_sweep_rows(torch, W, Proximity, device, w, corpus_dev, q_dev, batch, args.rho, bits,
                             args.bucket_capacity, w.taus or (0.0, 0.1, 0.25, 0.5, 1.0))
    print(json.dumps({"metric": "database_k_recall_sweep", "unit": "fraction", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": w.name, "queries": n_q, "batch": batch, "k": w.k}, "rows": rows}))


def probe_scaling(args, torch, np, W, Proximity, device):
    """Lookup time of the cache alone (no corpus) as the number of cached keys grows: the flat cache compares
    a query with every key, the bucketed one with one bucket of 20 (Section 3.2's cost argument, Section 4.4's
    measurement).  Per size: fill the cache with fresh unit vectors, then time calls of 1 and of 1 024 fresh
    queries at a tolerance nothing meets (every row is compared, misses, and replaces a key)."""
    dim, tau = W.PROBE_DIM, 0.05
    rows = []
    g = torch.Generator(device=device)
    g.manual_seed(1234)
    fresh = lambda n: torch.nn.functional.normalize(torch.randn(n, dim, device=device, generator=g), dim=1)
    for n_keys in (320, 1280, 5120, 20480, 81920):
        bits = max(1, (n_keys // 20 - 1).bit_length())            # buckets of 20: 2^bits * 20 >= n_keys
        planes = torch.from_numpy(W.lsh_planes(bits, dim, 0)).to(device)
        for name, px in (("flat", Proximity(None, dim, n_keys, 1, W.POLICY_LRU, 1024, device=device)),
                         (f"bucketed 2^{bits} x 20", Proximity(None, dim, 20, 1, W.POLICY_LRU, 1024, device=device,
                                                                lsh_planes=planes))):
            for b0 in range(0, 4 * n_keys, 1024):                  # four times the capacity: buckets fill up too
                px.search_batch(fresh(1024), tau)
            entry = {"cache": name, "capacity": n_keys, "resident": px.stats()["size"]}
            for batch, calls in ((1, 300), (1024, 20)):
                qs = [fresh(batch) for _ in range(calls)]
                out_ids = torch.empty((batch, 1), dtype=torch.int64, device=device)
                out_hit = torch.empty((batch,), dtype=torch.uint8, device=device)
                torch.cuda.synchronize(device)
                t0 = time.perf_counter()
                for q in qs:
                    px.search_batch(q, tau, out_ids=out_ids, out_hit=out_hit, want_dists=False)
                torch.cuda.synchronize(device)
                entry[f"us_per_query_batch{batch}"] = round((time.perf_counter() - t0) / (calls * batch) * 1e6, 3)
            rows.append(entry)
            px.close()
    print(json.dumps({"metric": "cache_lookup_time_vs_capacity", "unit": "us per query", "n_gpus": 1,
                      "data": "synthetic", "config": {"dim": dim, "tau": tau, "policy": "LRU"}, "rows": rows}))


def probe_microbench(args, torch, np, W, Proximity, device, steps=None, warmup=None):
    """Cache probe alone: 10 000 resident keys, batches of 4 096 queries, no corpus behind the cache.
    Returns the result line."""
    n_keys, dim, batch, tau = W.PROBE_KEYS, W.PROBE_DIM, W.PROBE_BATCH, W.PROBE_TAU
    steps = steps if steps is not None else (args.steps if args.steps is not None else 20)
    warmup = warmup if warmup is not None else (args.warmup if args.warmup is not None else 2)
    planes = None
    if args.lsh_bits > 0:
        planes = torch.from_numpy(W.lsh_planes(args.lsh_bits, dim, 0)).to(device)
    px = Proximity(None, dim, args.bucket_capacity if planes is not None else n_keys, 1, W.POLICY_LRU, batch,
                   device=device, lsh_planes=planes)
    keys = torch.from_numpy(W.probe_warm_keys(n_keys, dim, 0)).to(device)
    for b0 in range(0, n_keys, batch):
        px.search_batch(keys[b0:b0 + batch], tau)
    mix = W.ProbeMix(dim, 0)
    # Pass 1 (untimed) draws the batches: each is drawn against the keys resident when it arrives, so the
    # library's own cache is read back between calls.  Pass 2 clears the cache, warms it the same way and
    # replays the recorded batches back to back: the same states recur, and the timed calls are not
    # separated by host work (an idle GPU drops its clocks and the short kernels of a call would be timed slow).
    batches = []
    for step in range(warmup + steps):
        _, resident, _ = px.cache_dump(want_keys=True)
        q = torch.from_numpy(mix.batch(resident, batch)).to(device)
        px.search_batch(q, tau)
        batches.append(q)
    sizes_1 = px.stats()
    px.clear()
    for b0 in range(0, n_keys, batch):
        px.search_batch(keys[b0:b0 + batch], tau)
    out_ids = torch.empty((batch, 1), dtype=torch.int64, device=device)
    out_hit = torch.empty((warmup + steps, batch), dtype=torch.uint8, device=device)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for step in range(warmup):
        px.search_batch(batches[step], tau, out_ids=out_ids, out_hit=out_hit[step], want_dists=False)
    torch.cuda.synchronize(device)
    ev0.record()
    for step in range(warmup, warmup + steps):
        px.search_batch(batches[step], tau, out_ids=out_ids, out_hit=out_hit[step], want_dists=False)
    ev1.record()
    torch.cuda.synchronize(device)
    total_ms = ev0.elapsed_time(ev1)
    hits = int(out_hit[warmup:].sum().item())
    sizes_2 = px.stats()
    assert all(sizes_1[key] == sizes_2[key] for key in ("hits", "misses", "evictions", "size")), "replay diverged"
    flops = 2.0 * batch * (n_keys + batch) * dim
    ms = total_ms / steps
    probe_kernel = None
    if planes is None:
        # The probe's distance kernel alone, from the library's HIP events on a further replay of the first timed
        # batches: one record per row range (first row, rows); a slice of 64 rows meets the slots and the batch rows
        # up to its own last row.
        px.clear()
        for b0 in range(0, n_keys, batch):
            px.search_batch(keys[b0:b0 + batch], tau)
        for step in range(warmup):
            px.search_batch(batches[step], tau, out_ids=out_ids, out_hit=out_hit[step], want_dists=False)
        px.profile_start()
        for step in range(warmup, warmup + min(steps, 8)):
            px.search_batch(batches[step], tau, out_ids=out_ids, out_hit=out_hit[step], want_dists=False)
        rec = px.profile_stop(kind=1)   # the probe launches
        k_flops = k_ms = 0.0
        for _, r0, rows, r_ms in rec:
            for m0 in range(r0, r0 + rows, 64):
                k_flops += 2.0 * min(64, r0 + rows - m0) * (n_keys + min(m0 + 64, r0 + rows)) * dim
            k_ms += r_ms
        if rec and k_ms > 0:
            probe_kernel = {"kernel": "scan_regq_kernel (probe form)", "launches_timed": len(rec),
                            "avg_launch_ms": round(k_ms / len(rec), 5), "launches_per_call": round(len(rec) / min(steps, 8), 2),
                            "achieved_TFLOPs": round(k_flops / (k_ms * 1e-3) / 1e12, 2),
                            "frac_of_f32_mfma_peak": round(k_flops / (k_ms * 1e-3) / 1e12 / F32_MFMA_PEAK_TFLOPS, 4),
                            "algorithmic_flops_per_call": k_flops / min(steps, 8)}
    if planes is not None:
        # bucketed cache: no contraction; per row L inner products and at most b float64 distances
        line = {"metric": "cache_probes_per_sec", "value": round(batch / (ms * 1e-3), 1), "unit": "queries/s",
                "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
                "config": {"workload": f"probe, bucketed cache: {1 << args.lsh_bits} buckets x {args.bucket_capacity} "
                                       f"entries x {dim} f32 warmed with {n_keys} keys, batches of {batch} (half "
                                       f"perturbed resident keys, radius U(0,{W.PROBE_MAX_RADIUS}); half fresh), "
                                       f"tau={tau}, LRU, no corpus",
                           "hit_rate": round(hits / (steps * batch), 4), "resident_keys": px.stats()["size"]},
                "roofline": None, "cpu_baseline": None}
        px.close()
        return line
    line = {"metric": "cache_probes_per_sec", "value": round(batch / (ms * 1e-3), 1), "unit": "queries/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"probe: {n_keys} resident keys x {dim} f32, batches of {batch} (half perturbed "
                                   f"resident keys, radius U(0,{W.PROBE_MAX_RADIUS}); half fresh), tau={tau}, LRU, "
                                   "insert on miss, no corpus", "hit_rate": round(hits / (steps * batch), 4)},
            "roofline": {"bound": "mfma", "achieved": round(flops / (ms * 1e-3) / 1e12, 2),
                         "peak": F32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(flops / (ms * 1e-3) / 1e12 / F32_MFMA_PEAK_TFLOPS, 4), "traffic": None,
                         "note": "whole call (probe contraction, candidate extraction, resolver, insertion) "
                                 "against the probe contraction's 2*B*(c+B)*d flops",
                         "probe_kernel": probe_kernel},
            "cpu_baseline": None}
    px.close()
    return line


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2503_05530_amd import workloads as W
    from paper_2503_05530_amd.binding import Proximity

    device = torch.device("cuda:0")
    if args.calibrate_copy:
        src = torch.full((1 << 28,), 1.5, dtype=torch.float32, device=device)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize(device)
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4,
                          "copies": 5}))
        return
    if args.probe_scaling:
        return probe_scaling(args, torch, np, W, Proximity, device)
    if args.workload == "probe":
        print(json.dumps(probe_microbench(args, torch, np, W, Proximity, device)))
        return
    if args.recall_sweep:
        return recall_sweep(args, torch, np, W, Proximity, device)
    w = W.WORKLOADS[args.workload]
    line = measure_stream_workload(args, torch, np, W, Proximity, device, w, tau=args.tau, batch=args.batch,
                                   steps=args.steps, warmup=args.warmup, headline=True)
    print(json.dumps(line))


def make_corpus(torch, W, device, w, n_docs):
    """(host copy or None, device tensor): corpora of 8 M rows and more are drawn on the device, chunk by chunk."""
    if n_docs >= 8_000_000:
        corpus_dev = torch.empty((n_docs, w.dim), device=device,
                                 dtype=torch.bfloat16 if w.corpus_dtype == W.DTYPE_BF16 else torch.float32)
        for r0, chunk in W.device_corpus_chunks(n_docs, w.dim, w.seed, device, w.corpus_dtype):
            corpus_dev[r0:r0 + chunk.shape[0]] = chunk
        return None, corpus_dev
    corpus = W.corpus_for(w, n_docs)
    return corpus, torch.from_numpy(corpus).to(device)


def default_preroll(w, batch):
    """Rows replayed untimed before the warm-up calls: enough misses to fill the cache and settle the hit rate."""
    rows = 2048 if w.capacity <= 300 else 4096
    return min(rows, w.n_stream // 4) // PREROLL_BATCH * PREROLL_BATCH


def measure_stream_workload(args, torch, np, W, Proximity, device, w, tau=None, batch=None, steps=None, warmup=None,
                            headline=False):
    """One workload through proximity_search_batch: throughput of the timed calls, roofline of the scan kernel
    they launched.  With `headline` (the mid workload of the default run) also the sweep over the other
    (tau, batch) points and the other benchmark configurations, and the CPU oracle beside it."""
    tau = w.tau if tau is None else tau
    batch = w.batch if batch is None else batch
    n_docs = w.n_docs if args.n_docs is None or not headline else args.n_docs
    steps = steps if steps is not None else (20000 if batch == 1 else 1000)
    warmup = warmup if warmup is not None else (2000 if batch == 1 else 50)
    pre = default_preroll(w, batch)
    if pre + (steps + warmup) * batch > w.n_stream * 3 // 4:
        steps = max(1, (w.n_stream * 3 // 4 - pre) // batch - warmup)
    max_batch = max(batch, PREROLL_BATCH)

    t_gen = time.perf_counter()
    queries = W.stream_for(w)
    corpus, corpus_dev = make_corpus(torch, W, device, w, n_docs)
    q_dev = torch.from_numpy(queries).to(device)
    t_gen = time.perf_counter() - t_gen
    elem = 2 if w.corpus_dtype == W.DTYPE_BF16 else 4

    planes = planes_host = None
    if headline and args.lsh_bits > 0:
        planes_host = W.lsh_planes(args.lsh_bits, w.dim, w.seed)
        planes = torch.from_numpy(planes_host).to(device)
    capacity = args.bucket_capacity if planes is not None else w.capacity
    rho = args.rho if headline else 1
    metric_name = args.metric if headline else "l2"
    metric = {"l2": 0, "ip": 1, "cosine": 2}[metric_name]
    if metric == 2:
        tau = tau * tau / 2.0
    px = Proximity(corpus_dev, w.dim, capacity, w.k, w.policy, max_batch, rerank_factor=rho, lsh_planes=planes,
                   metric=metric, flags=1 if args.exact_scan else 0)      # (1: PROXIMITY_FLAG_NO_ROUNDED_SCAN)
    n_rows = len(queries)
    outs = (torch.empty((n_rows, w.k), dtype=torch.int64, device=device),
            torch.empty((n_rows, w.k), dtype=torch.float32, device=device),
            torch.empty((n_rows,), dtype=torch.uint8, device=device))

    dt, hit_rate, first_row = timed_run(torch, px, q_dev, tau, batch, warmup, steps, outs, device, pre)
    qps = steps * batch / dt

    # roofline of the dominant kernel, the corpus-scan distance kernel: HBM-bound while a launch serves
    # few queries, matrix-core-bound once 2*M flops per 4 corpus bytes pass the ridge (157.3 TF / 8 TB/s)
    next_call = first_row // batch + steps
    n_prof = max(1, min(steps, 4000 if batch <= 8 else 400, w.n_stream // batch - next_call))
    busy = profiled_scan(torch, px, q_dev, tau, batch, next_call, n_prof, outs, device)
    checks = px.stats()
    one_plane = checks["coarse_scan_calls"] > 0 and checks["coarse_scan_fails"] == 0
    roofline = scan_roofline(busy, n_docs, w.dim, batch, elem, one_plane)

    sweep = []
    if headline and not args.no_sweep and w.name == "mid":
        for s_tau, s_batch, s_warm, s_steps in ((0.0, 1, 100, 2000), (0.25, 64, 30, 300), (0.0, 64, 10, 200)):
            run_tau = s_tau * s_tau / 2.0 if metric == 2 else s_tau
            s_dt, s_hit, s_first = timed_run(torch, px, q_dev, run_tau, s_batch, s_warm, s_steps, outs, device, pre)
            s_busy = profiled_scan(torch, px, q_dev, run_tau, s_batch, s_first // s_batch + s_steps,
                                   min(s_steps, 200), outs, device)
            sweep.append({"workload": "mid", "tau": s_tau, "batch": s_batch, "steps": s_steps, "warmup": s_warm,
                          "cache_preroll_rows": pre,
                          "queries_per_s": round(s_steps * s_batch / s_dt, 1), "hit_rate": round(s_hit, 4),
                          "ms_per_step": round(1e3 * s_dt / s_steps, 4),
                          "roofline": scan_roofline(s_busy, n_docs, w.dim, s_batch, elem, one_plane)})
        if one_plane:
            # the same all-miss point with the operands multiplied as they are stored (float32 matrix instruction):
            # the scan that the rounded one falls back to when its exactness checks stop passing
            from paper_2503_05530_amd.binding import FLAG_NO_ROUNDED_SCAN
            pe = Proximity(corpus_dev, w.dim, capacity, w.k, w.policy, max_batch, rerank_factor=rho, lsh_planes=planes,
                           metric=metric, flags=FLAG_NO_ROUNDED_SCAN)
            e_dt, e_hit, e_first = timed_run(torch, pe, q_dev, 0.0, 64, 10, 200, outs, device, pre)
            e_busy = profiled_scan(torch, pe, q_dev, 0.0, 64, e_first // 64 + 200, 200, outs, device)
            sweep.append({"workload": "mid", "tau": 0.0, "batch": 64, "steps": 200, "warmup": 10,
                          "scan": "operands as stored (PROXIMITY_FLAG_NO_ROUNDED_SCAN)", "cache_preroll_rows": pre,
                          "queries_per_s": round(200 * 64 / e_dt, 1), "hit_rate": round(e_hit, 4),
                          "ms_per_step": round(1e3 * e_dt / 200, 4),
                          "roofline": scan_roofline(e_busy, n_docs, w.dim, 64, elem, False)})
            pe.close()

    cpu = None
    if headline and not args.no_cpu_baseline and corpus is not None:
        cpu = cpu_baseline(args, np, w, corpus, queries, tau, capacity, planes_host, metric, first_row)

    line = {
        "metric": "retrieval_queries_per_sec", "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(1e3 * dt / steps, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        # the type the scan's products are formed in (the ranking that decides every list is float64 throughout)
        "dtype": "bf16" if (elem == 2 and w.dim >= 64 and batch > 4) or (batch > 4 and one_plane) else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: corpus {n_docs}x{w.dim} {'bf16' if elem == 2 else 'f32'} unit Gaussian, "
                               f"{w.choice}({w.zipf_s}) stream of "
                               f"{w.n_stream} over {w.n_bases} bases (perturbation {w.radius}), capacity "
                               f"{w.capacity}, {'LRU' if w.policy else 'FIFO'}, k={w.k}",
                   "tau": tau, "batch": batch, "rerank_factor": rho, "distance": metric_name,
                   "cache": (f"bucketed: {1 << args.lsh_bits} buckets x {capacity}" if planes is not None
                             else f"flat: {w.capacity}"),
                   "cache_preroll_rows": pre, "first_timed_row": first_row,
                   "hit_rate": round(hit_rate, 4),
                   "queries_timed": steps * batch, "setup_s": round(t_gen, 1),
                   "searches_ranked_twice": checks["slack_exhausted"], "searches_not_proven_exact": checks["slack_unresolved"],
                   "rounded_scan_calls": checks["coarse_scan_calls"]},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    px.close()
    del px, corpus_dev, q_dev, outs
    torch.cuda.empty_cache()
    if headline:
        # the other benchmark configurations, each measured like the headline (own corpus, own roofline)
        if not args.no_sweep and w.name == "mid" and args.n_docs is None:
            for name, o_steps, o_warm in (("lowreuse", 150, 10), ("large", 40, 4)):
                free, _ = torch.cuda.mem_get_info(device)
                ow = W.WORKLOADS[name]
                need = ow.n_docs * ow.dim * (2 if ow.corpus_dtype == W.DTYPE_BF16 else 4) * 1.25
                if free < need:
                    sweep.append({"workload": name, "skipped": f"needs {need / 2**30:.0f} GiB of free device memory"})
                    continue
                o = measure_stream_workload(args, torch, np, W, Proximity, device, ow, steps=o_steps, warmup=o_warm)
                sweep.append({"workload": name, "tau": o["config"]["tau"], "batch": o["config"]["batch"],
                              "steps": o["steps"], "warmup": o["warmup"],
                              "cache_preroll_rows": o["config"]["cache_preroll_rows"],
                              "queries_per_s": o["value"], "hit_rate": o["config"]["hit_rate"],
                              "ms_per_step": o["ms_per_step"], "dtype": o["dtype"], "setup_s": o["config"]["setup_s"],
                              "roofline": o["roofline"]})
            p = probe_microbench(args, torch, np, W, Proximity, device, steps=20, warmup=2)
            sweep.append({"workload": "probe", "tau": W.PROBE_TAU, "batch": W.PROBE_BATCH, "steps": p["steps"],
                          "warmup": p["warmup"], "queries_per_s": p["value"], "hit_rate": p["config"]["hit_rate"],
                          "ms_per_step": p["ms_per_step"], "roofline": p["roofline"]})
        line["sweep"] = sweep
    return line


def cpu_baseline(args, np, w, corpus, queries, tau, capacity, planes_host, metric, first):
    """The oracle as it stands on this host, on a bounded sample of the same workload.
    `value`: the literal oracle (Algorithm 1 with the brute-force database call, element-wise float64 numpy) on
    `--cpu-sample` stream rows that follow the timed region's first row, after a decisions-only replay of the
    rows before them, with the BLAS pool held to one thread; `cores` is measured (CPU seconds / wall seconds).
    Beside it: an estimate for the first 2 000 rows of the stream (their decisions replayed and timed, every
    miss charged the sample's mean database call), the oracle's batched form on all cores with the BLAS
    thread count the pool reports, and the two pieces on their own."""
    from oracle import proximity_oracle as po
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        pools = [p for p in threadpool_info() if p.get("user_api") == "blas"]
        blas_threads = max([p["num_threads"] for p in pools], default=1)
    except ImportError:
        threadpool_limits = None
        blas_threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    k_store = args.rho * w.k
    no_db = lambda q: (np.full(k_store, -1, np.int64), np.full(k_store, np.inf))

    def fresh_oracle(retrieve):
        if planes_host is not None:
            return po.LshCacheOracle(corpus, planes_host, capacity, w.k, w.policy, retrieve=retrieve,
                                     rerank_factor=args.rho, metric=metric)
        return po.FlatCacheOracle(corpus, w.capacity, w.k, w.policy, rerank_factor=args.rho, retrieve=retrieve,
                                  metric=metric)

    def timed(fn):
        c0, t0 = os.times(), time.perf_counter()
        out = fn()
        wall = time.perf_counter() - t0
        c1 = os.times()
        return out, wall, (c1.user - c0.user + c1.system - c0.system) / max(wall, 1e-9)

    class one_thread:
        def __enter__(self):
            self.ctx = threadpool_limits(limits=1) if threadpool_limits else None
            if self.ctx:
                self.ctx.__enter__()

        def __exit__(self, *a):
            if self.ctx:
                self.ctx.__exit__(*a)

    # (1) the literal oracle on a short stretch, one thread
    orc = fresh_oracle(no_db)
    orc.lookup_stream(queries[:first], tau)            # decisions only: the cache state of the timed region
    orc.retrieve = lambda q: po.exact_knn(corpus, q, k_store, metric=metric)
    n_s = min(args.cpu_sample, len(queries) - first)
    with one_thread():
        (o_ids, o_d, o_hit, _), cdt, cores = timed(lambda: orc.lookup_stream(queries[first:first + n_s], tau))
    misses = int((o_hit == 0).sum())
    cpu = {"value": round(n_s / cdt, 4), "unit": "queries/s", "cores": max(1, round(cores)), "kind": "oracle",
           "sample": f"stream rows {first}..{first + n_s - 1} of the same workload after a decisions-only "
                     f"replay of rows 0..{first - 1}; {misses} misses, {cdt:.1f} s, literal float64 numpy oracle, "
                     f"BLAS pool limited to 1 thread",
           "cores_measured": round(cores, 2), "host_cpus": os.cpu_count(), "cpu_model": cpu_model(),
           "blas_threads_available": blas_threads}
    # (2) the first 2 000 rows of the stream: decisions replayed and timed; each miss charged one database call
    n_est = min(2000, len(queries))
    with one_thread():
        (e_hit, _, _), e_dt, _ = timed(lambda: po.simulate_decisions(queries[:n_est], tau, capacity, w.policy,
                                                                     planes=planes_host, metric=metric))
        _, scan_dt, _ = timed(lambda: po.exact_knn(corpus, queries[0], k_store, metric=metric))
    e_miss = int((e_hit == 0).sum())
    cpu["first_2000_rows_estimate"] = {
        "queries_per_s": round(n_est / (e_dt + e_miss * scan_dt), 4), "rows": n_est, "misses": e_miss,
        "decisions_s": round(e_dt, 3), "one_database_call_s": round(scan_dt, 3),
        "note": "decisions measured on all rows; database calls measured once and multiplied by the misses"}
    # (3) the pieces, oracle code as it stands: one cache probe (distances to c keys and the nearest) at two
    # cache sizes, one database call, and the batched form (float64 matrix product per block of rows) on all cores
    parts = {}
    with one_thread():
        for c_keys in (300, 10000):
            keys64 = po.as_f64_rows(corpus[:c_keys])
            _, p_dt, _ = timed(lambda: [po.l2_distances(queries[t], keys64).argmin() for t in range(20)])
            parts[f"probe_us_c{c_keys}"] = round(p_dt / 20 * 1e6, 1)
    parts[f"scan_s_{len(corpus)}_docs_one_thread"] = round(scan_dt, 3)
    _, b_dt, b_cores = timed(lambda: po.batched_exact_knn(corpus, queries[:64], w.k, metric=metric))
    parts["batched_scan_s_64_queries_all_cores"] = round(b_dt, 3)
    parts["batched_scan_cores_measured"] = round(b_cores, 2)
    parts["batched_scan_blas_threads"] = blas_threads
    cpu["parts"] = parts
    return cpu


if __name__ == "__main__":
    main()
