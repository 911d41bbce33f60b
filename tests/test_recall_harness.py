"""The k-recall sweep harness of bench.py (Section 4: database k-recall = the fraction of the k documents handed
out that the index itself would have returned for the query; hit rate = fraction of queries served from the
cache): its counting against a hand-worked example on the CPU, and its whole output against the oracle on the GPU."""
import numpy as np
import pytest
import torch

import bench
from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W


def test_k_recall_counting_on_a_hand_worked_example():
    # ten queries, k = 4; the index's own answers, and what a cache handed out
    truth = torch.tensor([[1, 2, 3, 4], [5, 6, 7, 8], [9, 10, 11, 12], [0, 1, 2, 3], [4, 5, 6, 7],
                          [8, 9, 10, 11], [12, 13, 14, 15], [1, 3, 5, 7], [2, 4, 6, 8], [0, 9, 18, 27]])
    ids = torch.tensor([[1, 2, 3, 4],       # the same list                     4/4
                        [8, 7, 6, 5],       # the same documents, other order   4/4
                        [9, 10, 40, 41],    # two of four                       2/4
                        [50, 51, 52, 53],   # none                              0/4
                        [4, 60, 61, 62],    # one                               1/4
                        [8, 9, 10, -1],     # three and a padding entry         3/4
                        [-1, -1, -1, -1],   # nothing found at all              0/4
                        [7, 5, 3, 99],      # three                             3/4
                        [2, 4, 6, 8],       #                                   4/4
                        [27, 0, 5, 6]])     # two                               2/4
    want = [1.0, 1.0, 0.5, 0.0, 0.25, 0.75, 0.0, 0.75, 1.0, 0.5]
    got = bench.k_recall_per_query(ids, truth)
    assert got.tolist() == want
    assert abs(float(got.mean()) - 0.575) < 1e-7
    # a padding id in the index's own answer is never "found" either
    assert bench.k_recall_per_query(torch.tensor([[-1, 3]]), torch.tensor([[-1, 3]])).tolist() == [0.5]


@pytest.mark.gpu
def test_recall_sweep_equals_oracle_hit_rates_and_recalls():
    """The harness on a small corpus against the same quantities computed from the oracle's outputs alone:
    hit rate from the oracle's flags, k-recall from the oracle's returned lists against the oracle's exact
    search, for the flat and the bucketed cache, with and without re-ranking, at three tolerances."""
    from paper_2503_05530_amd.binding import Proximity
    dev = torch.device("cuda:0")
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_for(w, 6000)
    q = W.stream_for(w, 512)
    bits, b, rho, batch, taus = 3, 6, 4, 64, (0.0, 0.25, 1.0)
    rows = bench.recall_sweep_rows(torch, W, Proximity, dev, w, torch.from_numpy(corpus).to(dev),
                                   torch.from_numpy(q).to(dev), batch, rho, bits, b, taus)
    truth, _ = po.batched_exact_knn(corpus, q, w.k)
    planes = W.lsh_planes(bits, w.dim, w.seed)
    assert len(rows) == 2 * 2 * len(taus)
    at = {(r["cache"].split()[0], r["rerank_factor"], r["tau"]): r for r in rows}
    some_hits = 0
    for cache, cap, pl in (("flat", w.capacity, None), ("bucketed", b, planes)):
        for r in (1, rho):
            for tau in taus:
                out = po.lookup_stream_deferred(corpus, q, tau, cap, w.k, w.policy, rerank_factor=r, planes=pl)
                ids, hit = out[0], out[2]
                recall = np.array([len(set(ids[t].tolist()) & set(truth[t].tolist())) / w.k for t in range(len(q))])
                row = at[(cache, r, tau)]
                assert row["hit_rate"] == round(float(hit.mean()), 4), (cache, r, tau)
                assert abs(row["k_recall"] - recall.mean()) < 1e-4, (cache, r, tau)
                if hit.any():
                    assert abs(row["k_recall_on_hits"] - recall[hit == 1].mean()) < 1e-4
                    some_hits += 1
                else:
                    assert row["k_recall_on_hits"] is None and row["k_recall"] == 1.0
    assert some_hits >= 6


def test_roofline_entry_by_hand():
    """bench.py's roofline entry for the scan kernel, worked by hand: which roof a launch is priced against (the
    ridge is peak flops x bytes per element / (2 x planes x HBM peak) queries per launch), achieved = algorithmic
    bytes or flops over the mean launch time, and the kernel the stats name."""
    n, d = 1_000_000, 768
    bytes_f32 = n * d * 4 + n * 4
    # one query per launch, 0.46 ms: HBM-bound, the scores-only form of the register-resident kernel
    r = bench.scan_roofline([(0.46, 1)] * 5, n, d, 1)
    assert r["bound"] == "hbm" and r["kernel"] == "scan_regq_kernel (scores only)"
    assert r["achieved"] == pytest.approx(bytes_f32 / 0.46e-3 / 1e9, rel=1e-4)
    assert r["frac"] == pytest.approx(bytes_f32 / 0.46e-3 / 1e9 / 8000.0, abs=1e-4)
    assert r["algorithmic_bytes_per_launch"] == bytes_f32 and r["traffic_counters"]["measured_in_this_run"] is False
    # 64 queries on the operands as stored: float32 matrix-bound (ridge 157.3e12 / 8e12 * 4 / 2 = 39 queries)
    r = bench.scan_roofline([(0.77, 64)] * 3, n, d, 64)
    assert r["bound"] == "mfma" and r["kernel"] == "scan_regq_kernel" and r["peak"] == 157.3
    assert r["achieved"] == pytest.approx(2.0 * 64 * n * d / 0.77e-3 / 1e12, rel=1e-3)
    # the same launch on rounded operands: bfloat16 matrix cores, one plane: ridge at 625 queries, so HBM-bound
    r = bench.scan_roofline([(0.5, 64)] * 3, n, d, 64, 4, True)
    assert r["bound"] == "hbm" and r["kernel"] == "scan_regq_kernel (rounded operands)"
    assert r["achieved"] == pytest.approx(bytes_f32 / 0.5e-3 / 1e9, rel=1e-4)
    assert r["achieved_TFLOPs"] == pytest.approx(2.0 * 64 * n * d / 0.5e-3 / 1e12, rel=1e-3)
    # a bfloat16 corpus, 128 queries: two planes put the ridge at 156 queries, one plane at 312
    nb, db = 8_000_000, 384
    r2 = bench.scan_roofline([(1.5, 127)] * 2, nb, db, 128, 2, False)
    r1 = bench.scan_roofline([(1.1, 127)] * 2, nb, db, 128, 2, True)
    assert r2["bound"] == "hbm" and r2["kernel"] == "scan_regq_kernel" and r1["kernel"] == "scan_regq_kernel (one plane)"
    assert r2["achieved_TFLOPs"] == pytest.approx(2 * 2.0 * 127 * nb * db / 1.5e-3 / 1e12, rel=1e-3)
    assert r1["achieved_TFLOPs"] == pytest.approx(2.0 * 127 * nb * db / 1.1e-3 / 1e12, rel=1e-3)
    r3 = bench.scan_roofline([(1.5, 200)] * 2, nb, db, 256, 2, False)        # past the two-plane ridge
    assert r3["bound"] == "mfma" and r3["peak"] == 2500.0
    assert bench.scan_roofline([], n, d, 1) is None
