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
