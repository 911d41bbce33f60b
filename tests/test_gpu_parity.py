"""GPU-vs-oracle parity through the C ABI (element by element, same seeded inputs)."""
import os

import numpy as np
import pytest
import torch

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

import parity as P
from test_oracle_pins import EVICTION_CASES, line_vectors

pytestmark = pytest.mark.gpu

DEV = torch.device("cuda:0")


@pytest.fixture(scope="module")
def B():
    import paper_2503_05530_amd.binding as b
    return b


def gpu_corpus(x: np.ndarray, bf16=False):
    t = torch.from_numpy(x).to(DEV)
    return t.to(torch.bfloat16) if bf16 else t


# ---------------------------------------------------------------------------
# The index search alone (Section 2.2)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n_docs,dim,k,nq", [
    (5000, 768, 10, 1), (5000, 768, 10, 3), (9001, 768, 32, 8), (4097, 384, 100, 5),
    (700, 64, 7, 2), (70000, 768, 10, 13), (3, 32, 5, 2), (8191, 1024, 16, 4), (300, 4096, 3, 8),
    # more than 8 queries: matrix-core scan, one tile shape per range of query counts
    (50000, 768, 10, 9), (50000, 768, 10, 40), (50011, 768, 32, 100), (30000, 768, 10, 300),
    (1000, 64, 7, 20), (200, 32, 100, 70), (131, 96, 5, 129), (40000, 768, 10, 80), (40000, 128, 32, 96),
])
def test_knn_matches_oracle_f32(B, n_docs, dim, k, nq):
    corpus = W.corpus_f32(n_docs, dim, 3)
    q = W.unit_rows(np.random.default_rng(5).standard_normal((nq, dim))).astype(np.float32)
    px = B.Proximity(gpu_corpus(corpus), dim, 0, k, B.POLICY_FIFO, max(nq, 1))
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    ids, dists = ids.cpu().numpy(), dists.cpu().numpy()
    o_ids, o_d = po.batched_exact_knn(corpus, q, k)
    P.assert_lists_match(ids, dists, o_ids, o_d, corpus, q, what=f"knn {n_docs}x{dim}")
    px.close()


@pytest.mark.parametrize("metric,dim,nq", [(po.METRIC_L2, 384, 1), (po.METRIC_COSINE, 384, 3), (po.METRIC_IP, 768, 4),
                                           (po.METRIC_L2, 768, 2)])
def test_few_queries_against_a_long_corpus(B, metric, dim, nq):
    """Calls of up to four rows on a corpus of half a million rows and more are scored by the register-resident
    kernel in its scores-only form (768 and 384 float32 columns); the corpus here ends inside a tile."""
    n_docs, k = 520_077, 7
    corpus = W.corpus_f32(n_docs, dim, 11)
    if metric != po.METRIC_L2:
        corpus *= lengths(n_docs, 0.5, 2.0, 12)
    q = (1.3 * W.unit_rows(np.random.default_rng(13).standard_normal((nq, dim)))).astype(np.float32)
    px = B.Proximity(gpu_corpus(corpus), dim, 0, k, B.POLICY_FIFO, 4, metric=metric)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.batched_exact_knn(corpus, q, k, metric=metric)
    P.assert_lists_match(ids.cpu().numpy(), dists.cpu().numpy(), o_ids, o_d, corpus, q, what=f"long corpus {dim}",
                         metric=metric)
    assert px.stats()["slack_unresolved"] == 0
    px.close()


def test_listing_probe_at_384_columns(B):
    """A cache of 3 000 keys of 384 columns probed with calls of 256 and of 1 700 rows: the probe that lists its
    candidates itself, in one range and in row ranges, against the oracle's decisions."""
    dim, cap, k = 384, 3000, 4
    corpus = W.corpus_f32(3000, dim, 21)
    base = W.base_queries(2500, dim, 22)
    idx = np.random.default_rng(23).integers(0, 2500, size=6000)
    q = W.perturbed_stream(base, idx, 0.1, 24)
    for policy, batch in ((po.POLICY_LRU, 256), (po.POLICY_FIFO, 1700)):
        want = po.lookup_stream_deferred(corpus, q, 0.25, cap, k, policy)
        px = B.Proximity(gpu_corpus(corpus), dim, cap, k, policy, batch)
        got = P.run_stream(px, q, 0.25, batch, DEV)
        P.assert_stream_parity(got, want[:4], corpus, q, what=f"listing probe, calls of {batch}")
        seq, _, _ = px.cache_dump()
        assert seq.tolist() == want[4].dump_seq().tolist()
        assert 0.2 < want[2].mean() < 0.8
        px.close()


@pytest.mark.parametrize("nq", [6, 128])
def test_knn_matches_oracle_bf16(B, nq):
    n_docs, dim, k = 20000, 384, 100
    x32 = W.corpus_f32(n_docs, dim, 9)
    bits = W.f32_to_bf16_bits(x32)
    xb = W.bf16_bits_to_f32(bits)                       # exact values the GPU holds
    t = torch.from_numpy(x32).to(DEV).to(torch.bfloat16)
    assert (t.view(torch.int16).cpu().numpy().view(np.uint16) == bits).all()
    q = W.unit_rows(np.random.default_rng(6).standard_normal((nq, dim))).astype(np.float32)
    px = B.Proximity(t, dim, 0, k, B.POLICY_FIFO, nq)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.batched_exact_knn(xb, q, k)
    P.assert_lists_match(ids.cpu().numpy(), dists.cpu().numpy(), o_ids, o_d, xb, q,
                         dist_rtol=P.DIST_RTOL_BF16, what="knn bf16")
    px.close()


@pytest.mark.parametrize("trial", range(24))
def test_knn_random_shapes_at_the_register_resident_dimensions(B, trial):
    """The same at the corpus types and dimensions the scan with its queries in registers is built for
    (float32 768 / 384, bfloat16 384 / 256), query counts around its one-, two- and four-group shapes and its
    passes of 64 / 128 queries, corpora that end inside a tile."""
    rng = np.random.default_rng([trial, 991])
    bf16 = bool(rng.integers(0, 2))
    dim = int(rng.choice([384, 256] if bf16 else [768, 384]))
    n_docs = int(rng.choice([130, 1000, 4097, 20000, 66000, 140000, 300000])) + int(rng.integers(0, 200))
    nq = int(rng.choice([5, 9, 16, 17, 31, 33, 48, 64, 65, 80, 100, 128, 129, 200]))
    k = int(rng.choice([1, 5, 10, 32, 100]))
    metric = int(rng.choice([po.METRIC_L2, po.METRIC_L2, po.METRIC_IP, po.METRIC_COSINE]))
    x = W.corpus_f32(n_docs, dim, 1000 + trial)
    if metric != po.METRIC_L2:
        x *= rng.uniform(0.5, 2.0, size=(n_docs, 1)).astype(np.float32)
    t = torch.from_numpy(x).to(DEV)
    if bf16:
        t = t.to(torch.bfloat16)
        x = t.to(torch.float32).cpu().numpy()             # exact values the GPU holds
    q = (rng.uniform(0.5, 1.5) * W.unit_rows(rng.standard_normal((nq, dim)))).astype(np.float32)
    px = B.Proximity(t, dim, 0, k, B.POLICY_FIFO, nq, metric=metric)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.batched_exact_knn(x, q, k, metric=metric)
    P.assert_lists_match(ids.cpu().numpy(), dists.cpu().numpy(), o_ids, o_d, x, q,
                         dist_rtol=P.DIST_RTOL_BF16 if bf16 else P.DIST_RTOL_F32,
                         what=f"bf16={bf16} dim={dim} n_docs={n_docs} nq={nq} k={k} metric={metric}", metric=metric)
    assert px.stats()["slack_unresolved"] == 0
    px.close()


@pytest.mark.parametrize("trial", range(30))
def test_knn_random_shapes(B, trial):
    """The index search alone at shapes drawn at random: dimensions from 32 to 2 048, corpus sizes around
    every threshold of the launch logic (tile and segment sizes, the head pass), k from 1 to the largest, query
    counts around every tile-shape boundary, both corpus types, all three distance functions."""
    rng = np.random.default_rng([trial, 99])
    dim = int(rng.choice([32, 64, 96, 128, 160, 256, 384, 512, 768, 1024, 2048]))
    n_docs = int(rng.choice([1, 7, 63, 129, 1000, 4095, 16383, 16384 * 8 - 1, 16384 * 8, 140001]))
    n_docs = min(n_docs, 60_000_000 // dim)
    k = int(rng.choice([1, 5, 10, 32, 100, B.MAX_K]))
    nq = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 31, 32, 33, 64, 65, 96, 97, 128, 129, 200]))
    bf16 = bool(rng.random() < 0.3)
    metric = int(rng.choice([po.METRIC_L2, po.METRIC_L2, po.METRIC_IP, po.METRIC_COSINE]))
    x32 = W.corpus_f32(n_docs, dim, trial)
    if metric != po.METRIC_L2:
        x32 = (x32 * rng.uniform(0.3, 3.0, size=(n_docs, 1))).astype(np.float32)
    corpus = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x32)) if bf16 else x32
    q = (W.unit_rows(rng.standard_normal((nq, dim))) * rng.uniform(0.5, 2.0, size=(nq, 1))).astype(np.float32)
    px = B.Proximity(gpu_corpus(x32, bf16), dim, 0, k, B.POLICY_FIFO, nq, metric=metric)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.batched_exact_knn(corpus, q, k, metric=metric)
    P.assert_lists_match(ids.cpu().numpy(), dists.cpu().numpy(), o_ids, o_d, corpus, q,
                         dist_rtol=P.DIST_RTOL_BF16 if bf16 else P.DIST_RTOL_F32,
                         what=f"n_docs {n_docs} dim {dim} k {k} nq {nq} bf16 {bf16} metric {metric}", metric=metric)
    px.close()


@pytest.mark.parametrize("nq", [1, 4, 70])
def test_knn_at_the_largest_k(B, nq):
    n_docs, dim, k = 40000, 768, B.MAX_K
    corpus = W.corpus_f32(n_docs, dim, 11)
    q = W.unit_rows(np.random.default_rng(12).standard_normal((nq, dim))).astype(np.float32)
    px = B.Proximity(gpu_corpus(corpus), dim, 0, k, B.POLICY_FIFO, nq)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.batched_exact_knn(corpus, q, k)
    P.assert_lists_match(ids.cpu().numpy(), dists.cpu().numpy(), o_ids, o_d, corpus, q, what=f"knn k={k}")
    px.close()


def test_knn_duplicate_rows_rank_by_index(B):
    corpus = W.corpus_f32(6000, 768, 4)
    corpus[4500] = corpus[17]
    corpus[99] = corpus[17]
    q = corpus[17:18].copy()
    px = B.Proximity(gpu_corpus(corpus), 768, 0, 5, B.POLICY_FIFO, 1)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.exact_knn(corpus, q[0], 5)
    assert ids.cpu().numpy()[0].tolist() == o_ids.tolist()
    assert ids.cpu().numpy()[0, :3].tolist() == [17, 99, 4500]
    assert dists.cpu().numpy()[0, :3].tolist() == [0.0, 0.0, 0.0]
    px.close()


# ---------------------------------------------------------------------------
# Algorithm 1: hand-worked traces, as one batch per query and as one batch in all
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", EVICTION_CASES, ids=[c["name"] for c in EVICTION_CASES])
@pytest.mark.parametrize("batch", [1, 2, 64])
def test_hand_worked_traces(B, case, batch):
    # rows of different lengths, so that the all-zero query has no near-tied neighbours
    corpus = W.corpus_f32(257, 32, 3) * (1.0 + np.arange(257, dtype=np.float32)[:, None] / 64.0)
    q = line_vectors(case["xs"], dim=32)
    orc = po.FlatCacheOracle(corpus, case["capacity"], 3, case["policy"])
    want = orc.lookup_stream(q, case["tau"])
    assert "".join("H" if h else "M" for h in want[2]) == case["flags"]
    px = B.Proximity(gpu_corpus(corpus), 32, case["capacity"], 3, case["policy"], 64)
    got = P.run_stream(px, q, case["tau"], batch, DEV)
    assert "".join("H" if h else "M" for h in got[2]) == case["flags"]
    assert P.assert_stream_parity(got, want, corpus, q, what=case["name"]) == 0
    seq, keys, ids = px.cache_dump(want_keys=True, want_ids=True)
    assert seq.tolist() == case["left"]
    if len(seq):
        assert (keys == q[seq]).all()
        assert (ids == orc.dump_ids()).all()
    st = px.stats()
    assert st["evictions"] == case["evictions"]
    assert st["hits"] == case["flags"].count("H") and st["misses"] == case["flags"].count("M")
    assert st["size"] == len(case["left"]) and st["queries"] == len(q)
    px.close()


# ---------------------------------------------------------------------------
# Small workload end to end, several batch sizes (same results for any split)
# ---------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_for(w)
    q = W.stream_for(w)
    out = {}
    for policy in (po.POLICY_FIFO, po.POLICY_LRU):
        out[policy] = po.lookup_stream_deferred(corpus, q, w.tau, w.capacity, w.k, policy)
    return w, corpus, q, out


@pytest.mark.parametrize("batch", [1, 7, 64, 256])
@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_tiny_workload(B, tiny, batch, policy):
    w, corpus, q, want = tiny
    o_ids, o_d, o_hit, o_src, dec = want[policy]
    px = B.Proximity(gpu_corpus(corpus), w.dim, w.capacity, w.k, policy, 256)
    got = P.run_stream(px, q, w.tau, batch, DEV)
    excused = P.assert_stream_parity(got, (o_ids, o_d, o_hit, o_src), corpus, q, what=f"tiny b{batch}")
    assert excused == 0
    seq, _, ids = px.cache_dump(want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist()
    assert (ids == o_ids[seq]).all()
    st = px.stats()
    assert st["hits"] == int(o_hit.sum()) and st["evictions"] == dec.n_evictions
    if policy == w.policy:
        assert st["hits"] == 697 and st["evictions"] == 253
    px.close()


def test_one_call_of_the_largest_batch(B):
    """8192 rows in a single call give what the same stream gives one row at a time in the oracle."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["tiny"], n_stream=B.MAX_BATCH, n_bases=1500, seed=21)
    corpus = W.corpus_f32(6000, w.dim, 21)
    q = W.stream_for(w)
    assert len(q) == B.MAX_BATCH
    want = po.lookup_stream_deferred(corpus, q, w.tau, 300, w.k, po.POLICY_LRU)
    px = B.Proximity(gpu_corpus(corpus), w.dim, 300, w.k, po.POLICY_LRU, B.MAX_BATCH)
    got = P.run_stream(px, q, w.tau, B.MAX_BATCH, DEV)
    P.assert_stream_parity(got, want[:4], corpus, q, what="largest batch")
    seq, _, _ = px.cache_dump()
    assert seq.tolist() == want[4].dump_seq().tolist()
    assert 0 < px.stats()["hits"] < B.MAX_BATCH and px.stats()["evictions"] > 0
    px.close()


@pytest.mark.parametrize("cap", [13000, 21000])
@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_cache_at_and_beyond_on_chip_state(B, policy, cap):
    """13 000 keys: near the largest eviction order the resolver holds on chip; 21 000: it no longer
    fits and the resolver works from device memory."""
    # The literal oracle needs minutes at this cache size.  At tau = 0 a query hits exactly when the
    # same vector is resident, so Algorithm 1 is a textbook FIFO/LRU cache keyed by vector identity
    # (test_oracle_pins shows the oracle equal to that model); the model is the expectation here, and
    # the oracle itself is compared on a prefix.
    from collections import OrderedDict
    dim = 32
    rng = np.random.default_rng(31)
    vecs = W.unit_rows(rng.standard_normal((cap + 600, dim))).astype(np.float32)
    which = np.concatenate([np.arange(cap + 300), rng.integers(0, cap + 300, size=700),
                            np.arange(cap + 300, cap + 600), rng.integers(0, cap + 600, size=700)])
    q = vecs[which]
    model, want_hit, evictions = OrderedDict(), [], 0
    for t, key in enumerate(which.tolist()):
        if key in model:
            want_hit.append(1)
            if policy == po.POLICY_LRU:
                model.move_to_end(key)
        else:
            want_hit.append(0)
            if len(model) >= cap:
                model.popitem(last=False)
                evictions += 1
            model[key] = t
    assert evictions > 100 and 300 < sum(want_hit) < 1400
    px = B.Proximity(None, dim, cap, 3, policy, 512, device=DEV)
    _, _, hit = P.run_stream(px, q, 0.0, 512, DEV)
    assert hit.tolist() == want_hit
    seq, _, _ = px.cache_dump()
    assert seq.tolist() == list(model.values())
    assert px.stats()["evictions"] == evictions
    px.close()
    o_hit, _, _ = po.simulate_decisions(q[:600], 0.0, cap, policy)
    assert hit[:600].tolist() == o_hit.tolist()


@pytest.mark.parametrize("trial", range(16))
def test_exact_match_model_at_many_sizes(B, trial):
    """tau = 0 on streams with heavily repeated vectors: Algorithm 1 is then a textbook FIFO/LRU cache keyed
    by vector identity (test_oracle_pins shows the oracle equal to that model), which is cheap enough to check
    capacities from 1 to beyond the on-chip limit, calls of up to 8 192 rows cut at random, tens of thousands
    of rows, hits on rows of the same call, and long eviction sequences."""
    from collections import OrderedDict
    rng = np.random.default_rng([trial, 4242])
    dim = 32
    cap = int(rng.choice([1, 2, 7, 63, 64, 65, 300, 1000, 4097, 10000, 16000, 18700, 19000]))
    policy = int(rng.integers(0, 2))
    max_batch = int(rng.choice([64, 512, 4096, 8192]))
    n_vec = int(cap * rng.choice([0.5, 1.2, 3.0])) + 5
    n = int(rng.choice([3000, 12000, 30000]))
    vecs = W.unit_rows(rng.standard_normal((n_vec, dim))).astype(np.float32)
    which = np.minimum((rng.pareto(1.0, size=n) * n_vec / 20).astype(np.int64), n_vec - 1)
    q = vecs[which]
    model, want_hit, evictions = OrderedDict(), [], 0
    for t, key in enumerate(which.tolist()):
        if key in model:
            want_hit.append(1)
            if policy == po.POLICY_LRU:
                model.move_to_end(key)
        else:
            want_hit.append(0)
            if len(model) >= cap:
                model.popitem(last=False)
                evictions += 1
            model[key] = t
    px = B.Proximity(None, dim, cap, 3, policy, max_batch, device=DEV)
    flags, r0 = [], 0
    while r0 < n:
        step = int(rng.integers(1, max_batch + 1))
        _, _, h = px.search_batch(torch.from_numpy(q[r0:r0 + step]).to(DEV), 0.0)
        flags.append(h)
        r0 += step
    hit = torch.cat(flags).cpu().numpy()
    what = f"cap {cap} policy {policy} max_batch {max_batch} rows {n}"
    assert hit.tolist() == want_hit, what
    seq, _, _ = px.cache_dump()
    assert seq.tolist() == list(model.values()), what
    assert px.stats()["evictions"] == evictions and px.stats()["hits"] == sum(want_hit), what
    px.close()
    o_hit, _, _ = po.simulate_decisions(q[:300], 0.0, cap, policy)
    assert hit[:300].tolist() == o_hit.tolist()


# ---------------------------------------------------------------------------
# Inner-product and cosine indexes (Section 2.2's other distance functions)
# ---------------------------------------------------------------------------
def lengths(n, lo, hi, seed):
    return np.random.default_rng(seed).uniform(lo, hi, size=(n, 1)).astype(np.float32)


@pytest.mark.parametrize("metric", [po.METRIC_IP, po.METRIC_COSINE])
@pytest.mark.parametrize("n_docs,dim,k,nq,bf16", [
    (5000, 768, 10, 1, False), (9001, 768, 32, 4, False), (50000, 768, 10, 40, False), (30011, 384, 100, 70, False),
    (40000, 768, 10, 100, False), (700, 32, 7, 20, False), (20000, 384, 100, 6, True), (20000, 384, 100, 128, True),
])
def test_knn_other_metrics(B, metric, n_docs, dim, k, nq, bf16):
    """Rows of very different lengths: the three distance functions rank differently."""
    x32 = W.corpus_f32(n_docs, dim, 3) * lengths(n_docs, 0.3, 3.0, 4)
    t = gpu_corpus(x32, bf16)
    corpus = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x32)) if bf16 else x32
    q = (W.unit_rows(np.random.default_rng(5).standard_normal((nq, dim))) * lengths(nq, 0.5, 2.0, 6)).astype(np.float32)
    px = B.Proximity(t, dim, 0, k, B.POLICY_FIFO, nq, metric=metric)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    o_ids, o_d = po.batched_exact_knn(corpus, q, k, metric=metric)
    l2_ids, _ = po.batched_exact_knn(corpus, q, k)
    assert (o_ids != l2_ids).any()
    P.assert_lists_match(ids.cpu().numpy(), dists.cpu().numpy(), o_ids, o_d, corpus, q,
                         dist_rtol=P.DIST_RTOL_BF16 if bf16 else P.DIST_RTOL_F32, what=f"knn metric {metric}",
                         metric=metric)
    px.close()


@pytest.mark.parametrize("batch", [1, 7, 64, 256])
@pytest.mark.parametrize("metric,policy", [(po.METRIC_IP, po.POLICY_LRU), (po.METRIC_COSINE, po.POLICY_FIFO),
                                           (po.METRIC_COSINE, po.POLICY_LRU)])
def test_tiny_workload_other_metrics(B, tiny, batch, metric, policy):
    w, corpus, q, _ = tiny
    xc = corpus * lengths(len(corpus), 0.3, 3.0, 21)
    if metric == po.METRIC_COSINE:
        # queries of all lengths; two of the same base are about 0.14^2 / 2 apart in cosine distance
        qs, tau = (q * lengths(len(q), 0.5, 2.0, 22)).astype(np.float32), 0.02
    else:
        qs, tau = q, w.tau          # the cache of an inner-product index compares by Euclidean distance
    want = po.lookup_stream_deferred(xc, qs, tau, w.capacity, w.k, policy, rerank_factor=2, metric=metric)
    o_ids, o_d, o_hit, o_src, dec, stored = want
    assert 500 < o_hit.sum() < 900
    px = B.Proximity(gpu_corpus(xc), w.dim, w.capacity, w.k, policy, 256, rerank_factor=2, metric=metric)
    got = P.run_stream(px, qs, tau, batch, DEV)
    excused = P.assert_stream_parity(got, (o_ids, o_d, o_hit, o_src), xc, qs, what=f"metric {metric} b{batch}",
                                     reranked=True, metric=metric)
    assert excused == 0
    seq, keys, ids = px.cache_dump(want_keys=True, want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist()
    assert (ids == stored[seq]).all()
    assert (keys == qs[seq]).all()       # a key is the query as it came, under every distance function
    st = px.stats()
    assert st["hits"] == int(o_hit.sum()) and st["evictions"] == dec.n_evictions
    px.close()


def test_cache_under_other_metrics_hand_worked(B):
    """The stream of the oracle's pin of the same name: only the cosine cache hits."""
    qs = np.zeros((5, 32), np.float32)
    qs[:, :2] = [[1, 0], [5, 0], [0, 1], [0, 2], [3, 3]]
    corpus = W.corpus_f32(500, 32, 9) * lengths(500, 0.3, 3.0, 10)
    for metric, flags in ((po.METRIC_COSINE, "MHMHM"), (po.METRIC_L2, "MMMMM"), (po.METRIC_IP, "MMMMM")):
        o = po.FlatCacheOracle(corpus, 8, 3, po.POLICY_LRU, metric=metric)
        want = o.lookup_stream(qs, 0.1)
        assert "".join("H" if h else "M" for h in want[2]) == flags
        for batch in (1, 5):
            px = B.Proximity(gpu_corpus(corpus), 32, 8, 3, po.POLICY_LRU, 8, metric=metric)
            got = P.run_stream(px, qs, 0.1, batch, DEV)
            P.assert_stream_parity(got, want, corpus, qs, what=f"hand-worked metric {metric}", metric=metric)
            px.close()


@pytest.mark.parametrize("metric", [po.METRIC_IP, po.METRIC_COSINE])
def test_bucketed_cache_other_metrics(B, tiny, metric):
    w, corpus, q, _ = tiny
    xc = corpus * lengths(len(corpus), 0.3, 3.0, 21)
    qs = (q * lengths(len(q), 0.5, 2.0, 22)).astype(np.float32) if metric == po.METRIC_COSINE else q
    tau = 0.02 if metric == po.METRIC_COSINE else w.tau
    planes = W.lsh_planes(3, w.dim, 5)
    want = po.lookup_stream_deferred(xc, qs, tau, 8, w.k, po.POLICY_LRU, planes=planes, metric=metric)
    assert 300 < want[2].sum() < 900
    for batch in (1, 100):
        px = B.Proximity(gpu_corpus(xc), w.dim, 8, w.k, po.POLICY_LRU, 128,
                         lsh_planes=torch.from_numpy(planes).to(DEV), metric=metric)
        got = P.run_stream(px, qs, tau, batch, DEV)
        P.assert_stream_parity(got, want[:4], xc, qs, what=f"bucketed metric {metric} b{batch}", metric=metric)
        seq, _, _ = px.cache_dump()
        assert seq.tolist() == want[4].dump_seq().tolist()
        px.close()


# ---------------------------------------------------------------------------
# Re-ranking factor (Section 3.3.4)
# ---------------------------------------------------------------------------
_RERANK_WANT = {}   # oracle outputs per policy, computed once


@pytest.mark.parametrize("batch", [1, 7, 64, 256])
@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_tiny_workload_with_reranking(B, tiny, batch, policy):
    w, corpus, q, _ = tiny
    rho = 4
    if policy not in _RERANK_WANT:
        _RERANK_WANT[policy] = po.lookup_stream_deferred(corpus, q, w.tau, w.capacity, w.k, policy, rerank_factor=rho)
    o_ids, o_d, o_hit, o_src, dec, stored = _RERANK_WANT[policy]
    px = B.Proximity(gpu_corpus(corpus), w.dim, w.capacity, w.k, policy, 256, rerank_factor=rho)
    got = P.run_stream(px, q, w.tau, batch, DEV)
    excused = P.assert_stream_parity(got, (o_ids, o_d, o_hit, o_src), corpus, q, what=f"rho=4 b{batch}", reranked=True)
    assert excused == 0
    seq, _, ids = px.cache_dump(want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist()
    assert ids.shape[1] == rho * w.k and (ids == stored[seq]).all()
    # the re-ranked answers are not simply the stored lists' heads
    hit_rows = np.flatnonzero(o_hit == 1)
    assert (o_ids[hit_rows] != stored[o_src[hit_rows], :w.k]).any()
    px.close()


@pytest.mark.parametrize("batch", [1, 4])
def test_reranking_hand_worked_line(B, batch):
    """The line example of the oracle's pins: documents at 0..9, k=2, rho=2, tau=3."""
    corpus = line_vectors(range(10), dim=32)
    q = line_vectors([4.4, 5.6, 2.0, 4.5], dim=32)
    px = B.Proximity(gpu_corpus(corpus), 32, 4, 2, po.POLICY_FIFO, 4, rerank_factor=2)
    ids, dists, hit = P.run_stream(px, q, 3.0, batch, DEV)
    assert hit.tolist() == [0, 1, 1, 1]
    assert ids.tolist() == [[4, 5], [6, 5], [3, 4], [4, 5]]
    np.testing.assert_allclose(dists, [[0.4, 0.6], [0.4, 0.6], [1.0, 2.0], [0.5, 0.5]], rtol=1e-5)
    _, _, stored = px.cache_dump(want_ids=True)
    assert stored.tolist() == [[4, 5, 3, 6]]
    px.close()


def test_reranking_bf16_corpus_and_no_corpus(B):
    n_docs, dim, k, rho = 20000, 384, 10, 3
    x32 = W.corpus_f32(n_docs, dim, 9)
    xb = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x32))
    base = W.base_queries(40, dim, 3)
    idx = np.random.default_rng(1).integers(0, 40, size=300)
    q = W.perturbed_stream(base, idx, 0.05, 3)
    want = po.lookup_stream_deferred(xb, q, 0.2, 16, k, po.POLICY_LRU, rerank_factor=rho)
    px = B.Proximity(torch.from_numpy(x32).to(DEV).to(torch.bfloat16), dim, 16, k, po.POLICY_LRU, 64,
                     rerank_factor=rho)
    got = P.run_stream(px, q, 0.2, 64, DEV)
    P.assert_stream_parity(got, want[:4], xb, q, dist_rtol=P.DIST_RTOL_BF16, what="rho=3 bf16", reranked=True)
    assert want[2].sum() > 100
    px.close()
    px = B.Proximity(None, dim, 16, k, po.POLICY_LRU, 64, device=DEV, rerank_factor=rho)
    ids, dists, hit = P.run_stream(px, q, 0.2, 64, DEV)
    assert (hit == want[2]).all() and (ids == -1).all() and np.isinf(dists).all()
    px.close()


# ---------------------------------------------------------------------------
# Bucketed cache (Section 3.2)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("batch", [1, 6])
def test_lsh_hand_worked_buckets(B, batch):
    """The isolation example of the oracle's pins: one hyperplane, one entry per bucket, tau = 1.5."""
    planes = np.zeros((1, 32), dtype=np.float32)
    planes[0, 0] = 1.0
    q = line_vectors([0.5, -0.5, 0.6, -10.0, -0.6, 0.4], dim=32)
    corpus = line_vectors(range(-10, 10), dim=32)
    px = B.Proximity(gpu_corpus(corpus), 32, 1, 2, po.POLICY_FIFO, 8, lsh_planes=torch.from_numpy(planes).to(DEV))
    ids, _, hit = P.run_stream(px, q, 1.5, batch, DEV)
    assert "".join("H" if h else "M" for h in hit) == "MMHMMH"
    assert ids[0].tolist() == ids[2].tolist() == ids[5].tolist() == [10, 11]
    seq, keys, _ = px.cache_dump(want_keys=True)
    assert seq.tolist() == [4, 0] and (keys == q[[4, 0]]).all()
    st = px.stats()
    assert st["evictions"] == 2 and st["hits"] == 2 and st["size"] == 2 and st["queries"] == 6
    px.close()


_LSH_WANT = {}


@pytest.mark.parametrize("batch", [1, 7, 64, 256])
@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_tiny_workload_bucketed(B, tiny, batch, policy):
    w, corpus, q, _ = tiny
    planes = W.lsh_planes(3, w.dim, 2)
    if policy not in _LSH_WANT:
        _LSH_WANT[policy] = po.lookup_stream_deferred(corpus, q, w.tau, 6, w.k, policy, planes=planes)
    o_ids, o_d, o_hit, o_src, dec = _LSH_WANT[policy]
    assert 300 < o_hit.sum() < 697 and dec.n_evictions > 100
    px = B.Proximity(gpu_corpus(corpus), w.dim, 6, w.k, policy, 256, lsh_planes=torch.from_numpy(planes).to(DEV))
    got = P.run_stream(px, q, w.tau, batch, DEV)
    assert P.assert_stream_parity(got, (o_ids, o_d, o_hit, o_src), corpus, q, what=f"lsh b{batch}") == 0
    seq, _, ids = px.cache_dump(want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist()
    assert (ids == o_ids[seq]).all()
    st, os_ = px.stats(), dec.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == os_[key], key
    px.close()


def test_bucketed_with_reranking_and_clear(B, tiny):
    w, corpus, q, _ = tiny
    q = q[:400]
    planes = W.lsh_planes(2, w.dim, 5)
    want = po.lookup_stream_deferred(corpus, q, w.tau, 5, w.k, po.POLICY_LRU, planes=planes, rerank_factor=3)
    px = B.Proximity(gpu_corpus(corpus), w.dim, 5, w.k, po.POLICY_LRU, 64, rerank_factor=3,
                     lsh_planes=torch.from_numpy(planes).to(DEV))
    for _ in range(2):          # the second pass starts from a cleared cache and must repeat the first
        got = P.run_stream(px, q, w.tau, 64, DEV)
        P.assert_stream_parity(got, want[:4], corpus, q, what="lsh rho=3", reranked=True)
        seq, _, stored = px.cache_dump(want_ids=True)
        assert seq.tolist() == want[4].dump_seq().tolist() and (stored == want[5][seq]).all()
        px.clear()
        assert px.stats()["size"] == 0 and len(px.cache_dump()[0]) == 0
    px.close()


@pytest.mark.parametrize("dim,bits,b,batch", [
    (64, 16, 4, 512),       # the most hyperplanes
    (64, 1, 256, 300),      # the largest bucket
    (1024, 2, 64, 128),     # a bucket whose keys do not fit on chip: distances read from device memory
    (4096, 1, 3, 4),        # the largest dimension, calls of four rows
])
def test_bucketed_limits(B, dim, bits, b, batch):
    rng = np.random.default_rng(dim + bits)
    planes = W.lsh_planes(bits, dim, 3)
    n_bases = 150 if (b << bits) >= 100 else 8          # a cache of six entries wants a small working set
    base = W.unit_rows(rng.standard_normal((n_bases, dim)))
    idx = rng.integers(0, n_bases, size=1500)
    q = W.unit_rows(base[idx] + rng.choice([0.0, 0.1, 0.4], size=1500)[:, None]
                    * W.unit_rows(rng.standard_normal((1500, dim)))).astype(np.float32)
    corpus = W.corpus_f32(300, dim, 5)
    want = po.lookup_stream_deferred(corpus, q, 0.3, b, 2, po.POLICY_LRU, planes=planes)
    assert 100 < want[2].sum() < 1400
    px = B.Proximity(gpu_corpus(corpus), dim, b, 2, po.POLICY_LRU, 512, lsh_planes=torch.from_numpy(planes).to(DEV))
    got = P.run_stream(px, q, 0.3, batch, DEV)
    P.assert_stream_parity(got, want[:4], corpus, q, what=f"bucketed {dim}/{bits}/{b}")
    seq, _, _ = px.cache_dump()
    assert seq.tolist() == want[4].dump_seq().tolist()
    assert px.stats()["evictions"] == want[4].n_evictions
    px.close()


def test_bucketed_probe_at_scale_without_corpus(B):
    """1024 buckets of 20 entries, calls of 8192 rows: flags and cache contents against the oracle's decisions."""
    dim, bits, b, tau = 128, 10, 20, 0.4
    planes = W.lsh_planes(bits, dim, 7)
    rng = np.random.default_rng(17)
    fresh = W.unit_rows(rng.standard_normal((30000, dim)))
    near = W.unit_rows(fresh[rng.integers(0, 30000, size=10960)] + 0.25 * W.unit_rows(rng.standard_normal((10960, dim))))
    q = np.concatenate([fresh, near])[rng.permutation(40960)].astype(np.float32)
    o_hit, _, dec = po.simulate_decisions(q, tau, b, po.POLICY_LRU, planes=planes)
    assert 1000 < o_hit.sum() < 9000 and dec.n_evictions > 5000
    px = B.Proximity(None, dim, b, 4, po.POLICY_LRU, 8192, device=DEV, lsh_planes=torch.from_numpy(planes).to(DEV))
    _, _, hit = P.run_stream(px, q, tau, 8192, DEV)
    assert (hit == o_hit).all()
    seq, _, _ = px.cache_dump()
    assert seq.tolist() == dec.dump_seq().tolist()
    st, os_ = px.stats(), dec.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == os_[key], key
    px.close()


def test_tau_zero_and_tau_huge(B, tiny):
    w, corpus, q, _ = tiny
    q = q[:200]
    knn_ids, knn_d = po.batched_exact_knn(corpus, q, w.k)
    px = B.Proximity(gpu_corpus(corpus), w.dim, w.capacity, w.k, w.policy, 64)
    ids, dists, hit = P.run_stream(px, q, 0.0, 64, DEV)
    assert hit.sum() == 0
    P.assert_lists_match(ids, dists, knn_ids, knn_d, corpus, q, what="tau=0")
    px.clear()
    ids, dists, hit = P.run_stream(px, q, 1e9, 64, DEV)
    assert hit.tolist() == [0] + [1] * 199
    assert (ids == ids[0:1]).all() and (ids[0] == knn_ids[0]).all()
    st = px.stats()
    assert st["size"] == 1 and st["queries"] == 200
    px.close()


def test_repeated_vector_hits_at_tau_zero(B, tiny):
    w, corpus, q, _ = tiny
    stream = np.stack([q[0], q[1], q[0], q[1], q[0]])
    px = B.Proximity(gpu_corpus(corpus), w.dim, 4, w.k, po.POLICY_LRU, 8)
    for batch in (1, 5):
        px.clear()
        ids, dists, hit = P.run_stream(px, stream, 0.0, batch, DEV)
        assert hit.tolist() == [0, 0, 1, 1, 1]
        assert (ids[2] == ids[0]).all() and (ids[3] == ids[1]).all()
    px.close()


def test_many_candidates_take_the_dense_path(B):
    """Rows with more in-tolerance sources than the candidate list holds."""
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(2000, w.dim, 2)
    base = W.base_queries(3, w.dim, 8)
    idx = np.random.default_rng(0).integers(0, 3, size=400)
    q = W.perturbed_stream(base, idx, 0.1, 8)
    for policy, cap in ((po.POLICY_LRU, 2), (po.POLICY_FIFO, 2), (po.POLICY_LRU, 200)):
        want = po.lookup_stream_deferred(corpus, q, 0.25, cap, 5, policy)
        px = B.Proximity(gpu_corpus(corpus), w.dim, cap, 5, policy, 400)
        got = P.run_stream(px, q, 0.25, 400, DEV)
        P.assert_stream_parity(got, want[:4], corpus, q, what="dense path")
        seq, _, _ = px.cache_dump()
        assert seq.tolist() == want[4].dump_seq().tolist()
        assert px.stats()["dense_resolves"] > 0
        px.close()


def test_many_candidates_in_a_call_probed_in_row_ranges(B):
    """The same with 2 600 rows in one call: the probe goes in row ranges beside the resolver, a row near the end
    has hundreds of earlier rows within the tolerance, and the blocks of the listing probe run out of room for
    their (row, source) pairs, so rows reach the dense path both ways (list overflow, block overflow)."""
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(2000, w.dim, 2)
    base = W.base_queries(3, w.dim, 8)
    idx = np.random.default_rng(1).integers(0, 3, size=2600)
    q = W.perturbed_stream(base, idx, 0.1, 9)
    for policy, cap in ((po.POLICY_LRU, 2), (po.POLICY_FIFO, 300)):
        want = po.lookup_stream_deferred(corpus, q, 0.25, cap, 5, policy)
        px = B.Proximity(gpu_corpus(corpus), w.dim, cap, 5, policy, 2600)
        got = P.run_stream(px, q, 0.25, 2600, DEV)
        P.assert_stream_parity(got, want[:4], corpus, q, what="dense path, row ranges")
        seq, _, _ = px.cache_dump()
        assert seq.tolist() == want[4].dump_seq().tolist()
        assert px.stats()["dense_resolves"] > 1000
        px.close()


def test_no_corpus_and_no_cache(B):
    w = W.WORKLOADS["tiny"]
    q = W.stream_for(w, 40)
    px = B.Proximity(None, w.dim, 8, 4, po.POLICY_LRU, 16, device=DEV)
    ids, dists, hit = P.run_stream(px, q, 0.25, 16, DEV)
    o_hit, _, _ = po.simulate_decisions(q, 0.25, 8, po.POLICY_LRU)
    assert (hit == o_hit).all() and (ids == -1).all() and np.isinf(dists).all()
    px.close()
    corpus = W.corpus_f32(1000, w.dim, 1)
    px = B.Proximity(gpu_corpus(corpus), w.dim, 0, 4, po.POLICY_LRU, 16)
    ids, dists, hit = P.run_stream(px, q, 1e9, 16, DEV)
    assert hit.sum() == 0 and px.stats()["size"] == 0
    o_ids, o_d = po.batched_exact_knn(corpus, q, 4)
    P.assert_lists_match(ids, dists, o_ids, o_d, corpus, q, what="capacity 0")
    px.close()


def test_call_errors_leave_state_untouched(B, tiny):
    w, corpus, q, _ = tiny
    px = B.Proximity(gpu_corpus(corpus), w.dim, 4, w.k, po.POLICY_LRU, 8)
    qd = torch.from_numpy(q[:8]).to(DEV)
    ids = torch.empty((8, w.k), dtype=torch.int64, device=DEV)
    hit = torch.empty(8, dtype=torch.uint8, device=DEV)
    lib, h = B.lib, px.handle
    assert lib.proximity_search_batch(h, qd.data_ptr(), 8, w.k + 1, 0.1, ids.data_ptr(), None, hit.data_ptr(), None) == B.ERR_K_MISMATCH
    assert lib.proximity_search_batch(h, qd.data_ptr(), 9, w.k, 0.1, ids.data_ptr(), None, hit.data_ptr(), None) == B.ERR_BATCH_TOO_LARGE
    for bad in (float("nan"), float("inf"), -1.0):
        assert lib.proximity_search_batch(h, qd.data_ptr(), 8, w.k, bad, ids.data_ptr(), None, hit.data_ptr(), None) == B.ERR_BAD_TAU
    assert lib.proximity_search_batch(h, None, 8, w.k, 0.1, ids.data_ptr(), None, hit.data_ptr(), None) == B.ERR_INVALID_ARG
    assert lib.proximity_search_batch(h, qd.data_ptr(), 8, w.k, 0.1, ids.data_ptr(), None, None, None) == B.ERR_INVALID_ARG
    assert "out_hit" in B.last_error(h)
    # a pointer into the middle of a row: rows are read 16 bytes at a time, so it is turned away, not followed
    assert lib.proximity_search_batch(h, qd.data_ptr() + 4, 7, w.k, 0.1, ids.data_ptr(), None, hit.data_ptr(), None) == B.ERR_INVALID_ARG
    assert "aligned" in B.last_error(h)
    assert lib.proximity_knn_batch(h, qd.data_ptr() + 8, 7, w.k, ids.data_ptr(), None, None) == B.ERR_INVALID_ARG
    assert px.stats()["queries"] == 0
    assert lib.proximity_search_batch(h, qd.data_ptr(), 0, w.k, 0.1, None, None, None, None) == B.OK
    px.close()


def test_same_batch_three_times_is_bit_identical(B, tiny):
    w, corpus, q, _ = tiny
    outs = []
    for _ in range(3):
        px = B.Proximity(gpu_corpus(corpus), w.dim, w.capacity, w.k, w.policy, 128)
        outs.append(P.run_stream(px, q[:512], w.tau, 128, DEV))
        px.close()
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert (a == b).all()


def test_two_instances_interleaved(B, tiny):
    """Two handles alive at once, calls alternating between them: no state is shared."""
    w, corpus, q, want = tiny
    q = q[:384]
    planes = W.lsh_planes(2, w.dim, 9)
    want_b = po.lookup_stream_deferred(corpus, q, w.tau, 4, w.k, po.POLICY_FIFO, planes=planes, rerank_factor=2)
    corpus_dev = gpu_corpus(corpus)
    a = B.Proximity(corpus_dev, w.dim, w.capacity, w.k, po.POLICY_LRU, 64)
    b = B.Proximity(corpus_dev, w.dim, 4, w.k, po.POLICY_FIFO, 64, rerank_factor=2,
                    lsh_planes=torch.from_numpy(planes).to(DEV))
    outs_a, outs_b = [], []
    for r0 in range(0, len(q), 48):
        rows = torch.from_numpy(q[r0:r0 + 48]).to(DEV)
        outs_a.append(a.search_batch(rows, w.tau))
        outs_b.append(b.search_batch(rows, w.tau))
        outs_b.append(b.search_batch(rows[:0], w.tau))          # an empty call in between changes nothing
    cat = lambda outs, j: torch.cat([o[j] for o in outs]).cpu().numpy()
    o_ids, o_d, o_hit, o_src, _ = want[po.POLICY_LRU]
    P.assert_stream_parity((cat(outs_a, 0), cat(outs_a, 1), cat(outs_a, 2)),
                           (o_ids[:384], o_d[:384], o_hit[:384], o_src[:384]), corpus, q, what="instance a")
    P.assert_stream_parity((cat(outs_b, 0), cat(outs_b, 1), cat(outs_b, 2)), want_b[:4], corpus, q,
                           what="instance b", reranked=True)
    a.close()
    b.close()
