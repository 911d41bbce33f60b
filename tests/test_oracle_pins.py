"""Pins for the CPU oracle: checks against things other than the oracle itself.

Hand-worked eviction traces (tests/golden/eviction_streams.txt), reductions to
textbook exact-match FIFO/LRU caches, brute-force loops, library
nearest-neighbour routines and closed forms for the extreme tolerances.
"""
import collections
import math
import os

import numpy as np
import pytest

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def line_vectors(xs, dim=4):
    q = np.zeros((len(xs), dim), dtype=np.float32)
    q[:, 0] = np.asarray(xs, dtype=np.float32)
    return q


def read_eviction_cases():
    cases = []
    with open(os.path.join(GOLDEN, "eviction_streams.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, policy, cap, tau, xs, flags, ev, left, src = [p.strip() for p in line.split("|")]
            cases.append(dict(
                name=name, policy=po.POLICY_FIFO if policy == "FIFO" else po.POLICY_LRU,
                capacity=int(cap), tau=float(tau), xs=[float(v) for v in xs.split()],
                flags=flags, evictions=int(ev), left=[int(v) for v in left.split()],
                src=[int(v) for v in src.split()]))
    return cases


EVICTION_CASES = read_eviction_cases()


def small_corpus(n=64, dim=4, seed=3):
    return W.corpus_f32(n, dim, seed)


# ---------------------------------------------------------------------------
# Algorithm 1 + Section 3.3.2 against hand-worked traces
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", EVICTION_CASES, ids=[c["name"] for c in EVICTION_CASES])
def test_hand_worked_eviction_traces(case):
    corpus = small_corpus()
    orc = po.FlatCacheOracle(corpus, case["capacity"], 3, case["policy"])
    q = line_vectors(case["xs"])
    ids, dists, hit, src = orc.lookup_stream(q, case["tau"])
    assert "".join("H" if h else "M" for h in hit) == case["flags"]
    assert orc.n_evictions == case["evictions"]
    assert orc.dump_seq().tolist() == case["left"]
    assert src.tolist() == case["src"]
    # every returned list is the database result of the query named by `src`
    for t in range(len(q)):
        want, _ = po.exact_knn(corpus, q[src[t]], 3)
        assert ids[t].tolist() == want.tolist()


def test_two_similar_queries_walkthrough():
    """Section 3.1's example: q1 misses and is stored; a close q2 gets q1's indices."""
    corpus = small_corpus(200, 16, 5)
    rng = np.random.default_rng(11)
    q1 = rng.standard_normal(16).astype(np.float32)
    q2 = (q1 + 1e-3 * rng.standard_normal(16)).astype(np.float32)
    orc = po.FlatCacheOracle(corpus, 8, 5, po.POLICY_LRU)
    i1, _, h1, _ = orc.lookup(q1, 0.5)
    i2, _, h2, s2 = orc.lookup(q2, 0.5)
    assert (h1, h2, s2) == (False, True, 0)
    assert i1.tolist() == i2.tolist()
    assert orc.stats()["scans"] == 1


# ---------------------------------------------------------------------------
# The database call against brute force and library routines
# ---------------------------------------------------------------------------
def test_exact_knn_matches_pure_python_loops():
    rng = np.random.default_rng(0)
    corpus = rng.standard_normal((37, 5)).astype(np.float32)
    q = rng.standard_normal(5).astype(np.float32)
    d = []
    for j in range(37):
        acc = 0.0
        for i in range(5):
            diff = float(q[i]) - float(corpus[j, i])
            acc += diff * diff
        d.append((math.sqrt(acc), j))
    d.sort()
    ids, dists = po.exact_knn(corpus, q, 7)
    assert ids.tolist() == [j for _, j in d[:7]]
    np.testing.assert_allclose(dists, [v for v, _ in d[:7]], rtol=1e-14)


def test_exact_knn_matches_library_neighbours():
    from scipy.spatial.distance import cdist
    from sklearn.neighbors import NearestNeighbors

    rng = np.random.default_rng(1)
    corpus = rng.standard_normal((500, 24))
    queries = rng.standard_normal((6, 24))
    nn = NearestNeighbors(n_neighbors=9, algorithm="brute", metric="euclidean").fit(corpus)
    lib_d, lib_i = nn.kneighbors(queries)
    full = cdist(queries, corpus, metric="euclidean")
    for r in range(6):
        ids, dists = po.exact_knn(corpus, queries[r], 9)
        assert ids.tolist() == lib_i[r].tolist()
        np.testing.assert_allclose(dists, lib_d[r], rtol=1e-10)
        np.testing.assert_allclose(dists, np.sort(full[r])[:9], rtol=1e-12)


def test_unit_norm_ranking_is_inner_product_ranking():
    """For unit rows |q-x|^2 = 2 - 2 q.x, so L2 order is descending inner-product order."""
    corpus = W.corpus_f32(3000, 48, 7).astype(np.float64)
    corpus /= np.linalg.norm(corpus, axis=1, keepdims=True)
    q = W.base_queries(4, 48, 7)
    for r in range(4):
        ids, dists = po.exact_knn(corpus, q[r], 12)
        ip = corpus @ q[r]
        assert ids.tolist() == np.argsort(-ip, kind="stable")[:12].tolist()
        np.testing.assert_allclose(dists ** 2, 2.0 - 2.0 * ip[ids], rtol=0, atol=1e-12)


def test_exact_knn_ties_and_padding():
    corpus = np.zeros((6, 3), dtype=np.float32)
    corpus[:, 0] = [2, 1, 1, 5, 1, 2]          # three rows at distance 1, two at distance 2
    ids, dists = po.exact_knn(corpus, np.zeros(3, np.float32), 4)
    assert ids.tolist() == [1, 2, 4, 0]
    assert dists.tolist() == [1.0, 1.0, 1.0, 2.0]
    ids, dists = po.exact_knn(corpus, np.zeros(3, np.float32), 8)
    assert ids.tolist() == [1, 2, 4, 0, 5, 3, -1, -1]
    assert np.isinf(dists[6:]).all()
    ids, dists = po.exact_knn(None, np.zeros(3, np.float32), 2)
    assert ids.tolist() == [-1, -1] and np.isinf(dists).all()


def test_batched_knn_equals_literal_knn_including_ties():
    rng = np.random.default_rng(5)
    corpus = rng.standard_normal((700, 16)).astype(np.float32)
    corpus[100] = corpus[3]
    corpus[650] = corpus[3]
    queries = rng.standard_normal((9, 16)).astype(np.float32)
    queries[0] = corpus[3]                      # distance 0 to three identical rows
    b_ids, b_d = po.batched_exact_knn(corpus, queries, 11, chunk_rows=128)
    for r in range(9):
        ids, d = po.exact_knn(corpus, queries[r], 11)
        assert b_ids[r].tolist() == ids.tolist()
        np.testing.assert_allclose(b_d[r], d, rtol=1e-13, atol=1e-15)
    assert b_ids[0, :3].tolist() == [3, 100, 650]


def uneven_blocks(corpus, sizes):
    """(first_row, rows) blocks of the given sizes, in row order, covering the corpus."""
    r0 = 0
    for s in sizes:
        yield r0, corpus[r0:r0 + s]
        r0 += s
    assert r0 == len(corpus)


def test_knn_over_chunks_equals_literal_knn_on_uneven_blocks_with_ties():
    """The streamed form (Section 2.2's search over a corpus that arrives block by block) against the literal
    brute force: duplicated rows spread over several blocks, blocks smaller than k, a one-row last block, a
    query sitting on a duplicated row, and k larger than the corpus."""
    rng = np.random.default_rng(11)
    corpus = rng.standard_normal((331, 12)).astype(np.float32)
    for j in (40, 41, 97, 205, 330):           # five copies of row 7, the last one alone in the last block
        corpus[j] = corpus[7]
    corpus[300] = corpus[299]                   # a pair of equal rows inside one block
    queries = rng.standard_normal((7, 12)).astype(np.float32)
    queries[0] = corpus[7]                      # distance 0 to six identical rows
    queries[1] = corpus[299]
    sizes = [3, 5, 33, 1, 57, 100, 2, 64, 60, 5, 1]       # several blocks hold fewer than k rows
    for k in (1, 4, 9, 40):
        c_ids, c_d = po.exact_knn_over_chunks(uneven_blocks(corpus, sizes), queries, k)
        for r in range(len(queries)):
            ids, d = po.exact_knn(corpus, queries[r], k)
            assert c_ids[r].tolist() == ids.tolist(), (k, r)
            np.testing.assert_allclose(c_d[r], d, rtol=1e-13, atol=1e-15)
    c_ids, _ = po.exact_knn_over_chunks(uneven_blocks(corpus, sizes), queries, 9)
    assert c_ids[0, :6].tolist() == [7, 40, 41, 97, 205, 330]      # equal distances rank by index across blocks
    assert c_ids[1, :2].tolist() == [299, 300]
    # k larger than the corpus: every row ranked, then padding
    small = corpus[:6]
    c_ids, c_d = po.exact_knn_over_chunks(uneven_blocks(small, [2, 3, 1]), queries[:2], 9)
    for r in range(2):
        ids, d = po.exact_knn(small, queries[r], 9)
        assert c_ids[r].tolist() == ids.tolist() and c_ids[r, 6:].tolist() == [-1, -1, -1]
        assert np.isinf(c_d[r, 6:]).all()
        np.testing.assert_allclose(c_d[r, :6], d[:6], rtol=1e-13)


def test_knn_over_chunks_matches_library_neighbours():
    from sklearn.neighbors import NearestNeighbors

    rng = np.random.default_rng(12)
    corpus = rng.standard_normal((900, 20))
    queries = rng.standard_normal((5, 20))
    nn = NearestNeighbors(n_neighbors=13, algorithm="brute", metric="euclidean").fit(corpus)
    lib_d, lib_i = nn.kneighbors(queries)
    c_ids, c_d = po.exact_knn_over_chunks(uneven_blocks(corpus, [7, 300, 1, 292, 300]), queries, 13)
    assert (c_ids == lib_i).all()
    np.testing.assert_allclose(c_d, lib_d, rtol=1e-10)


# ---------------------------------------------------------------------------
# Extreme tolerances and counters
# ---------------------------------------------------------------------------
def test_zero_tolerance_never_hits_without_repeats_and_returns_exact_knn():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(2000, w.dim, w.seed)
    q = W.stream_for(w, 60)
    orc = po.FlatCacheOracle(corpus, 50, 10, po.POLICY_FIFO)
    ids, dists, hit, src = orc.lookup_stream(q, 0.0)
    assert hit.sum() == 0
    from sklearn.neighbors import NearestNeighbors
    nn = NearestNeighbors(n_neighbors=10, algorithm="brute").fit(corpus.astype(np.float64))
    lib_d, lib_i = nn.kneighbors(q.astype(np.float64))
    assert (ids == lib_i).all()
    np.testing.assert_allclose(dists, lib_d, rtol=1e-9)


def test_zero_tolerance_repeat_hits_and_still_returns_exact_knn():
    corpus = small_corpus(300, 8, 2)
    rng = np.random.default_rng(4)
    a, b = rng.standard_normal((2, 8)).astype(np.float32)
    orc = po.FlatCacheOracle(corpus, 4, 5, po.POLICY_LRU)
    ids, _, hit, _ = orc.lookup_stream(np.stack([a, b, a, b, a]), 0.0)
    assert hit.tolist() == [0, 0, 1, 1, 1]
    assert ids[2].tolist() == po.exact_knn(corpus, a, 5)[0].tolist()
    assert ids[3].tolist() == po.exact_knn(corpus, b, 5)[0].tolist()


def test_huge_tolerance_hits_everything_after_the_first_query():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(1500, w.dim, w.seed)
    q = W.stream_for(w, 40)
    for policy in (po.POLICY_FIFO, po.POLICY_LRU):
        orc = po.FlatCacheOracle(corpus, 3, 10, policy)
        ids, _, hit, src = orc.lookup_stream(q, 1e9)
        assert hit.tolist() == [0] + [1] * 39
        first = po.exact_knn(corpus, q[0], 10)[0]
        assert (ids == first[None, :]).all()
        assert (src == 0).all()


@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
@pytest.mark.parametrize("capacity", [1, 7, 500])
def test_counters_obey_algorithm_one(policy, capacity):
    w = W.WORKLOADS["tiny"]
    q = W.stream_for(w, 400)
    hit, src, orc = po.simulate_decisions(q, 0.25, capacity, policy)
    s = orc.stats()
    assert s["hits"] + s["misses"] == s["queries"] == 400
    assert s["misses"] == s["scans"] == s["inserts"]
    assert s["evictions"] == max(0, s["misses"] - capacity)
    assert s["size"] == min(capacity, s["misses"])
    assert int(hit.sum()) == s["hits"]


# ---------------------------------------------------------------------------
# Reduction to textbook exact-match caches
# ---------------------------------------------------------------------------
def textbook_cache_flags(keys, capacity, policy):
    """Hit/miss sequence of a classical exact-match FIFO or LRU cache over hashable keys."""
    store = collections.OrderedDict()
    flags = []
    for key in keys:
        if key in store:
            flags.append(1)
            if policy == po.POLICY_LRU:
                store.move_to_end(key)
        else:
            flags.append(0)
            if capacity > 0:
                if len(store) >= capacity:
                    store.popitem(last=False)
                store[key] = True
    return flags


@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_zero_tolerance_is_an_exact_match_cache(policy):
    """Section 3.3.3: tau = 0 is a cache with exact matching."""
    rng = np.random.default_rng(9)
    vocab = rng.standard_normal((40, 12)).astype(np.float32)
    which = rng.integers(0, 40, size=600)
    hit, _, _ = po.simulate_decisions(vocab[which], 0.0, 9, policy)
    assert hit.tolist() == textbook_cache_flags(which.tolist(), 9, policy)


@pytest.mark.parametrize("name", ["tiny"])
def test_tiny_stream_reduces_to_cache_over_base_ids(name):
    """Rewordings of one base lie ~0.14 apart, different bases > 1.2 apart, so at
    tau = 0.25 the approximate cache behaves as an exact-match cache keyed by base id."""
    w = W.WORKLOADS[name]
    idx = W.zipf_choice(w.n_stream, w.n_bases, w.zipf_s, w.seed)
    q = W.stream_for(w)
    for policy in (po.POLICY_FIFO, po.POLICY_LRU):
        hit, _, orc = po.simulate_decisions(q, w.tau, w.capacity, policy)
        assert hit.tolist() == textbook_cache_flags(idx.tolist(), w.capacity, policy)
    hit, _, orc = po.simulate_decisions(q, w.tau, w.capacity, w.policy)
    # counts an independent simulation of this recipe also reached
    assert int(hit.sum()) == 697 and orc.n_evictions == 253
    assert "".join(str(int(h)) for h in hit[:16]) == "0001101100100010"
    hit0, _, orc0 = po.simulate_decisions(q, 0.1, w.capacity, w.policy)
    assert int(hit0.sum()) == 0 and orc0.n_evictions == 950


# ---------------------------------------------------------------------------
# Deferred-scan form equals the literal form
# ---------------------------------------------------------------------------
def test_deferred_form_equals_literal_form():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(4000, w.dim, w.seed)
    q = W.stream_for(w, 300)
    for policy, cap in ((po.POLICY_FIFO, 50), (po.POLICY_LRU, 20)):
        lit = po.FlatCacheOracle(corpus, cap, 10, policy)
        ids, dists, hit, src = lit.lookup_stream(q, 0.25)
        d_ids, d_dists, d_hit, d_src, dec = po.lookup_stream_deferred(corpus, q, 0.25, cap, 10, policy)
        assert (hit == d_hit).all() and (src == d_src).all()
        assert (ids == d_ids).all()
        np.testing.assert_allclose(dists, d_dists, rtol=1e-13)
        assert dec.dump_seq().tolist() == lit.dump_seq().tolist()


# ---------------------------------------------------------------------------
# Re-ranking factor (Section 3.3.4)
# ---------------------------------------------------------------------------
def test_rerank_factor_one_is_the_plain_procedure():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(2000, w.dim, w.seed)
    q = W.stream_for(w, 200)
    a = po.FlatCacheOracle(corpus, 20, 10, po.POLICY_LRU).lookup_stream(q, 0.25)
    b = po.FlatCacheOracle(corpus, 20, 10, po.POLICY_LRU, rerank_factor=1).lookup_stream(q, 0.25)
    for x, y in zip(a, b):
        assert (x == y).all()


def test_rerank_hand_worked_line():
    """Documents at 0,1,..,9 on a line, k=2, rho=2 (4 stored per key), tau=3, capacity 4.
    q=4.4 misses: stores [4,5,3,6] (distances .4,.6,1.4,1.6), returns [4,5].
    q=5.6 hits (1.2 away): of the stored 4,5,3,6 the nearest are 6 (.4) and 5 (.6) -> [6,5].
    q=2.0 hits (2.4 away): nearest of the stored are 3 (1.0), then 4 (2.0) -> [3,4]; the true
    neighbours 2 and 1 are not among the stored and cannot come back.
    q=4.5 hits: 4 and 5 tie at .5 -> lower index first -> [4,5]."""
    corpus = line_vectors(range(10))
    orc = po.FlatCacheOracle(corpus, 4, 2, po.POLICY_FIFO, rerank_factor=2)
    ids, dists, hit, _ = orc.lookup_stream(line_vectors([4.4, 5.6, 2.0, 4.5]), 3.0)
    assert hit.tolist() == [0, 1, 1, 1]
    assert ids.tolist() == [[4, 5], [6, 5], [3, 4], [4, 5]]
    np.testing.assert_allclose(dists, [[0.4, 0.6], [0.4, 0.6], [1.0, 2.0], [0.5, 0.5]], rtol=1e-6)
    assert orc.dump_ids().tolist() == [[4, 5, 3, 6]]


def test_rerank_of_the_whole_index_is_exact_search():
    """When rho * k covers every document, a hit re-ranks the whole index: its answer is the exact
    k-NN of the current query, whatever key it matched."""
    sk = pytest.importorskip("sklearn.neighbors")
    corpus = small_corpus(40, 8, 5)
    rng = np.random.default_rng(9)
    q = rng.standard_normal((30, 8)).astype(np.float32)
    orc = po.FlatCacheOracle(corpus, 3, 5, po.POLICY_LRU, rerank_factor=8)     # 8 * 5 = 40 = N
    ids, dists, hit, _ = orc.lookup_stream(q, 1e9)
    assert hit.tolist() == [0] + [1] * 29
    nn = sk.NearestNeighbors(n_neighbors=5, algorithm="brute").fit(corpus.astype(np.float64))
    want_d, want_i = nn.kneighbors(q.astype(np.float64))
    assert (ids == want_i).all()
    np.testing.assert_allclose(dists, want_d, rtol=1e-12)


def test_rerank_matches_pure_python_and_keeps_to_the_stored_documents():
    corpus = small_corpus(500, 6, 7)
    rng = np.random.default_rng(10)
    base = rng.standard_normal(6)
    q = (base[None, :] + 0.3 * rng.standard_normal((25, 6))).astype(np.float32)
    k, rho = 4, 3
    orc = po.FlatCacheOracle(corpus, 2, k, po.POLICY_FIFO, rerank_factor=rho)
    ids, dists, hit, src = orc.lookup_stream(q, 1e9)
    stored = po.exact_knn(corpus, q[0], k * rho)[0].tolist()
    assert ids[0].tolist() == stored[:k]                         # a miss hands out the first k of what it stores
    for t in range(1, 25):
        assert hit[t] == 1 and src[t] == 0
        scored = []
        for j in stored:                                         # plain loops: distance of q[t] to each stored document
            s = 0.0
            for a, b in zip(q[t].tolist(), corpus[j].tolist()):
                s += (float(np.float32(a)) - float(np.float32(b))) ** 2
            scored.append((math.sqrt(s), j))
        scored.sort()
        assert ids[t].tolist() == [j for _, j in scored[:k]]
        np.testing.assert_allclose(dists[t], [d for d, _ in scored[:k]], rtol=1e-12)


def test_rerank_deferred_form_equals_literal_form():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(3000, w.dim, w.seed)
    q = W.stream_for(w, 250)
    for policy, cap in ((po.POLICY_FIFO, 30), (po.POLICY_LRU, 10)):
        lit = po.FlatCacheOracle(corpus, cap, 5, policy, rerank_factor=4)
        ids, dists, hit, src = lit.lookup_stream(q, 0.25)
        d_ids, d_dists, d_hit, d_src, dec, stored = po.lookup_stream_deferred(corpus, q, 0.25, cap, 5, policy,
                                                                              rerank_factor=4)
        assert (hit == d_hit).all() and (src == d_src).all() and (ids == d_ids).all()
        np.testing.assert_allclose(dists, d_dists, rtol=1e-13)
        assert (lit.dump_ids() == stored[lit.dump_seq()]).all()
        assert hit.sum() > 50


# ---------------------------------------------------------------------------
# Bucketed variant (Section 3.2)
# ---------------------------------------------------------------------------
def test_lsh_code_by_hand_and_by_loops():
    planes = np.zeros((2, 4), dtype=np.float32)
    planes[0, 0] = 1.0                       # bit 0: first coordinate >= 0
    planes[1, 1] = 1.0                       # bit 1: second coordinate >= 0
    for vec, code in (((1, 1), 3), ((-1, 1), 2), ((1, -1), 1), ((-1, -1), 0), ((0, -1), 1), ((-2, 0), 2)):
        q = np.zeros(4, dtype=np.float32)
        q[:2] = vec
        assert po.lsh_bucket(q, planes) == code
    rng = np.random.default_rng(3)
    planes = W.lsh_planes(7, 16, 1)
    for q in rng.standard_normal((50, 16)).astype(np.float32):
        code = 0
        for i in range(7):
            s = 0.0
            for a, b in zip(q.tolist(), planes[i].tolist()):
                s += a * b
            if s >= 0:
                code += 2 ** i
        assert po.lsh_bucket(q, planes) == code
    assert po.lsh_bucket(rng.standard_normal(16), np.zeros((0, 16))) == 0


def test_lsh_hand_worked_buckets_are_isolated():
    """One hyperplane (sign of the first coordinate), one entry per bucket, tau = 1.5.
    0.5 M (bucket +); -0.5 M (1.0 from 0.5, but the other bucket); 0.6 H; -10 M evicts -0.5 in bucket -;
    -0.6 M (its bucket now holds only -10) evicts -10; 0.4 H (bucket + was never disturbed).
    A single flat cache of the same total size would have hit on the second query."""
    planes = np.zeros((1, 4), dtype=np.float32)
    planes[0, 0] = 1.0
    xs = [0.5, -0.5, 0.6, -10.0, -0.6, 0.4]
    q = line_vectors(xs)
    corpus = line_vectors(range(-10, 10))
    orc = po.LshCacheOracle(corpus, planes, 1, 2, po.POLICY_FIFO)
    ids, _, hit, src = orc.lookup_stream(q, 1.5)
    assert "".join("H" if h else "M" for h in hit) == "MMHMMH"
    assert src.tolist() == [0, 1, 0, 3, 4, 0]
    assert orc.stats()["evictions"] == 2 and orc.dump_seq().tolist() == [4, 0]   # bucket 0 (negative side) first
    assert ids[2].tolist() == ids[0].tolist() == [10, 11]                         # documents 0 and 1 sit at rows 10, 11
    flat = po.FlatCacheOracle(corpus, 2, 2, po.POLICY_FIFO)
    assert flat.lookup_stream(q, 1.5)[2].tolist()[:2] == [0, 1]


def test_lsh_without_hyperplanes_is_the_flat_cache():
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(1500, w.dim, w.seed)
    q = W.stream_for(w, 300)
    for policy in (po.POLICY_FIFO, po.POLICY_LRU):
        a = po.FlatCacheOracle(corpus, 12, 5, policy).lookup_stream(q, 0.25)
        lsh = po.LshCacheOracle(corpus, np.zeros((0, w.dim)), 12, 5, policy)
        b = lsh.lookup_stream(q, 0.25)
        for x, y in zip(a, b):
            assert (x == y).all()


@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_lsh_equals_one_flat_cache_per_code(policy):
    """Splitting the stream by hash code beforehand and giving each part to its own flat cache is the same thing."""
    w = W.WORKLOADS["tiny"]
    corpus = W.corpus_f32(1200, w.dim, w.seed)
    q = W.stream_for(w, 400)
    planes = W.lsh_planes(3, w.dim, 0)
    codes = ((q.astype(np.float64) @ planes.astype(np.float64).T) >= 0).astype(np.int64) @ (1 << np.arange(3))
    lsh = po.LshCacheOracle(corpus, planes, 4, 5, policy)
    ids, dists, hit, src = lsh.lookup_stream(q, 0.25)
    assert len(set(codes.tolist())) > 3 and 30 < hit.sum() < 390
    for code in sorted(set(codes.tolist())):
        rows = np.flatnonzero(codes == code)
        f_ids, f_d, f_hit, f_src = po.FlatCacheOracle(corpus, 4, 5, policy).lookup_stream(q[rows], 0.25)
        assert (hit[rows] == f_hit).all() and (ids[rows] == f_ids).all()
        assert (src[rows] == rows[f_src]).all()                 # positions within the part map back to the stream


@pytest.mark.parametrize("policy", [po.POLICY_FIFO, po.POLICY_LRU])
def test_lsh_zero_tolerance_is_a_set_associative_cache(policy):
    """tau = 0: a textbook b-way set-associative cache keyed by vector identity, set = hash code."""
    rng = np.random.default_rng(8)
    vecs = rng.standard_normal((60, 8)).astype(np.float32)
    planes = W.lsh_planes(2, 8, 4)
    which = rng.integers(0, 60, size=500)
    sets = {}
    want = []
    for key in which.tolist():
        code = po.lsh_bucket(vecs[key], planes)
        way = sets.setdefault(code, collections.OrderedDict())
        if key in way:
            want.append(1)
            if policy == po.POLICY_LRU:
                way.move_to_end(key)
        else:
            want.append(0)
            if len(way) >= 3:
                way.popitem(last=False)
            way[key] = True
    hit, _, _ = po.simulate_decisions(vecs[which], 0.0, 3, policy, planes=planes)
    assert hit.tolist() == want and 50 < sum(want) < 450


# ---------------------------------------------------------------------------
# Other distance functions (Section 2.2: Euclidean, inner product or cosine)
# ---------------------------------------------------------------------------
def scaled_corpus(n, dim, seed):
    """Rows of very different lengths, so that the three distance functions rank differently."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, dim)) * rng.uniform(0.2, 5.0, size=(n, 1))).astype(np.float32)


def test_metric_distances_by_hand():
    q = np.array([1.0, 0.0])
    rows = np.array([[2.0, 0.0], [0.0, 3.0], [-1.0, 0.0], [1.0, 1.0]])
    np.testing.assert_allclose(po.metric_distances(q, rows, po.METRIC_COSINE),
                               [0.0, 1.0, 2.0, 1.0 - 1.0 / math.sqrt(2.0)], atol=1e-15)
    np.testing.assert_allclose(po.metric_distances(q, rows, po.METRIC_IP), [-2.0, 0.0, 1.0, -1.0], atol=0)
    np.testing.assert_allclose(po.metric_distances(q, rows, po.METRIC_L2),
                               [1.0, math.sqrt(10.0), 2.0, 1.0], atol=1e-15)
    # ranked lists: cosine and inner product agree here, Euclidean does not
    assert po.exact_knn(rows, q, 4, metric=po.METRIC_COSINE)[0].tolist() == [0, 3, 1, 2]
    assert po.exact_knn(rows, q, 4, metric=po.METRIC_IP)[0].tolist() == [0, 3, 1, 2]
    assert po.exact_knn(rows, q, 4, metric=po.METRIC_L2)[0].tolist() == [0, 3, 2, 1]
    # the cache of an inner-product index compares by Euclidean distance
    np.testing.assert_allclose(po.key_distances(q, rows, po.METRIC_IP), po.l2_distances(q, rows), atol=0)
    np.testing.assert_allclose(po.key_distances(q, rows, po.METRIC_COSINE),
                               po.metric_distances(q, rows, po.METRIC_COSINE), atol=0)


def test_metric_knn_matches_pure_python_loops():
    corpus = scaled_corpus(41, 6, 2)
    q = np.random.default_rng(3).standard_normal(6).astype(np.float32)
    cos, ip = [], []
    for j in range(41):
        dot = xx = qq = 0.0
        for i in range(6):
            dot += float(q[i]) * float(corpus[j, i])
            xx += float(corpus[j, i]) ** 2
            qq += float(q[i]) ** 2
        cos.append((1.0 - dot / (math.sqrt(xx) * math.sqrt(qq)), j))
        ip.append((-dot, j))
    for metric, ref in ((po.METRIC_COSINE, sorted(cos)), (po.METRIC_IP, sorted(ip))):
        ids, dists = po.exact_knn(corpus, q, 9, metric=metric)
        assert ids.tolist() == [j for _, j in ref[:9]]
        np.testing.assert_allclose(dists, [v for v, _ in ref[:9]], rtol=1e-13, atol=1e-15)


def test_metric_knn_matches_library_neighbours():
    from scipy.spatial.distance import cdist
    from sklearn.neighbors import NearestNeighbors

    corpus = scaled_corpus(600, 20, 4).astype(np.float64)
    queries = np.random.default_rng(5).standard_normal((5, 20)) * 3.0
    nn = NearestNeighbors(n_neighbors=8, algorithm="brute", metric="cosine").fit(corpus)
    lib_d, lib_i = nn.kneighbors(queries)
    full = cdist(queries, corpus, metric="cosine")
    for r in range(5):
        ids, dists = po.exact_knn(corpus, queries[r], 8, metric=po.METRIC_COSINE)
        assert ids.tolist() == lib_i[r].tolist()
        np.testing.assert_allclose(dists, lib_d[r], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(dists, np.sort(full[r])[:8], rtol=1e-9, atol=1e-12)
        ids, dists = po.exact_knn(corpus, queries[r], 8, metric=po.METRIC_IP)
        prod = corpus @ queries[r]
        assert ids.tolist() == np.argsort(-prod, kind="stable")[:8].tolist()
        np.testing.assert_allclose(dists, -np.sort(prod)[::-1][:8], rtol=1e-12)
    b_ids, b_d = po.batched_exact_knn(corpus, queries, 8, chunk_rows=128, metric=po.METRIC_COSINE)
    assert b_ids.tolist() == lib_i.tolist()
    np.testing.assert_allclose(b_d, lib_d, rtol=1e-9, atol=1e-12)
    b_ids, _ = po.batched_exact_knn(corpus, queries, 8, chunk_rows=128, metric=po.METRIC_IP)
    assert b_ids.tolist() == [np.argsort(-(corpus @ queries[r]), kind="stable")[:8].tolist() for r in range(5)]


def test_cosine_properties():
    """Cosine distance ignores lengths, and on unit vectors it is half the squared Euclidean distance."""
    corpus = scaled_corpus(300, 16, 6).astype(np.float64)
    q = np.random.default_rng(7).standard_normal(16)
    d = po.metric_distances(q, corpus, po.METRIC_COSINE)
    scale = np.random.default_rng(8).uniform(0.1, 9.0, size=(300, 1))
    np.testing.assert_allclose(po.metric_distances(4.5 * q, corpus * scale, po.METRIC_COSINE), d, rtol=0, atol=1e-14)
    unit = corpus / np.linalg.norm(corpus, axis=1, keepdims=True)
    qu = q / np.linalg.norm(q)
    np.testing.assert_allclose(d, po.l2_distances(qu, unit) ** 2 / 2.0, rtol=0, atol=1e-14)
    assert (d >= -1e-15).all() and (d <= 2.0 + 1e-15).all()
    # on unit vectors all three distance functions rank alike
    want = po.exact_knn(unit, qu, 15)[0].tolist()
    assert po.exact_knn(unit, qu, 15, metric=po.METRIC_COSINE)[0].tolist() == want
    assert po.exact_knn(unit, qu, 15, metric=po.METRIC_IP)[0].tolist() == want


def test_cosine_distance_of_identical_vectors_is_exactly_zero():
    """Section 3.3.3: a tolerance of 0 is exact matching, so a vector must be at distance exactly 0 from a
    bit-identical copy of itself (and, the formula being free of lengths, from its multiples by powers of two,
    which scale every term exactly) -- for every vector, not just for lucky roundings."""
    rng = np.random.default_rng(31)
    for dim in (4, 33, 384, 768):
        v = (rng.standard_normal((400, dim)) * rng.uniform(1e-3, 1e3, size=(400, 1))).astype(np.float32)
        for r in range(0, 400, 7):
            d = po.metric_distances(v[r], v[r:r + 1], po.METRIC_COSINE)
            assert d[0] == 0.0
            assert po.metric_distances(v[r], 4.0 * v[r:r + 1], po.METRIC_COSINE)[0] == 0.0
            assert po.metric_distances(0.5 * v[r], v[r:r + 1], po.METRIC_COSINE)[0] == 0.0
        # and nothing else is at zero: the nearest other row is clearly away
        d = po.metric_distances(v[0], v[1:], po.METRIC_COSINE)
        assert d.min() > 1e-3
    # an exact-match cache under cosine: repeats hit at tau = 0, whatever their power-of-two length
    vocab = rng.standard_normal((30, 24)).astype(np.float32)
    which = rng.integers(0, 30, size=500)
    q = vocab[which] * rng.choice([0.5, 1.0, 2.0, 8.0], size=(500, 1)).astype(np.float32)
    for policy in (po.POLICY_FIFO, po.POLICY_LRU):
        hit, _, _ = po.simulate_decisions(q, 0.0, 7, policy, metric=po.METRIC_COSINE)
        assert hit.tolist() == textbook_cache_flags(which.tolist(), 7, policy)


def test_cache_under_other_metrics_hand_worked():
    """(1,0), (5,0), (0,1), (0,2), (3,3) with tau = 0.1 and room for every key: the second and fourth
    query point the same way as the one before them, so the cosine cache hits on both although they
    are far away; the Euclidean cache, and with it the cache of an inner-product index, hits on neither."""
    qs = np.array([[1, 0], [5, 0], [0, 1], [0, 2], [3, 3]], dtype=np.float32)
    qs = np.concatenate([qs, np.zeros((5, 2), np.float32)], axis=1)
    corpus = scaled_corpus(50, 4, 9)
    for metric, flags in ((po.METRIC_COSINE, "MHMHM"), (po.METRIC_L2, "MMMMM"), (po.METRIC_IP, "MMMMM")):
        o = po.FlatCacheOracle(corpus, 8, 3, po.POLICY_LRU, metric=metric)
        ids, dists, hit, src = o.lookup_stream(qs, 0.1)
        assert "".join("H" if h else "M" for h in hit) == flags
        for t in range(5):
            own_ids, own_d = po.exact_knn(corpus, qs[src[t]], 3, metric=metric)
            assert ids[t].tolist() == own_ids.tolist()
            np.testing.assert_allclose(dists[t], own_d, rtol=0, atol=0)
    # the hit at position 1 returns what (1,0) stored; under cosine that is also (5,0)'s own answer
    o = po.FlatCacheOracle(corpus, 8, 3, po.POLICY_LRU, metric=po.METRIC_COSINE)
    ids, _, _, _ = o.lookup_stream(qs, 0.1)
    assert ids[1].tolist() == po.exact_knn(corpus, qs[1], 3, metric=po.METRIC_COSINE)[0].tolist()


@pytest.mark.parametrize("metric", [po.METRIC_IP, po.METRIC_COSINE])
def test_metric_deferred_form_equals_literal_form(metric):
    w = W.WORKLOADS["tiny"]
    corpus = scaled_corpus(3000, w.dim, 10)
    q = W.stream_for(w, 260) * np.random.default_rng(11).uniform(0.5, 2.0, size=(260, 1)).astype(np.float32)
    tau = 0.25 if metric == po.METRIC_IP else 0.012
    lit = po.FlatCacheOracle(corpus, 20, 5, po.POLICY_LRU, rerank_factor=2, metric=metric)
    l_ids, l_d, l_hit, l_src = lit.lookup_stream(q, tau)
    d_ids, d_d, d_hit, d_src, dec, _ = po.lookup_stream_deferred(corpus, q, tau, 20, 5, po.POLICY_LRU,
                                                                rerank_factor=2, metric=metric)
    assert 20 < l_hit.sum() < 240
    assert (l_hit == d_hit).all() and (l_src == d_src).all() and (l_ids == d_ids).all()
    np.testing.assert_allclose(l_d, d_d, rtol=1e-12, atol=1e-14)
    assert dec.dump_seq().tolist() == lit.dump_seq().tolist()


# ---------------------------------------------------------------------------
# Input generators (recipe checks, not method arithmetic)
# ---------------------------------------------------------------------------
def test_generator_recipe_is_stable():
    w = W.WORKLOADS["tiny"]
    idx = W.zipf_choice(w.n_stream, w.n_bases, w.zipf_s, w.seed)
    assert idx[:16].tolist() == [0, 3, 12, 0, 0, 2, 0, 3, 5, 1, 5, 74, 16, 19, 0, 76]
    q = W.stream_for(w, 8)
    np.testing.assert_allclose(q[0, :4], [0.00262298, -0.03258461, -0.02650609, -0.03384795], atol=2e-8)
    np.testing.assert_allclose(np.linalg.norm(q.astype(np.float64), axis=1), 1.0, atol=1e-6)
    assert (W.stream_for(w, 8) == W.stream_for(w)[:8]).all()
    x = W.corpus_f32(100, 32, 1, chunk_rows=7)
    assert (x == W.corpus_f32(100, 32, 1)).all()


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-39, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8],
                 dtype=np.float32)
    bits = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(bits)
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert (back == ref).all()
