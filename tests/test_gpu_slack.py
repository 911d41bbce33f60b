"""The exactness check of the index search (Section 2.2 asks for the exact ranked list of the k nearest rows):
float32 scores pick k + 8 candidates, float64 distances rank them, and a query whose candidate list cannot be
proven to hold the k nearest under the float32 error bound is ranked again from every row within that bound.
The corpora here are built so that float32 cannot tell the rows around the k-th apart: the answers must still
be the oracle's, id for id, and the counters must show that the second ranking ran."""
import numpy as np
import pytest
import torch

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


@pytest.fixture(scope="module")
def B():
    import paper_2503_05530_amd.binding as b
    return b


def crowded_corpus(n_docs, dim, n_near, spread, seed):
    """Unit Gaussian rows of which n_near, scattered over the corpus, are copies of one row displaced by
    `spread` per element (float32 values; spread = 0 gives exact duplicates)."""
    rng = np.random.default_rng(seed)
    x = W.corpus_f32(n_docs, dim, seed)
    where = np.sort(rng.choice(n_docs, size=n_near, replace=False))
    centre = x[where[0]].astype(np.float64)
    x[where] = (centre[None, :] + spread * rng.standard_normal((n_near, dim))).astype(np.float32)
    return x, where, centre


@pytest.mark.parametrize("n_queries", [1, 3, 24, 70, 128])
@pytest.mark.parametrize("dim,k", [(64, 10), (768, 10), (384, 32)])
def test_rows_float32_cannot_tell_apart_are_ranked_exactly(B, n_queries, dim, k):
    """A hundred rows within 3e-8 per element of each other, the queries a small step away from them: their
    distances to a query differ in the ninth digit, so the k nearest are decided among them by float64 alone,
    and the float32 candidate list (k + 8, or the longer one of a scan on rounded operands) is an arbitrary
    subset of the hundred."""
    x, where, centre = crowded_corpus(7000, dim, 100, 3e-8, 50 + dim)
    rng = np.random.default_rng(7)
    q = (centre[None, :] + 0.02 * W.unit_rows(rng.standard_normal((n_queries, dim)))).astype(np.float32)
    o_ids, o_d = po.batched_exact_knn(x, q, k)
    assert np.isin(o_ids, where).all()                      # the answer lies inside the crowd
    px = B.Proximity(torch.from_numpy(x).to(DEV), dim, 0, k, B.POLICY_FIFO, max(n_queries, 4))
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    torch.cuda.synchronize(DEV)
    st = px.stats()
    assert (ids.cpu().numpy() == o_ids).all()
    np.testing.assert_allclose(dists.cpu().numpy(), o_d, rtol=1e-6)
    assert st["slack_exhausted"] == n_queries and st["slack_unresolved"] == 0
    # a second call on the same instance: the device-side list of noted queries was cleared
    ids2, _ = px.knn_batch(torch.from_numpy(q).to(DEV))
    assert (ids2.cpu().numpy() == o_ids).all()
    assert px.stats()["slack_exhausted"] == 2 * n_queries and px.stats()["slack_unresolved"] == 0
    # through the cache as well: misses take the same search, hits return the stored exact lists
    both = np.concatenate([q, q])                            # every query once more: exact repeats hit
    pc = B.Proximity(torch.from_numpy(x).to(DEV), dim, len(both), k, B.POLICY_LRU, len(both))
    ids3, _, hit = pc.search_batch(torch.from_numpy(both).to(DEV), 1e-4)
    want = po.lookup_stream_deferred(x, both, 1e-4, len(both), k, po.POLICY_LRU)
    assert want[2].sum() == n_queries
    assert (hit.cpu().numpy() == want[2]).all() and (ids3.cpu().numpy() == want[0]).all()
    assert pc.stats()["slack_exhausted"] > 0 and pc.stats()["slack_unresolved"] == 0
    px.close()
    pc.close()


@pytest.mark.parametrize("metric", [po.METRIC_IP, po.METRIC_COSINE])
@pytest.mark.parametrize("n_queries", [2, 40])
def test_crowded_rows_under_the_other_distance_functions(B, metric, n_queries):
    dim, k = 128, 7
    x, where, centre = crowded_corpus(5000, dim, 30, 3e-8, 61)
    rng = np.random.default_rng(8)
    q = (1.7 * (centre[None, :] + 0.02 * W.unit_rows(rng.standard_normal((n_queries, dim))))).astype(np.float32)
    o_ids, o_d = po.batched_exact_knn(x, q, k, metric=metric)
    px = B.Proximity(torch.from_numpy(x).to(DEV), dim, 0, k, B.POLICY_FIFO, max(n_queries, 4), metric=metric)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    assert (ids.cpu().numpy() == o_ids).all()
    np.testing.assert_allclose(dists.cpu().numpy(), o_d, rtol=1e-5, atol=1e-9)
    st = px.stats()
    assert st["slack_exhausted"] > 0 and st["slack_unresolved"] == 0
    px.close()


@pytest.mark.parametrize("n_queries", [2, 128])
def test_duplicated_documents_in_a_bfloat16_corpus(B, n_queries):
    """Eighty identical rows (bfloat16 cannot hold nearer-than-identical neighbours; more of them than the longest
    candidate list, k + 32 on the one-plane scan): equal distances rank by index, on the matrix-core scan and on
    the streaming scan alike."""
    dim, k = 384, 20
    x, where, centre = crowded_corpus(9000, dim, 80, 0.0, 62)
    x16 = torch.from_numpy(x).to(DEV).to(torch.bfloat16)
    xh = x16.to(torch.float32).cpu().numpy()
    rng = np.random.default_rng(9)
    q = (centre[None, :] + 0.05 * W.unit_rows(rng.standard_normal((n_queries, dim)))).astype(np.float32)
    o_ids, _ = po.batched_exact_knn(xh, q, k)
    assert (o_ids == where[None, :k]).all()
    px = B.Proximity(x16, dim, 0, k, B.POLICY_FIFO, max(n_queries, 4))
    ids, _ = px.knn_batch(torch.from_numpy(q).to(DEV))
    assert (ids.cpu().numpy() == o_ids).all()
    st = px.stats()
    assert st["slack_exhausted"] == n_queries and st["slack_unresolved"] == 0
    px.close()


def test_a_crowd_larger_than_the_second_ranking_holds_is_counted(B):
    """Three thousand identical rows: more than the 2 048 the second ranking collects per query."""
    dim, k = 64, 5
    x, where, centre = crowded_corpus(12000, dim, 3000, 0.0, 63)
    q = (centre[None, :] + 0.01 * W.unit_rows(np.random.default_rng(3).standard_normal((2, dim)))).astype(np.float32)
    o_ids, _ = po.batched_exact_knn(x, q, k)
    for n in (2, 20):
        qq = np.repeat(q, n // 2, axis=0)
        px = B.Proximity(torch.from_numpy(x).to(DEV), dim, 0, k, B.POLICY_FIFO, 32)
        ids, _ = px.knn_batch(torch.from_numpy(qq).to(DEV))
        assert (ids.cpu().numpy() == np.repeat(o_ids, n // 2, axis=0)).all()
        st = px.stats()
        assert st["slack_exhausted"] == n and st["slack_unresolved"] == n
        px.clear()
        assert px.stats()["slack_exhausted"] == 0 and px.stats()["slack_unresolved"] == 0
        px.close()


def test_ordinary_corpora_pass_the_check(B):
    """Unit Gaussian rows at the benchmark's dimensions: the gap between the k-th and the (k+8)-th neighbour is
    far above the float32 error bound, so no query is ranked twice."""
    for dim, k, n_docs, nq in ((768, 10, 200_000, 64), (384, 100, 150_000, 128), (768, 32, 100_000, 3)):
        x = torch.from_numpy(W.corpus_f32(n_docs, dim, 2)).to(DEV)
        q = torch.from_numpy(W.stream_for(W.WORKLOADS["tiny"] if dim == 768 else W.WORKLOADS["lowreuse"], nq)).to(DEV)
        px = B.Proximity(x, dim, 0, k, B.POLICY_FIFO, max(nq, 4))
        px.knn_batch(q)
        st = px.stats()
        assert st["slack_exhausted"] == 0 and st["slack_unresolved"] == 0, (dim, k, st)
        px.close()


def device_corpus(x, kind):
    """The rows on the device as float32 or bfloat16, and the same values as float32 on the host for the oracle."""
    xd = torch.from_numpy(x).to(DEV)
    if kind == "f32":
        return xd, x
    x16 = xd.to(torch.bfloat16)
    return x16, x16.to(torch.float32).cpu().numpy()


@pytest.mark.parametrize("kind,dim,k,n_docs,n_queries", [
    ("bf16", 384, 100, 300_000, 128), ("bf16", 256, 10, 200_000, 40), ("bf16", 384, 3, 150_000, 5),
    ("bf16", 256, 160, 140_000, 70), ("f32", 768, 10, 200_000, 64), ("f32", 384, 100, 150_000, 128),
    ("f32", 768, 32, 250_000, 100), ("f32", 384, 5, 140_000, 7), ("f32", 768, 120, 140_000, 33)])
def test_scan_on_rounded_operands_of_ordinary_rows(B, kind, dim, k, n_docs, n_queries):
    """Calls of more than four rows are pre-ranked on the bfloat16 matrix cores with the queries rounded to
    bfloat16 (one plane of the split) and float32 rows rounded likewise, with a longer candidate list and the
    rounding's error in the exactness check: on unit Gaussian rows the check passes for every query, and the
    lists are the oracle's."""
    xd, xh = device_corpus(W.corpus_f32(n_docs, dim, 5), kind)
    q = W.stream_for(W.WORKLOADS["mid" if dim == 768 else "lowreuse"], n_queries)[:, :dim].copy()
    o_ids, o_d = po.batched_exact_knn(xh, q, k)
    px = B.Proximity(xd, dim, 0, k, B.POLICY_FIFO, n_queries)
    ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
    torch.cuda.synchronize(DEV)
    assert (ids.cpu().numpy() == o_ids).all()
    np.testing.assert_allclose(dists.cpu().numpy(), o_d, rtol=1e-6)
    st = px.stats()
    assert st["coarse_scan_calls"] == 1 and st["coarse_scan_fails"] == 0, st
    assert st["slack_exhausted"] == 0 and st["slack_unresolved"] == 0, st
    px.close()
    # the same search with the operands as they are: the same lists
    pe = B.Proximity(xd, dim, 0, k, B.POLICY_FIFO, n_queries, flags=B.FLAG_NO_ROUNDED_SCAN)
    ids_e, _ = pe.knn_batch(torch.from_numpy(q).to(DEV))
    assert (ids_e.cpu().numpy() == o_ids).all()
    assert pe.stats()["coarse_scan_calls"] == 0
    pe.close()


@pytest.mark.parametrize("kind,k", [("bf16", 200), ("f32", 160)])
def test_more_neighbours_than_a_list_of_rounded_scores_holds(B, kind, k):
    dim, n_queries = 384, 24          # 272 and 264 candidates: more than the ranking kernel holds
    xd, xh = device_corpus(W.corpus_f32(140_000, dim, 6), kind)
    q = W.stream_for(W.WORKLOADS["lowreuse"], n_queries)
    o_ids, _ = po.batched_exact_knn(xh, q, k)
    px = B.Proximity(xd, dim, 0, k, B.POLICY_FIFO, n_queries)
    ids, _ = px.knn_batch(torch.from_numpy(q).to(DEV))
    assert (ids.cpu().numpy() == o_ids).all()
    st = px.stats()
    assert st["coarse_scan_calls"] == 0 and st["slack_exhausted"] == 0, st
    px.close()


@pytest.mark.parametrize("metric", [po.METRIC_L2, po.METRIC_IP, po.METRIC_COSINE])
@pytest.mark.parametrize("kind,dim", [("bf16", 384), ("f32", 768), ("f32", 384)])
def test_a_crowd_within_the_rounding_of_the_operands(B, kind, dim, metric):
    """Two hundred rows whose scores differ by less than the error rounded operands can cause, more of them than
    the list of a scan on rounded operands holds: the check fails for every query of the first call, the second
    ranking still returns the oracle's lists, and the instance scans the operands as they are from then on."""
    k, n_queries = 10, 64
    x, where, centre = crowded_corpus(140_000, dim, 200, 5e-4, 64)
    xd, xh = device_corpus(x, kind)
    rng = np.random.default_rng(10)
    q = (1.3 * (centre[None, :] + 0.05 * W.unit_rows(rng.standard_normal((n_queries, dim))))).astype(np.float32)
    o_ids, o_d = po.batched_exact_knn(xh, q, k, metric=metric)
    assert np.isin(o_ids, where).all()
    px = B.Proximity(xd, dim, 0, k, B.POLICY_FIFO, n_queries, metric=metric)
    for call in range(3):
        ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
        torch.cuda.synchronize(DEV)
        assert (ids.cpu().numpy() == o_ids).all(), call
        np.testing.assert_allclose(dists.cpu().numpy(), o_d, rtol=1e-5, atol=1e-9)
        st = px.stats()
        assert st["coarse_scan_calls"] == 1 and st["coarse_scan_fails"] == n_queries, (call, st)
        assert st["slack_exhausted"] >= n_queries and st["slack_unresolved"] == 0, (call, st)
    px.close()


@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("spread", ["apart", "together"])
def test_a_candidate_list_that_does_not_fill(B, kind, spread):
    """A corpus in an order that defeats the sample: the only rows anywhere near the queries, eighteen of them, sit
    among its first 16 384 rows, so the bound a scan on rounded operands takes from that sample (its eighteenth
    best score, k + 8) lets through those eighteen rows and nothing else, and the list of about forty does not
    fill.  The exactness check then compares the bound itself, not a kept score, with the k-th distance: where
    the eighteen lie well apart the list is proven exact as it stands; where they lie closer together than the
    rounding can tell it is not, and the second ranking returns the exact list."""
    dim, k, n_docs, n_queries = 384, 10, 140_000, 24
    rng = np.random.default_rng(21)
    x = 3.0 * W.corpus_f32(n_docs, dim, 9)                       # far from everything below
    centre = W.unit_rows(rng.standard_normal(dim))
    where = np.sort(rng.choice(16_000, size=18, replace=False))
    steps = 0.05 * np.arange(1, 19) if spread == "apart" else 0.4 + 1e-4 * np.arange(18)
    x[where] = (centre[None, :] + steps[:, None] * W.unit_rows(rng.standard_normal((18, dim)))).astype(np.float32)
    xd, xh = device_corpus(x, kind)
    q = (centre[None, :] + 0.01 * W.unit_rows(rng.standard_normal((n_queries, dim)))).astype(np.float32)
    o_ids, o_d = po.batched_exact_knn(xh, q, k)
    assert np.isin(o_ids, where).all()
    px = B.Proximity(xd, dim, 0, k, B.POLICY_FIFO, n_queries)
    for call in range(2):
        ids, dists = px.knn_batch(torch.from_numpy(q).to(DEV))
        torch.cuda.synchronize(DEV)
        assert (ids.cpu().numpy() == o_ids).all(), call
        np.testing.assert_allclose(dists.cpu().numpy(), o_d, rtol=1e-5)
    st = px.stats()
    assert st["slack_unresolved"] == 0, st
    if spread == "apart":
        assert st["slack_exhausted"] == 0 and st["coarse_scan_calls"] == 2, st
    else:
        assert st["slack_exhausted"] >= n_queries and st["coarse_scan_fails"] == n_queries, st
    px.close()
