"""Parity at the full sizes of the benchmark workloads, in the launch configurations bench.py times.

At these sizes the literal oracle cannot replay every database call, so each test checks
  * hit/miss flags, counters and the cache's eviction order for every query of the stretch
    (decisions-only oracle replay: the branch of Algorithm 1 never reads a database result);
  * document ids and distances on the rows whose answering query lies in an early window, for
    which the oracle's exact k-NN is computed one batch of queries at a time;
  * that every hit row returns exactly the list of the row the oracle says answered it.
"""
import numpy as np
import pytest
import torch

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

import parity as P

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


@pytest.fixture(scope="module")
def B():
    import paper_2503_05530_amd.binding as b
    return b


def check_against_decisions(got, decisions, queries, px, knn_window, knn_ids, knn_d, corpus_rows, dist_rtol, what,
                            metric=po.METRIC_L2):
    """Flags for all rows; ids/dists for rows answered by a query inside the k-NN window."""
    ids, dists, hit = got
    o_hit, o_src, dec = decisions
    mism = np.flatnonzero(hit != o_hit)
    assert len(mism) == 0, f"{what}: flags differ first at rows {mism[:5]}"
    # a hit returns the answering row's list, whatever it is
    hit_rows = np.flatnonzero(o_hit == 1)
    assert (ids[hit_rows] == ids[o_src[hit_rows]]).all(), f"{what}: a hit row differs from its source row"
    assert (dists[hit_rows] == dists[o_src[hit_rows]]).all()
    rows = np.flatnonzero(o_src < knn_window)
    assert len(rows) > 0
    excused = P.assert_lists_match(ids[rows], dists[rows], knn_ids[o_src[rows]], knn_d[o_src[rows]],
                                   corpus_rows, np.asarray(queries)[o_src[rows]], dist_rtol, what, metric)
    seq, _, dump_ids = px.cache_dump(want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist(), f"{what}: cache contents differ"
    assert (dump_ids == ids[seq]).all(), f"{what}: stored lists differ from the lists returned at insertion"
    st = px.stats()
    os_ = dec.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == os_[key], f"{what}: counter {key}"
    return excused, len(rows)


# ---------------------------------------------------------------------------
# Mid: 1 M x 768 float32, LRU c=300, k=10, tau sweep x batch {1, 64}
# ---------------------------------------------------------------------------
MID_ROWS = 5120       # stream prefix replayed (80 batches of 64)
MID_WINDOW = 384      # rows whose exact k-NN the oracle computes


@pytest.fixture(scope="module")
def mid():
    w = W.WORKLOADS["mid"]
    corpus = W.corpus_for(w)
    q = W.stream_for(w, MID_ROWS)
    knn_ids, knn_d = po.batched_exact_knn(corpus, q[:MID_WINDOW], w.k, chunk_rows=1 << 17)
    decisions = {}
    for tau in (0.0, 0.1, 0.25, 0.5, 1.0):
        decisions[tau] = po.simulate_decisions(q, tau, w.capacity, w.policy)
    corpus_dev = torch.from_numpy(corpus).to(DEV)
    return w, corpus, corpus_dev, q, knn_ids, knn_d, decisions


@pytest.mark.parametrize("batch", [1, 64])
@pytest.mark.parametrize("tau", [0.0, 0.1, 0.25, 0.5, 1.0])
def test_mid_workload(B, mid, tau, batch):
    w, corpus, corpus_dev, q, knn_ids, knn_d, decisions = mid
    px = B.Proximity(corpus_dev, w.dim, w.capacity, w.k, w.policy, 64)
    got = P.run_stream(px, q, tau, batch, DEV)
    excused, n = check_against_decisions(got, decisions[tau], q, px, MID_WINDOW, knn_ids, knn_d, corpus,
                                         P.DIST_RTOL_F32, f"mid tau={tau} batch={batch}")
    assert excused == 0
    if tau >= 0.25:
        assert (decisions[tau][0] == decisions[0.25][0]).all()   # one regime above the rewording radius
    else:
        assert decisions[tau][0].sum() == 0
    px.close()


@pytest.mark.parametrize("metric", [po.METRIC_IP, po.METRIC_COSINE])
def test_mid_workload_other_metrics(B, mid, metric):
    """The mid workload on an inner-product and on a cosine index (Section 2.2), calls of 1 and of 64 rows.
    Rows and queries have unit length up to float32 rounding, so the tolerance that separates rewordings
    from other queries is tau = 0.25 as a Euclidean distance (inner-product index) and tau^2 / 2 as a cosine
    distance."""
    w, corpus, corpus_dev, q, _, _, _ = mid
    tau = 0.25 if metric == po.METRIC_IP else 0.25 * 0.25 / 2.0
    knn_ids, knn_d = po.batched_exact_knn(corpus, q[:MID_WINDOW], w.k, chunk_rows=1 << 17, metric=metric)
    decisions = po.simulate_decisions(q, tau, w.capacity, w.policy, metric=metric)
    assert 3000 < decisions[0].sum() < 4000
    for batch in (1, 64):
        px = B.Proximity(corpus_dev, w.dim, w.capacity, w.k, w.policy, 64, metric=metric)
        got = P.run_stream(px, q, tau, batch, DEV)
        excused, n = check_against_decisions(got, decisions, q, px, MID_WINDOW, knn_ids, knn_d, corpus,
                                             P.DIST_RTOL_F32, f"mid metric={metric} batch={batch}", metric=metric)
        assert excused == 0
        px.close()


@pytest.mark.parametrize("batch", [1, 64])
def test_mid_workload_with_reranking(B, mid, batch):
    """Re-ranking factor 4 (Section 3.3.4) at the mid workload's size: 40 neighbours stored per key."""
    w, corpus, corpus_dev, q, knn_ids, knn_d, decisions = mid
    rho, tau = 4, 0.25
    if "knn" not in _MID_RERANK:
        _MID_RERANK["knn"] = po.batched_exact_knn(corpus, q[:MID_WINDOW], rho * w.k, chunk_rows=1 << 17)
    big_ids, big_d = _MID_RERANK["knn"]
    assert (big_ids[:, :w.k] == knn_ids).all()
    o_hit, o_src, dec = decisions[tau]
    px = B.Proximity(corpus_dev, w.dim, w.capacity, w.k, w.policy, 64, rerank_factor=rho)
    ids, dists, hit = P.run_stream(px, q, tau, batch, DEV)
    assert (hit == o_hit).all()
    rows = np.flatnonzero(o_src < MID_WINDOW)
    want_ids = np.empty((len(rows), w.k), dtype=np.int64)
    want_d = np.empty((len(rows), w.k))
    for j, t in enumerate(rows):
        if o_hit[t]:
            want_ids[j], want_d[j] = po.rerank_stored(corpus, po.as_f64_rows(q[t]), big_ids[o_src[t]], w.k)
        else:
            want_ids[j], want_d[j] = big_ids[t, :w.k], big_d[t, :w.k]
    assert o_hit[rows].sum() > 500
    excused = P.assert_lists_match(ids[rows], dists[rows], want_ids, want_d, corpus, q[rows], P.DIST_RTOL_F32,
                                   f"mid rho=4 batch={batch}")
    assert excused == 0
    seq, _, stored = px.cache_dump(want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist()
    early = seq < MID_WINDOW
    assert (stored[early] == big_ids[seq[early]]).all()
    st, os_ = px.stats(), dec.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == os_[key]
    px.close()


@pytest.mark.parametrize("batch", [1, 64])
def test_mid_workload_bucketed(B, mid, batch):
    """The bucketed cache (Section 3.2) at the mid workload's size: 16 buckets of 20 entries."""
    w, corpus, corpus_dev, q, knn_ids, knn_d, _ = mid
    tau, bits, b = 0.25, 4, 20
    planes = W.lsh_planes(bits, w.dim, w.seed)
    if "dec" not in _MID_LSH:
        _MID_LSH["dec"] = po.simulate_decisions(q, tau, b, w.policy, planes=planes)
    decisions = _MID_LSH["dec"]
    assert 2000 < decisions[0].sum() < 5000 and decisions[2].n_evictions > 500
    px = B.Proximity(corpus_dev, w.dim, b, w.k, w.policy, 64, lsh_planes=torch.from_numpy(planes).to(DEV))
    got = P.run_stream(px, q, tau, batch, DEV)
    excused, n = check_against_decisions(got, decisions, q, px, MID_WINDOW, knn_ids, knn_d, corpus,
                                         P.DIST_RTOL_F32, f"mid bucketed batch={batch}")
    assert excused == 0 and n > 500
    px.close()


_MID_LSH = {}
_MID_RERANK = {}


def test_mid_any_split_gives_the_same_result(B, mid):
    w, corpus, corpus_dev, q, *_ = mid
    outs = []
    for sizes in ([64] * 16, [1] * 7 + [9, 33, 64, 2, 5, 17, 40, 8] * 6, [37] * 28):
        px = B.Proximity(corpus_dev, w.dim, w.capacity, w.k, w.policy, 64)
        ids, dists, hit, r0 = [], [], [], 0
        for n in sizes:
            if r0 + n > 1024:
                n = 1024 - r0
            if n <= 0:
                break
            i, d, h = px.search_batch(torch.from_numpy(q[r0:r0 + n]).to(DEV), 0.25)
            ids.append(i); dists.append(d); hit.append(h); r0 += n
        assert r0 == 1024
        outs.append((torch.cat(ids).cpu().numpy(), torch.cat(dists).cpu().numpy(), torch.cat(hit).cpu().numpy(),
                     px.cache_dump()[0]))
        px.close()
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert (a == b).all()


# ---------------------------------------------------------------------------
# Low reuse: 8 M x 384 bfloat16, FIFO c=1000, k=100, batch 128, tau=0.2
# ---------------------------------------------------------------------------
def device_corpus(w, n_docs=None):
    n = w.n_docs if n_docs is None else n_docs
    dtype = torch.bfloat16 if w.corpus_dtype == W.DTYPE_BF16 else torch.float32
    x = torch.empty((n, w.dim), dtype=dtype, device=DEV)
    for r0, chunk in W.device_corpus_chunks(n, w.dim, w.seed, DEV, w.corpus_dtype):
        x[r0:r0 + chunk.shape[0]] = chunk
    return x


def host_chunks(x_dev, rows=1 << 19):
    """Corpus blocks as float32 on the host, exact values (bfloat16 widens exactly)."""
    for r0 in range(0, x_dev.shape[0], rows):
        yield r0, x_dev[r0:r0 + rows].to(torch.float32).cpu().numpy()


def test_lowreuse_workload(B):
    w = W.WORKLOADS["lowreuse"]
    n_rows, window = 6400, 96        # 50 batches of 128; oracle k-NN for the first 96 rows
    x = device_corpus(w)
    q = W.stream_for(w, n_rows)
    decisions = po.simulate_decisions(q, w.tau, w.capacity, w.policy)
    knn_ids, knn_d = po.exact_knn_over_chunks(host_chunks(x), q[:window], w.k)
    px = B.Proximity(x, w.dim, w.capacity, w.k, w.policy, w.batch)
    got = P.run_stream(px, q, w.tau, w.batch, DEV)

    class Rows:                      # rows gathered on demand from the device copy
        def __getitem__(self, idx):
            return x[torch.from_numpy(np.asarray(idx)).to(DEV)].to(torch.float32).cpu().numpy()

    excused, n = check_against_decisions(got, decisions, q, px, window, knn_ids, knn_d, Rows(),
                                         P.DIST_RTOL_BF16, "lowreuse")
    assert excused <= 1
    assert decisions[0].mean() < 0.05            # expected hit rate near zero
    px.close()


# ---------------------------------------------------------------------------
# Large: 24 M x 768 float32 (about 74 GB resident), LRU c=300, k=32, batch 256, tau=0.5
# ---------------------------------------------------------------------------
def test_large_workload(B):
    w = W.WORKLOADS["large"]
    free, total = torch.cuda.mem_get_info(DEV)
    if free < 100 * (1 << 30):
        pytest.skip("needs about 100 GB of free device memory")
    n_rows, window = 2560, 48        # 10 batches of 256; oracle k-NN for the first 48 rows
    x = device_corpus(w)
    q = W.stream_for(w, n_rows)
    decisions = po.simulate_decisions(q, w.tau, w.capacity, w.policy)
    knn_ids, knn_d = po.exact_knn_over_chunks(host_chunks(x, 1 << 20), q[:window], w.k)
    px = B.Proximity(x, w.dim, w.capacity, w.k, w.policy, w.batch)
    got = P.run_stream(px, q, w.tau, w.batch, DEV)

    class Rows:
        def __getitem__(self, idx):
            return x[torch.from_numpy(np.asarray(idx)).to(DEV)].cpu().numpy()

    excused, n = check_against_decisions(got, decisions, q, px, window, knn_ids, knn_d, Rows(),
                                         P.DIST_RTOL_F32, "large")
    assert excused <= 1
    assert px.stats()["inbatch_hits"] > 0        # hits on keys stored earlier in the same batch occur
    px.close()
    del x
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# Probe microbenchmark: 10 000 resident keys, batches of 4 096, tau=0.3, LRU, no corpus
# ---------------------------------------------------------------------------
def warm_oracle(keys, policy):
    """Oracle state after the warm-up stream: distinct random unit vectors are ~1.41 apart, far
    above tau, so every one of them missed and was stored, in order (checked on the GPU side)."""
    orc = po.FlatCacheOracle(None, len(keys), 1, policy,
                             retrieve=lambda q: (np.full(1, -1, np.int64), np.full(1, np.inf)))
    for t, key in enumerate(keys):
        orc.entries.append(po._Entry(po.as_f64_rows(key).copy(), np.full(1, -1, np.int64), np.full(1, np.inf), t))
    orc.n_queries = orc.n_misses = orc.n_inserts = orc.n_scans = len(keys)
    return orc


@pytest.mark.parametrize("n_keys,batch,n_batches,oracle_rows", [(1500, 1024, 3, 3072), (W.PROBE_KEYS, W.PROBE_BATCH, 2, 160)])
def test_probe_microbenchmark(B, n_keys, batch, n_batches, oracle_rows):
    dim, tau = W.PROBE_DIM, W.PROBE_TAU
    keys = W.probe_warm_keys(n_keys, dim, 0)
    mix = W.ProbeMix(dim, 0)

    def make_px():
        px = B.Proximity(None, dim, n_keys, 1, po.POLICY_LRU, batch, device=DEV)
        _, _, hit = P.run_stream(px, keys, tau, batch, DEV)
        assert hit.sum() == 0 and px.stats()["size"] == n_keys
        return px

    px = make_px()
    orc = warm_oracle(keys, po.POLICY_LRU)
    # the batches depend on which keys are resident, so they are drawn against the GPU's own dump,
    # and every decision is then checked against the oracle replaying the same rows
    batches, flags = [], []
    for _ in range(n_batches):
        _, resident, _ = px.cache_dump(want_keys=True)
        qb = mix.batch(resident, batch)
        _, _, hit = px.search_batch(torch.from_numpy(qb).to(DEV), tau)
        batches.append(qb)
        flags.append(hit.cpu().numpy())
    stream = np.concatenate(batches)
    flags = np.concatenate(flags)
    st = px.stats()
    assert st["misses"] == st["inserts"] and st["size"] == n_keys
    assert st["evictions"] == st["misses"] - n_keys
    assert 0.10 < flags.mean() < 0.40
    # oracle replay of the first rows (each lookup scans every resident key in float64)
    o_hit = np.array([orc.lookup(stream[t], tau)[2] for t in range(oracle_rows)], dtype=np.uint8)
    assert (flags[:oracle_rows] == o_hit).all()
    if oracle_rows == len(stream):
        seq, _, _ = px.cache_dump()
        assert seq.tolist() == orc.dump_seq().tolist()
    # the same rows one query per call must give the same flags and the same cache
    px1 = make_px()
    n1 = len(stream) if len(stream) <= 4096 else 1536
    _, _, hit1 = P.run_stream(px1, stream[:n1], tau, 1, DEV)
    assert (hit1 == flags[:n1]).all()
    if n1 == len(stream):
        assert px1.cache_dump()[0].tolist() == px.cache_dump()[0].tolist()
    px.close()
    px1.close()
