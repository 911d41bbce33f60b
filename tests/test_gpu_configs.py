"""Parity at the full sizes of the benchmark workloads, in the launch configurations bench.py times, over the
whole length of each query stream.

At these sizes the literal oracle cannot replay every database call, so each test checks
  * hit/miss flags, counters and the cache's eviction order for every query of the stream against the oracle's
    decisions (Algorithm 1 replayed with the database call left out: its branch never reads a database
    result).  The oracle's replay of the full streams is stored under tests/golden/ (written by
    tests/golden/make_stream_decisions.py, checked against the live oracle by tests/test_stream_golden.py);
  * document ids and distances on the rows whose answering query lies in a window at the start, in the middle
    or at the end of the stream, for which the oracle's exact k-NN is computed here;
  * that every hit row returns exactly the list of the row the oracle says answered it.
"""
import hashlib

import numpy as np
import pytest
import torch

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

import parity as P
import stream_golden as SG

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


@pytest.fixture(scope="module")
def B():
    import paper_2503_05530_amd.binding as b
    return b


def check_against_decisions(got, decisions, queries, px, knn_window, knn_ids, knn_d, corpus_rows, dist_rtol, what,
                            metric=po.METRIC_L2):
    """Flags for all rows; ids/dists for rows answered by a query inside the k-NN window (the first
    `knn_window` rows)."""
    o_hit, o_src, dec = decisions
    return check_stream(got, o_hit, o_src, dec.dump_seq().tolist(), dec.stats(), queries, px,
                        np.arange(knn_window), knn_ids, knn_d, corpus_rows, dist_rtol, what, metric)


def check_stream(got, o_hit, o_src, o_dump, o_counters, queries, px, knn_rows, knn_ids, knn_d, corpus_rows,
                 dist_rtol, what, metric=po.METRIC_L2):
    """Flags, cache contents and counters for every row; ids/dists for the rows answered by one of `knn_rows`
    (stream positions, ascending), whose oracle k-NN lists are knn_ids / knn_d in that order."""
    ids, dists, hit = got
    mism = np.flatnonzero(hit != o_hit)
    assert len(mism) == 0, f"{what}: flags differ first at rows {mism[:5]}"
    # a hit returns the answering row's list, whatever it is
    hit_rows = np.flatnonzero(o_hit == 1)
    assert (ids[hit_rows] == ids[o_src[hit_rows]]).all(), f"{what}: a hit row differs from its source row"
    assert (dists[hit_rows] == dists[o_src[hit_rows]]).all()
    knn_rows = np.asarray(knn_rows)
    at = np.searchsorted(knn_rows, o_src)
    at = np.minimum(at, len(knn_rows) - 1)
    rows = np.flatnonzero(knn_rows[at] == o_src)
    assert len(rows) > 0
    excused = P.assert_lists_match(ids[rows], dists[rows], knn_ids[at[rows]], knn_d[at[rows]],
                                   corpus_rows, np.asarray(queries)[o_src[rows]], dist_rtol, what, metric)
    seq, _, dump_ids = px.cache_dump(want_ids=True)
    assert seq.tolist() == list(o_dump), f"{what}: cache contents differ"
    assert (dump_ids == ids[seq]).all(), f"{what}: stored lists differ from the lists returned at insertion"
    st = px.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == o_counters[key], f"{what}: counter {key}"
    assert st["slack_unresolved"] == 0, f"{what}: a ranked list was not proven exact"
    # (ordinary rows: the candidate lists are long enough all but never, also those of scans on rounded operands)
    assert st["slack_exhausted"] <= st["misses"] // 1000, f"{what}: {st['slack_exhausted']} searches ranked twice"
    return excused, len(rows)


def golden_trace(name, tau, n_rows=None):
    """The oracle's stored decisions for a whole stream as a replayable trace: the textbook cache over base ids
    (or over the positions themselves where nothing ever hits) after it has been shown equal, row for row,
    to what the oracle stored -- flags, answering rows, final contents, counters.  Prefixes of the stream are
    then read off the trace."""
    w = W.WORKLOADS[name]
    sec = SG.read_decisions(name)[f"{name} tau={tau!r}"]
    if int(sec["hits"]) == 0:
        keys = list(range(w.n_stream))
    elif w.choice == "zipf":
        keys = W.zipf_choice(w.n_stream, w.n_bases, w.zipf_s, w.seed).tolist()
    else:
        keys = W.uniform_choice(w.n_stream, w.n_bases, w.seed).tolist()
    n = w.n_stream if n_rows is None else n_rows
    trace = SG.TextbookTrace(keys, w.capacity, w.policy, snapshots=[n])
    assert (trace.flags == sec["flags"]).all() and SG.sha_i64(trace.src) == sec["source_seq_sha256"]
    assert trace.snapshots[w.n_stream] == [int(v) for v in sec["dump_seq"].split()]
    full = trace.counters(w.n_stream)
    assert (full["hits"], full["evictions"]) == (int(sec["hits"]), int(sec["evictions"]))
    return trace.flags[:n], trace.src[:n], trace.snapshots[n], trace.counters(n)


def run_stream_into(px, q_dev, tau, batch, n_rows):
    """The first n_rows of a device-resident stream, `batch` rows per call, into preallocated outputs."""
    k = px.k
    ids = torch.empty((n_rows, k), dtype=torch.int64, device=DEV)
    dists = torch.empty((n_rows, k), dtype=torch.float32, device=DEV)
    hit = torch.empty((n_rows,), dtype=torch.uint8, device=DEV)
    for r0 in range(0, n_rows, batch):
        r1 = min(n_rows, r0 + batch)
        px.search_batch(q_dev[r0:r1], tau, ids[r0:r1], dists[r0:r1], hit[r0:r1])
    torch.cuda.synchronize(DEV)
    return ids.cpu().numpy(), dists.cpu().numpy(), hit.cpu().numpy()


def window_rows(n_stream, width):
    """Stream positions of three windows: the start, the middle and the end."""
    mid0 = n_stream // 2
    return np.concatenate([np.arange(0, width), np.arange(mid0, mid0 + width), np.arange(n_stream - width, n_stream)])


# ---------------------------------------------------------------------------
# Mid: 1 M x 768 float32, LRU c=300, k=10, tau sweep x batch {1, 64}
# ---------------------------------------------------------------------------
MID_ROWS = 5120       # stream prefix the variants (re-ranking, buckets, other distances, call splits) replay
MID_WINDOW = 384      # rows of it whose exact k-NN the oracle computes


@pytest.fixture(scope="module")
def mid():
    w = W.WORKLOADS["mid"]
    corpus = W.corpus_for(w)
    q = W.stream_for(w, MID_ROWS)
    knn_ids, knn_d = po.batched_exact_knn(corpus, q[:MID_WINDOW], w.k, chunk_rows=1 << 17)
    decisions = {}
    for tau in (0.25,):            # the variants below (re-ranking, buckets, other distances) run at this tolerance
        decisions[tau] = po.simulate_decisions(q, tau, w.capacity, w.policy)
    corpus_dev = torch.from_numpy(corpus).to(DEV)
    return w, corpus, corpus_dev, q, knn_ids, knn_d, decisions


MID_FULL_WINDOW = 128     # rows per window (start, middle, end of the stream) whose exact k-NN the oracle computes
MID_ALL_MISS_ROWS_B1 = 20_000   # one query per call at tau <= 0.1: every call scans the corpus (0.5 ms each),
                                # so those two legs replay this prefix; every other leg replays all 100 000 rows


@pytest.fixture(scope="module")
def mid_full(mid):
    w, corpus, corpus_dev, _, _, _, _ = mid
    q = W.stream_for(w)
    rows = window_rows(w.n_stream, MID_FULL_WINDOW)
    head = np.arange(MID_FULL_WINDOW)
    knn_ids, knn_d = po.batched_exact_knn(corpus, q[rows], w.k, chunk_rows=1 << 17)
    return q, torch.from_numpy(q).to(DEV), rows, knn_ids, knn_d, head


@pytest.mark.parametrize("batch", [1, 64])
@pytest.mark.parametrize("tau", [0.0, 0.1, 0.25, 0.5, 1.0])
def test_mid_workload_full_stream(B, mid, mid_full, tau, batch):
    """All 100 000 queries of the mid workload (Algorithm 1 over the whole stream): every flag, the final cache
    contents and the counters against the oracle's stored decisions, and the literal counts of the recipe."""
    w, corpus, corpus_dev, _, _, _, _ = mid
    q, q_dev, rows, knn_ids, knn_d, head = mid_full
    n = MID_ALL_MISS_ROWS_B1 if (batch == 1 and tau <= 0.1) else w.n_stream
    o_hit, o_src, o_dump, o_counters = golden_trace("mid", tau, n)
    if n == w.n_stream:
        want = (69_624, 30_076) if tau >= 0.25 else (0, 99_700)
        assert (o_counters["hits"], o_counters["evictions"]) == want
        use, use_ids, use_d = rows, knn_ids, knn_d
    else:
        use, use_ids, use_d = head, knn_ids[:len(head)], knn_d[:len(head)]
    px = B.Proximity(corpus_dev, w.dim, w.capacity, w.k, w.policy, 64)
    got = run_stream_into(px, q_dev, tau, batch, n)
    excused, n_checked = check_stream(got, o_hit, o_src, o_dump, o_counters, q, px, use, use_ids, use_d, corpus,
                                      P.DIST_RTOL_F32, f"mid tau={tau} batch={batch} rows={n}")
    assert excused == 0 and n_checked >= int((o_hit[use] == 0).sum()) > len(use) // 8
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
    """All 50 000 queries, 128 per call (the last call carries 80); oracle k-NN for three windows of 32 rows."""
    w = W.WORKLOADS["lowreuse"]
    x = device_corpus(w)
    q = W.stream_for(w)
    o_hit, o_src, o_dump, o_counters = golden_trace("lowreuse", w.tau)
    assert (o_counters["hits"], o_counters["evictions"]) == (435, 48_565)
    rows = window_rows(w.n_stream, 32)
    knn_ids, knn_d = po.exact_knn_over_chunks(host_chunks(x), q[rows], w.k)
    px = B.Proximity(x, w.dim, w.capacity, w.k, w.policy, w.batch)
    got = run_stream_into(px, torch.from_numpy(q).to(DEV), w.tau, w.batch, w.n_stream)

    class Rows:                      # rows gathered on demand from the device copy
        def __getitem__(self, idx):
            return x[torch.from_numpy(np.asarray(idx)).to(DEV)].to(torch.float32).cpu().numpy()

    excused, n = check_stream(got, o_hit, o_src, o_dump, o_counters, q, px, rows, knn_ids, knn_d, Rows(),
                              P.DIST_RTOL_BF16, "lowreuse")
    assert excused <= 1 and n >= int((o_hit[rows] == 0).sum()) > len(rows) // 2
    px.close()


# ---------------------------------------------------------------------------
# Large: 24 M x 768 float32 (about 74 GB resident), LRU c=300, k=32, batch 256, tau=0.5
# ---------------------------------------------------------------------------
def test_large_workload(B):
    w = W.WORKLOADS["large"]
    free, total = torch.cuda.mem_get_info(DEV)
    if free < 100 * (1 << 30):
        pytest.skip("needs about 100 GB of free device memory")
    # all 20 000 queries, 256 per call (the last call carries 32); oracle k-NN for three windows of 16 rows
    x = device_corpus(w)
    q = W.stream_for(w)
    o_hit, o_src, o_dump, o_counters = golden_trace("large", w.tau)
    assert (o_counters["hits"], o_counters["evictions"]) == (15_221, 4_479)
    rows = window_rows(w.n_stream, 16)
    knn_ids, knn_d = po.exact_knn_over_chunks(host_chunks(x, 1 << 20), q[rows], w.k)
    px = B.Proximity(x, w.dim, w.capacity, w.k, w.policy, w.batch)
    got = run_stream_into(px, torch.from_numpy(q).to(DEV), w.tau, w.batch, w.n_stream)

    class Rows:
        def __getitem__(self, idx):
            return x[torch.from_numpy(np.asarray(idx)).to(DEV)].cpu().numpy()

    excused, n = check_stream(got, o_hit, o_src, o_dump, o_counters, q, px, rows, knn_ids, knn_d, Rows(),
                              P.DIST_RTOL_F32, "large")
    assert excused <= 1 and n >= int((o_hit[rows] == 0).sum()) >= 8
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


@pytest.mark.parametrize("n_keys,batch,n_batches", [(1500, 1024, 3), (W.PROBE_KEYS, W.PROBE_BATCH, 2)])
def test_probe_microbenchmark(B, n_keys, batch, n_batches):
    """The cache alone on the mix of the lookup-time measurement of Section 4.4: half of the rows are resident
    keys displaced by up to twice the tolerance, so their distances straddle tau and the float64 decision
    matters.  Every flag of every batch and the final cache contents are the oracle's: replayed live at the
    small size; at the full size (10 000 keys, calls of 4 096 rows) read from the oracle's stored replay of
    the same two batches, which were drawn against the oracle's own resident keys."""
    dim, tau = W.PROBE_DIM, W.PROBE_TAU
    keys = W.probe_warm_keys(n_keys, dim, 0)
    mix = W.ProbeMix(dim, 0)
    full_size = n_keys == W.PROBE_KEYS
    stored = SG.read_decisions("probe") if full_size else None

    def make_px():
        px = B.Proximity(None, dim, n_keys, 1, po.POLICY_LRU, batch, device=DEV)
        _, _, hit = P.run_stream(px, keys, tau, batch, DEV)
        assert hit.sum() == 0 and px.stats()["size"] == n_keys
        return px

    px = make_px()
    orc = None if full_size else warm_oracle(keys, po.POLICY_LRU)
    # a batch depends on which keys are resident when it starts: it is drawn against the library's own dump,
    # which equals the oracle's as long as every earlier decision did (the stored digest of each batch's
    # bytes shows it at the full size)
    batches, flags = [], []
    for b in range(n_batches):
        _, resident, _ = px.cache_dump(want_keys=True)
        qb = mix.batch(resident, batch)
        _, _, hit = px.search_batch(torch.from_numpy(qb).to(DEV), tau)
        hit = hit.cpu().numpy()
        if full_size:
            sec = stored[f"probe batch={b}"]
            assert hashlib.sha256(qb.tobytes()).hexdigest() == sec["batch_sha256"], f"batch {b} differs from the oracle's"
            assert int(sec["rows"]) == batch and float(sec["tau"]) == tau
            mism = np.flatnonzero(hit != sec["flags"])
            assert len(mism) == 0, f"batch {b}: flags differ first at rows {mism[:5]}"
            assert px.stats()["hits"] == int(sec["hits_total"]) and px.stats()["evictions"] == int(sec["evictions_total"])
            assert SG.sha_i64(px.cache_dump()[0]) == sec["dump_seq_sha256"], f"batch {b}: cache contents differ"
        else:
            o_hit = np.array([orc.lookup(qb[t], tau)[2] for t in range(batch)], dtype=np.uint8)
            assert (hit == o_hit).all()
            assert px.cache_dump()[0].tolist() == orc.dump_seq().tolist()
        batches.append(qb)
        flags.append(hit)
    stream = np.concatenate(batches)
    flags = np.concatenate(flags)
    st = px.stats()
    assert st["misses"] == st["inserts"] and st["size"] == n_keys
    assert st["evictions"] == st["misses"] - n_keys
    assert 0.10 < flags.mean() < 0.40
    # the same rows one query per call must give the same flags and the same cache
    px1 = make_px()
    n1 = len(stream) if len(stream) <= 4096 else 1536
    _, _, hit1 = P.run_stream(px1, stream[:n1], tau, 1, DEV)
    assert (hit1 == flags[:n1]).all()
    if n1 == len(stream):
        assert px1.cache_dump()[0].tolist() == px.cache_dump()[0].tolist()
    px.close()
    px1.close()
