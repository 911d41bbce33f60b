"""CPU oracle for the Proximity-FLAT retrieval step.  TEST INFRASTRUCTURE ONLY.

This is a deliberately plain, slow, float64 restatement of what the retrieval
step computes, written from the paper and sharing nothing with the GPU path:
only tests, the smoke check and the benchmark's CPU-baseline leg may import it.
The product (the HIP library and its Python binding) never calls into it.

What it follows
---------------
* ``FlatCacheOracle.lookup`` is the cache lookup procedure of Algorithm 1
  (Section 3.1), one query at a time, in the order the paper gives: distances
  from the query to every cached key, the nearest key, the test against the
  tolerance tau, and on a miss the database call, the eviction when the cache
  already holds c entries, and the insertion of (query, result).
* ``exact_knn`` is the database call for a flat index, i.e. the definition of
  nearest-neighbour search in Section 2.2: the k stored vectors closest to the
  query, returned as a ranked list of indices.  It is brute force: every
  Euclidean distance in direct-difference form, then a full stable sort.
* Eviction follows Section 3.3.2: FIFO removes the oldest inserted entry
  whatever its use; LRU removes the entry unused for longest, where a hit
  uses the matched entry and an insertion uses the new one.
* ``LshCacheOracle`` is the bucketed variant of Section 3.2: ``lsh_bucket`` turns
  the signs of the query's inner products with L given hyperplane normals into
  an L-bit code, the code names a bucket, and each bucket is a cache of the
  kind above (capacity b, its own FIFO/LRU order) that sees only the queries
  with its code.  The normals are an input: the oracle draws nothing.
* ``rerank_factor`` is the re-ranking factor rho of Section 3.3.4: the database
  call asks for rho * k neighbours, all of them are stored with the key, a miss
  hands the first k to the caller, and a hit orders the stored rho * k documents
  by their distance to the *current* query (``rerank_stored``) and hands out the
  k nearest.  rho = 1 is the plain procedure: nothing is re-ranked.
* ``metric`` selects the distance function d of Section 2.2 (Euclidean, inner
  product or cosine, fixed when the index is built): ``metric_distances`` is what
  the database ranks by and reports, ``key_distances`` is what the cache compares
  with tau (Section 3.1 compares query and key with the database's distance).

Readings where the paper is silent (each listed in the design notes):
the hit test is ``<=``; an empty cache misses; equal nearest distances pick
the older entry; only the matched entry is refreshed under LRU; a hit inserts
nothing and returns the stored list unchanged (re-ranking factor 1); ranked
lists order equal distances by document index and are padded with -1 / +inf
when the index holds fewer than k vectors; capacity 0 disables caching; with
rho > 1 a hit ranks by (distance to the current query, document index) and
reports those distances, and rho is a whole number; an inner product of
exactly zero gives hash bit 1 (the hash formula of Section 3.2 includes zero), bit i of the code has
weight 2^i, and L = 0 means a single bucket; the cosine distance is 1 - cos; the
inner-product "distance" is the negated inner product (larger product = closer),
and because that is no distance between two queries (a query is not nearest to
itself under it) the cache of an inner-product index compares query and key by
Euclidean distance.

Parity status: every function here is pinned by tests that do not re-use its
own formula (hand-worked eviction streams, reduction to textbook exact-match
FIFO/LRU caches, brute-force loops, library nearest-neighbour routines, closed
forms for tau = 0 and tau = infinity), the block-streamed search
``exact_knn_over_chunks`` included (literal search and a library routine, on uneven
blocks with duplicated rows).  Document ids at full corpus scale have
no independent pin beyond those small cases ("parity unpinned" at that scale).
"""
from __future__ import annotations

from typing import Callable, List, Optional, Tuple

import numpy as np

POLICY_FIFO = 0
POLICY_LRU = 1
METRIC_L2 = 0
METRIC_IP = 1
METRIC_COSINE = 2


def as_f64_rows(a) -> np.ndarray:
    """Exact widening of float32 (or already-float64) rows to float64."""
    return np.asarray(a, dtype=np.float64)


def l2_distances(q: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """Euclidean distance from q to every row: sqrt(sum_i (q_i - x_i)^2), float64."""
    diff = as_f64_rows(rows) - as_f64_rows(q)[None, :]
    return np.sqrt(np.sum(diff * diff, axis=1))


def metric_distances(q: np.ndarray, rows: np.ndarray, metric: int = METRIC_L2) -> np.ndarray:
    """Distance from q to every row under the index's distance function (Section 2.2), float64:
    Euclidean; negated inner product; or cosine distance 1 - q.x / (|q| |x|).

    The cosine form is evaluated as 1 - q.x / sqrt((q.q) (x.x)) with the three sums taken the same way, so that
    a row bit-identical to q is at distance exactly 0 (the three sums are then one number s, and
    sqrt(s * s) == s in binary floating point; sqrt(s) * sqrt(s) can differ from s in the last place).
    Section 3.3.3 reads a tolerance of 0 as exact matching: an identical query must be a hit at tau = 0.
    """
    if metric == METRIC_L2:
        return l2_distances(q, rows)
    q64, x = as_f64_rows(q), as_f64_rows(rows)
    dots = np.sum(x * q64[None, :], axis=1)
    if metric == METRIC_IP:
        return -dots
    if metric == METRIC_COSINE:
        qq = np.sum(q64[None, :] * q64[None, :], axis=1)[0]
        return 1.0 - dots / np.sqrt(np.sum(x * x, axis=1) * qq)
    raise ValueError("metric must be L2 (0), inner product (1) or cosine (2)")


def key_distances(q: np.ndarray, keys: np.ndarray, metric: int = METRIC_L2) -> np.ndarray:
    """Distance between a query and cached keys, the quantity compared with tau: the index's own
    distance, except for an inner-product index, whose cache falls back to Euclidean distance."""
    return metric_distances(q, keys, METRIC_L2 if metric == METRIC_IP else metric)


def exact_knn(corpus: np.ndarray, q: np.ndarray, k: int,
              chunk_rows: int = 1 << 18, metric: int = METRIC_L2) -> Tuple[np.ndarray, np.ndarray]:
    """Ranked k nearest corpus rows of q (Section 2.2): ids int64[k], dists float64[k].

    Rows are independent, so distances are evaluated a block of rows at a time
    only to bound memory; the ranking is one stable sort over all of them, so
    equal distances keep ascending document index.
    """
    n = 0 if corpus is None else int(corpus.shape[0])
    d = np.empty(n, dtype=np.float64)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        d[r0:r1] = metric_distances(q, corpus[r0:r1], metric)
    order = np.argsort(d, kind="stable")[:k]
    ids = np.full(k, -1, dtype=np.int64)
    dists = np.full(k, np.inf, dtype=np.float64)
    ids[: len(order)] = order
    dists[: len(order)] = d[order]
    return ids, dists


def rerank_stored(corpus: np.ndarray, q: np.ndarray, stored_ids: np.ndarray, k: int,
                  metric: int = METRIC_L2) -> Tuple[np.ndarray, np.ndarray]:
    """Section 3.3.4, the hit side: of the documents stored with the matched key, the k
    nearest to the current query, ranked; ids int64[k], dists float64[k] (padded -1 / +inf)."""
    valid = np.asarray([i for i in np.asarray(stored_ids).tolist() if i >= 0], dtype=np.int64)
    ids = np.full(k, -1, dtype=np.int64)
    dists = np.full(k, np.inf, dtype=np.float64)
    if len(valid):
        d = metric_distances(q, corpus[valid], metric)
        order = sorted(range(len(valid)), key=lambda j: (d[j], int(valid[j])))[:k]
        ids[: len(order)] = valid[order]
        dists[: len(order)] = d[order]
    return ids, dists


class _Entry:
    __slots__ = ("key", "ids", "dists", "seq")

    def __init__(self, key, ids, dists, seq):
        self.key, self.ids, self.dists, self.seq = key, ids, dists, seq


class FlatCacheOracle:
    """Algorithm 1 with its stored state: tolerance per call, capacity c, database D, dict C.

    ``entries`` is kept in eviction order: index 0 is the next victim.  For
    FIFO that is insertion order; for LRU it is order of last use.
    ``retrieve(q) -> (ids, dists)`` is the database call; by default the exact
    flat search over ``corpus``.
    """

    def __init__(self, corpus: Optional[np.ndarray], capacity: int, k: int, policy: int,
                 retrieve: Optional[Callable] = None, rerank_factor: int = 1, metric: int = METRIC_L2):
        if policy not in (POLICY_FIFO, POLICY_LRU):
            raise ValueError("policy must be FIFO (0) or LRU (1)")
        if int(rerank_factor) != rerank_factor or rerank_factor < 1:
            raise ValueError("rerank_factor must be a whole number >= 1")
        self.corpus = corpus
        self.capacity = int(capacity)
        self.k = int(k)
        self.rho = int(rerank_factor)
        self.k_store = self.rho * self.k          # neighbours asked of the database and kept per key
        self.policy = int(policy)
        self.metric = int(metric)
        self.retrieve = retrieve if retrieve is not None else (
            lambda q: exact_knn(corpus, q, self.k_store, metric=self.metric))
        self.entries: List[_Entry] = []
        self.n_queries = 0
        self.n_hits = 0
        self.n_misses = 0
        self.n_inserts = 0
        self.n_evictions = 0
        self.n_scans = 0

    # -- Algorithm 1 -------------------------------------------------------
    def lookup(self, q, tau: float, seq: Optional[int] = None):
        """Process one query.  Returns (ids, dists, hit, source_seq).

        ``source_seq`` is the stream position of the query whose database
        result is returned: the query itself on a miss, the matched key's
        inserting query on a hit.  ``seq`` is this query's stream position when
        the cache sees only part of a stream (a bucket of ``LshCacheOracle``);
        by default the number of queries this cache has processed.
        """
        q64 = as_f64_rows(q).copy()
        tau = float(tau)
        if seq is None:
            seq = self.n_queries
        self.n_queries += 1

        best = -1
        if self.entries:
            keys = np.stack([e.key for e in self.entries])
            dists = key_distances(q64, keys, self.metric)
            min_dist = dists.min()
            # nearest key; among equal distances the oldest insertion
            cands = [i for i in range(len(self.entries)) if dists[i] == min_dist]
            best = min(cands, key=lambda i: self.entries[i].seq)
            if min_dist <= tau:
                e = self.entries[best]
                self.n_hits += 1
                if self.policy == POLICY_LRU:
                    self.entries.append(self.entries.pop(best))
                if self.rho == 1:
                    return e.ids.copy(), e.dists.copy(), True, e.seq
                r_ids, r_d = rerank_stored(self.corpus, q64, e.ids, self.k, self.metric)
                return r_ids, r_d, True, e.seq

        ids, nd = self.retrieve(q64)
        self.n_scans += 1
        self.n_misses += 1
        if self.capacity > 0:
            if len(self.entries) >= self.capacity:
                self.entries.pop(0)
                self.n_evictions += 1
            self.entries.append(_Entry(q64, np.asarray(ids).copy(), np.asarray(nd).copy(), seq))
            self.n_inserts += 1
        return np.asarray(ids)[: self.k].copy(), np.asarray(nd)[: self.k].copy(), False, seq

    def lookup_stream(self, queries, tau: float):
        """Process rows of ``queries`` in order.  Returns ids[n,k], dists[n,k], hit[n], source_seq[n]."""
        n = len(queries)
        ids = np.empty((n, self.k), dtype=np.int64)
        dists = np.empty((n, self.k), dtype=np.float64)
        hit = np.zeros(n, dtype=np.uint8)
        src = np.empty(n, dtype=np.int64)
        for t in range(n):
            ids[t], dists[t], h, src[t] = self.lookup(queries[t], tau)
            hit[t] = 1 if h else 0
        return ids, dists, hit, src

    # -- inspection ----------------------------------------------------------
    def dump_seq(self) -> np.ndarray:
        """Inserting-query positions of the live keys, next victim first."""
        return np.array([e.seq for e in self.entries], dtype=np.int64)

    def dump_keys(self) -> np.ndarray:
        if not self.entries:
            return np.zeros((0, 0), dtype=np.float64)
        return np.stack([e.key for e in self.entries])

    def dump_ids(self) -> np.ndarray:
        if not self.entries:
            return np.zeros((0, self.k_store), dtype=np.int64)
        return np.stack([e.ids for e in self.entries])

    def stats(self) -> dict:
        return dict(queries=self.n_queries, hits=self.n_hits, misses=self.n_misses,
                    inserts=self.n_inserts, evictions=self.n_evictions, scans=self.n_scans,
                    size=len(self.entries))


# ---------------------------------------------------------------------------
# Section 3.2: the bucketed variant.
# ---------------------------------------------------------------------------

def lsh_bucket(q, planes) -> int:
    """The L-bit code of q read as an integer: bit i is 1 exactly when q . r_i >= 0, r_i = planes[i]."""
    planes = np.asarray(planes, dtype=np.float64)
    if planes.size == 0:
        return 0
    dots = planes.reshape(-1, len(q)) @ as_f64_rows(q)
    return int(sum(1 << i for i, v in enumerate(dots) if v >= 0.0))


class LshCacheOracle:
    """One cache of capacity ``bucket_capacity`` per hash code; a query is looked up, and on a miss
    stored, only in the bucket its code names, and each bucket evicts on its own (Section 3.2).

    Same call surface as ``FlatCacheOracle``.  ``dump_*`` list the buckets in ascending code, each in its
    own eviction order (next victim first).
    """

    def __init__(self, corpus: Optional[np.ndarray], planes, bucket_capacity: int, k: int, policy: int,
                 retrieve: Optional[Callable] = None, rerank_factor: int = 1, metric: int = METRIC_L2):
        self.corpus, self.planes, self.metric = corpus, np.asarray(planes, dtype=np.float64), int(metric)
        self.bucket_capacity, self.k, self.policy, self.rho = int(bucket_capacity), int(k), int(policy), int(rerank_factor)
        self.k_store = self.rho * self.k
        self.retrieve = retrieve
        self.buckets = {}
        self.n_queries = 0

    def _bucket(self, code: int) -> FlatCacheOracle:
        if code not in self.buckets:
            self.buckets[code] = FlatCacheOracle(self.corpus, self.bucket_capacity, self.k, self.policy,
                                                 retrieve=self.retrieve, rerank_factor=self.rho, metric=self.metric)
        return self.buckets[code]

    def lookup(self, q, tau: float):
        seq = self.n_queries
        self.n_queries += 1
        cache = self._bucket(lsh_bucket(as_f64_rows(q), self.planes))
        if self.retrieve is not None:
            cache.retrieve = self.retrieve            # the caller may swap the database call between queries
        return cache.lookup(q, tau, seq=seq)

    def lookup_stream(self, queries, tau: float):
        n = len(queries)
        ids = np.empty((n, self.k), dtype=np.int64)
        dists = np.empty((n, self.k), dtype=np.float64)
        hit = np.zeros(n, dtype=np.uint8)
        src = np.empty(n, dtype=np.int64)
        for t in range(n):
            ids[t], dists[t], h, src[t] = self.lookup(queries[t], tau)
            hit[t] = 1 if h else 0
        return ids, dists, hit, src

    def dump_seq(self) -> np.ndarray:
        parts = [self.buckets[c].dump_seq() for c in sorted(self.buckets)]
        return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)

    def dump_ids(self) -> np.ndarray:
        parts = [self.buckets[c].dump_ids() for c in sorted(self.buckets) if self.buckets[c].entries]
        return np.concatenate(parts) if parts else np.zeros((0, self.k_store), dtype=np.int64)

    def stats(self) -> dict:
        total = dict(queries=0, hits=0, misses=0, inserts=0, evictions=0, scans=0, size=0)
        for cache in self.buckets.values():
            for key, v in cache.stats().items():
                total[key] += v
        return total

    @property
    def n_evictions(self) -> int:
        return self.stats()["evictions"]


# ---------------------------------------------------------------------------
# Deferred-scan form, for streams whose literal replay would take hours.
#
# The branch of Algorithm 1 reads only distances between the query and cached
# keys, never a database result, so the sequence of hits, misses, insertions and
# evictions can be replayed first with the database call left out, and the
# database results filled in afterwards for the queries that missed.  The tests
# show this gives the same outputs as the literal form on the small workload.
# ---------------------------------------------------------------------------

def simulate_decisions(queries, tau: float, capacity: int, policy: int,
                       oracle: Optional[FlatCacheOracle] = None, planes=None, metric: int = METRIC_L2):
    """Replay Algorithm 1's control flow only.  Returns (hit[n], source_seq[n], oracle).
    With ``planes`` the cache is the bucketed one and ``capacity`` is per bucket."""
    k_dummy = 1
    no_db = lambda q: (np.full(k_dummy, -1, np.int64), np.full(k_dummy, np.inf))
    if oracle is None and planes is not None:
        oracle = LshCacheOracle(None, planes, capacity, k_dummy, policy, retrieve=no_db, metric=metric)
    if oracle is None:
        oracle = FlatCacheOracle(None, capacity, k_dummy, policy,
                                 retrieve=lambda q: (np.full(k_dummy, -1, np.int64),
                                                     np.full(k_dummy, np.inf)), metric=metric)
    _, _, hit, src = oracle.lookup_stream(queries, tau)
    return hit, src, oracle


def batched_exact_knn(corpus: np.ndarray, queries: np.ndarray, k: int,
                      chunk_rows: int = 1 << 16, metric: int = METRIC_L2) -> Tuple[np.ndarray, np.ndarray]:
    """Ranked exact k-NN for several queries at once, float64.

    (Described for the Euclidean distance.  The other two rank by the same matrix product:
    -q.x, or -q.x / |x| for cosine, whose order per query is that of the cosine distance.)

    Squared distances come from the identity |q-x|^2 = |q|^2 + |x|^2 - 2 q.x with
    a float64 matrix product per block of corpus rows; each block keeps its k
    best by (distance, index), the survivors are ranked by one stable sort, and
    the k winners' distances are then re-evaluated in direct-difference form.
    """
    q64 = as_f64_rows(queries)
    m, n = q64.shape[0], (0 if corpus is None else int(corpus.shape[0]))
    qn = np.sum(q64 * q64, axis=1)
    cand_d2 = [np.empty(0) for _ in range(m)]
    cand_id = [np.empty(0, dtype=np.int64) for _ in range(m)]
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        x = as_f64_rows(corpus[r0:r1])
        if metric == METRIC_L2:
            d2 = qn[:, None] + np.sum(x * x, axis=1)[None, :] - 2.0 * (q64 @ x.T)
        elif metric == METRIC_IP:
            d2 = -(q64 @ x.T)
        else:
            d2 = -(q64 @ x.T) / np.sqrt(np.sum(x * x, axis=1))[None, :]
        kk = min(k, r1 - r0)
        kth = np.partition(d2, kk - 1, axis=1)[:, kk - 1]
        for i in range(m):
            # every row of the block at or below the block's k-th smallest value:
            # at least k of them, more only when values tie exactly
            keep = np.flatnonzero(d2[i] <= kth[i])
            cand_d2[i] = np.concatenate([cand_d2[i], d2[i, keep]])
            cand_id[i] = np.concatenate([cand_id[i], keep + r0])
    ids = np.full((m, k), -1, dtype=np.int64)
    dists = np.full((m, k), np.inf)
    for i in range(m):
        # candidate ids ascend (blocks in order, rows in order), so a stable sort
        # on distance ranks equal distances by document index
        order = np.argsort(cand_d2[i], kind="stable")[:k]
        best = cand_id[i][order]
        ids[i, : len(best)] = best
        if len(best):
            dists[i, : len(best)] = metric_distances(q64[i], corpus[best], metric)
    return ids, dists


def lookup_stream_deferred(corpus, queries, tau: float, capacity: int, k: int, policy: int,
                           knn_chunk: int = 256, rerank_factor: int = 1, planes=None, metric: int = METRIC_L2):
    """Outputs of ``FlatCacheOracle.lookup_stream`` computed decisions-first.

    Returns ids[n,k], dists[n,k], hit[n], source_seq[n], decision_oracle; with
    ``rerank_factor`` > 1 a sixth item, stored_ids[n, rerank_factor*k]: what each query that
    missed stored with its key.
    """
    hit, src, dec = simulate_decisions(queries, tau, capacity, policy, planes=planes, metric=metric)
    n = len(queries)
    k_store = int(rerank_factor) * k
    miss_rows = np.flatnonzero(hit == 0)
    stored_ids = np.full((n, k_store), -1, dtype=np.int64)
    stored_d = np.full((n, k_store), np.inf, dtype=np.float64)
    for c0 in range(0, len(miss_rows), knn_chunk):
        rows = miss_rows[c0:c0 + knn_chunk]
        i_, d_ = batched_exact_knn(corpus, np.asarray(queries)[rows], k_store, metric=metric)
        stored_ids[rows], stored_d[rows] = i_, d_
    ids = stored_ids[:, :k].copy()
    dists = stored_d[:, :k].copy()
    hit_rows = np.flatnonzero(hit == 1)
    if rerank_factor == 1:
        ids[hit_rows] = ids[src[hit_rows]]
        dists[hit_rows] = dists[src[hit_rows]]
        return ids, dists, hit, src, dec
    for t in hit_rows:
        ids[t], dists[t] = rerank_stored(corpus, as_f64_rows(queries[t]), stored_ids[src[t]], k, metric)
    return ids, dists, hit, src, dec, stored_ids


def exact_knn_over_chunks(chunks, queries, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """``batched_exact_knn`` for a corpus that arrives as (first_row, rows) blocks in row order.

    For corpora too large to hold twice in host memory.  Same arithmetic: per block the
    float64 matrix-product form of the squared distance, every row at or below the block's
    k-th smallest kept, one stable sort over the survivors, and the winners' distances
    re-evaluated in direct-difference form from the rows saved while their block was at hand.
    """
    q64 = as_f64_rows(queries)
    m = q64.shape[0]
    qn = np.sum(q64 * q64, axis=1)
    cand_d2 = [np.empty(0) for _ in range(m)]
    cand_id = [np.empty(0, dtype=np.int64) for _ in range(m)]
    cand_row = [np.empty((0, q64.shape[1])) for _ in range(m)]
    for r0, block in chunks:
        x = as_f64_rows(block)
        d2 = qn[:, None] + np.sum(x * x, axis=1)[None, :] - 2.0 * (q64 @ x.T)
        kk = min(k, x.shape[0])
        kth = np.partition(d2, kk - 1, axis=1)[:, kk - 1]
        for i in range(m):
            keep = np.flatnonzero(d2[i] <= kth[i])
            d2_all = np.concatenate([cand_d2[i], d2[i, keep]])
            id_all = np.concatenate([cand_id[i], keep + r0])
            row_all = np.concatenate([cand_row[i], x[keep]])
            order = np.argsort(d2_all, kind="stable")[:k]   # ids ascend, so ties rank by index
            cand_d2[i], cand_id[i], cand_row[i] = d2_all[order], id_all[order], row_all[order]
    ids = np.full((m, k), -1, dtype=np.int64)
    dists = np.full((m, k), np.inf)
    for i in range(m):
        n = len(cand_id[i])
        ids[i, :n] = cand_id[i]
        if n:
            dists[i, :n] = l2_distances(q64[i], cand_row[i])
    return ids, dists
