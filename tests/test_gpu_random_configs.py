"""Seeded random configurations, GPU against the oracle: every switch of the interface drawn at random
(dimension, k, capacity, policy, corpus type and size, re-ranking factor, bucketed or flat cache, tolerance,
how the stream is cut into calls), on streams that mix rewordings at several radii, exact repeats and fresh
vectors, so that distances fall on both sides of the tolerance.  Seeds 0..79 use the Euclidean index, seeds
from 80 on alternate between the inner-product and the cosine index on corpora whose rows have lengths
0.3..3 (for cosine the queries get other lengths as well, and the tolerance becomes tau^2 / 2, the cosine
distance of unit vectors tau apart; tau = 0 included)."""
import numpy as np
import pytest
import torch

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

import parity as P

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def draw_case(seed):
    rng = np.random.default_rng([seed, 99])
    dim = int(rng.choice([32, 64, 96, 128, 384, 768]))
    k = int(rng.choice([1, 3, 10, 17, 32]))
    rho = int(rng.choice([1, 1, 2, 4]))
    n_docs = int(rng.choice([0, 5, 700, 3000, 20000]))
    bf16 = bool(rng.random() < 0.25) and n_docs > 0
    lsh_bits = int(rng.choice([0, 0, 1, 3, 5]))
    capacity = int(rng.choice([0, 1, 2, 7, 40])) if lsh_bits == 0 else int(rng.choice([1, 2, 5]))
    policy = int(rng.choice([po.POLICY_FIFO, po.POLICY_LRU]))
    n_bases = int(rng.choice([3, 12, 60]))
    n = int(rng.choice([150, 400]))
    tau = float(rng.choice([0.0, 0.05, 0.2, 0.45, 1e9]))
    bases = W.unit_rows(rng.standard_normal((n_bases, dim)))
    idx = rng.integers(0, n_bases, size=n)
    radius = rng.choice([0.0, 0.03, 0.15, 0.3, 0.6], size=n)
    q = W.unit_rows(bases[idx] + radius[:, None] * W.unit_rows(rng.standard_normal((n, dim)))).astype(np.float32)
    repeats = rng.random(n) < 0.15                       # exact repeats of an earlier row
    for t in np.flatnonzero(repeats):
        if t > 0:
            q[t] = q[rng.integers(0, t)]
    cuts, r0 = [], 0
    while r0 < n:
        step = int(rng.choice([1, 2, 4, 5, 9, 33, 64, 200]))
        cuts.append((r0, min(n, r0 + step)))
        r0 += step
    metric = po.METRIC_L2 if seed < 80 else (po.METRIC_IP if seed % 2 == 0 else po.METRIC_COSINE)
    if metric == po.METRIC_COSINE:
        tau = min(1e9, tau * tau / 2.0)
        if tau == 0.0 or rng.random() < 0.5:
            # lengths that are powers of two scale every term of the cosine distance exactly, so a repeat at
            # another length is at distance exactly 0 on both sides and tau = 0 is the exact-match cache of
            # Section 3.3.3 (bit-identical repeats, and their exact multiples, hit; nothing else does)
            q = (q * rng.choice([0.5, 1.0, 2.0, 4.0], size=(n, 1))).astype(np.float32)
        else:
            # arbitrary lengths: a repeat is the same direction rounded to float32 at another length, whose
            # cosine distance is a few 1e-16 either side of zero in any float64 evaluation -- a comparison
            # of that with zero is rounding noise on both sides, so these streams keep tau above it
            q = (q * rng.uniform(0.5, 2.0, size=(n, 1))).astype(np.float32)
            tau = max(tau, 1e-12)
    return dict(dim=dim, k=k, rho=rho, n_docs=n_docs, bf16=bf16, lsh_bits=lsh_bits, capacity=capacity, policy=policy,
                tau=tau, q=q, cuts=cuts, seed=seed, metric=metric)


@pytest.mark.parametrize("seed", range(120))
def test_random_configuration(seed):
    import paper_2503_05530_amd.binding as B
    c = draw_case(seed)
    dim, k, rho, q, metric = c["dim"], c["k"], c["rho"], c["q"], c["metric"]
    corpus = corpus_dev = None
    if c["n_docs"] > 0:
        x32 = W.corpus_f32(c["n_docs"], dim, seed)
        if metric != po.METRIC_L2:
            x32 = x32 * np.random.default_rng([seed, 98]).uniform(0.3, 3.0, size=(c["n_docs"], 1)).astype(np.float32)
        if c["bf16"]:
            corpus = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x32))
            corpus_dev = torch.from_numpy(x32).to(DEV).to(torch.bfloat16)
        else:
            corpus, corpus_dev = x32, torch.from_numpy(x32).to(DEV)
    planes = W.lsh_planes(c["lsh_bits"], dim, seed) if c["lsh_bits"] and c["capacity"] else None
    what = {key: v for key, v in c.items() if key not in ("q", "cuts")}

    if corpus is None:
        hit, src, dec = po.simulate_decisions(q, c["tau"], c["capacity"], c["policy"], planes=planes, metric=metric)
        want = None
    else:
        want = po.lookup_stream_deferred(corpus, q, c["tau"], c["capacity"], k, c["policy"], rerank_factor=rho,
                                         planes=planes, metric=metric)
        hit, src, dec = want[2], want[3], want[4]

    px = B.Proximity(corpus_dev, dim, c["capacity"], k, c["policy"], 256, device=DEV, rerank_factor=rho,
                     lsh_planes=None if planes is None else torch.from_numpy(planes).to(DEV), metric=metric)
    ids, dists, flags = [], [], []
    for r0, r1 in c["cuts"]:
        i, d, h = px.search_batch(torch.from_numpy(q[r0:r1]).to(DEV), c["tau"])
        ids.append(i); dists.append(d); flags.append(h)
    ids, dists, flags = (torch.cat(x).cpu().numpy() for x in (ids, dists, flags))
    assert (flags == hit).all(), f"{what}: flags differ first at {np.flatnonzero(flags != hit)[:5]}"
    if want is None:
        assert (ids == -1).all() and np.isinf(dists).all()
    else:
        P.assert_stream_parity((ids, dists, flags), want[:4], corpus, q,
                               dist_rtol=P.DIST_RTOL_BF16 if c["bf16"] else P.DIST_RTOL_F32, what=str(what),
                               reranked=rho > 1, metric=metric)
    seq, _, stored = px.cache_dump(want_ids=True)
    assert seq.tolist() == dec.dump_seq().tolist(), what
    if want is not None and len(seq):
        if rho > 1:
            want_stored = want[5][seq]
            if c["n_docs"] >= rho * k + 8:          # away from padding, stored lists must agree outright
                assert (stored == want_stored).all(), what
        else:
            assert (stored == ids[seq]).all(), what
    st, os_ = px.stats(), dec.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == os_[key], (what, key)
    px.close()


@pytest.mark.parametrize("trial", range(12))
def test_random_stream_at_larger_capacity(trial):
    """Cache decisions alone (no corpus) on longer streams against larger caches than the cases above:
    capacities 100 to 5 000, 2 000 to 6 000 rows cut into calls of up to 4 096, skewed reuse of the bases and
    radii on both sides of the tolerance, so that long candidate lists, the full-row fallback, hits on rows of
    the same call and thousands of evictions all occur; Euclidean and cosine."""
    import paper_2503_05530_amd.binding as B
    rng = np.random.default_rng([trial, 777])
    dim = int(rng.choice([32, 64, 128]))
    cap = int(rng.choice([100, 500, 2000, 5000]))
    policy = int(rng.integers(0, 2))
    metric = int(rng.choice([po.METRIC_L2, po.METRIC_L2, po.METRIC_COSINE]))
    max_batch = int(rng.choice([64, 1024, 4096]))
    n = int(rng.choice([2000, 6000]))
    n_bases = int(cap * rng.choice([0.3, 1.0, 2.5])) + 3
    tau = float(rng.choice([0.1, 0.3, 0.5]))
    bases = W.unit_rows(rng.standard_normal((n_bases, dim)))
    idx = np.minimum((rng.pareto(1.2, size=n) * n_bases / 10).astype(np.int64), n_bases - 1)
    radius = rng.choice([0.0, 0.05, 0.2, 0.35, 0.6], size=n)
    q = W.unit_rows(bases[idx] + radius[:, None] * W.unit_rows(rng.standard_normal((n, dim)))).astype(np.float32)
    if metric == po.METRIC_COSINE:
        q = (q * rng.uniform(0.5, 2.0, size=(n, 1))).astype(np.float32)
        tau = tau * tau / 2.0
    o_hit, _, dec = po.simulate_decisions(q, tau, cap, policy, metric=metric)
    px = B.Proximity(None, dim, cap, 3, policy, max_batch, device=DEV, metric=metric)
    flags, r0 = [], 0
    while r0 < n:
        step = int(rng.integers(1, max_batch + 1))
        _, _, h = px.search_batch(torch.from_numpy(q[r0:r0 + step]).to(DEV), tau)
        flags.append(h)
        r0 += step
    hit = torch.cat(flags).cpu().numpy()
    what = f"dim {dim} cap {cap} policy {policy} metric {metric} max_batch {max_batch} rows {n} tau {tau}"
    assert (hit == o_hit).all(), f"{what}: flags differ first at {np.flatnonzero(hit != o_hit)[:5]}"
    seq, _, _ = px.cache_dump()
    assert seq.tolist() == dec.dump_seq().tolist(), what
    st, os_ = px.stats(), dec.stats()
    for key in ("queries", "hits", "misses", "inserts", "evictions", "size"):
        assert st[key] == os_[key], (what, key)
    px.close()
