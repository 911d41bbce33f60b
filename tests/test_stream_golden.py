"""The stored oracle decisions on the full benchmark streams (tests/golden/decisions_*.txt) against what fixes
them: the live oracle on stretches at the start, in the middle and at the end of each stream, a textbook
exact-match cache over base ids on every row, and the hit/eviction counts an independent simulation of the
same recipe reached (Algorithm 1 and the eviction policies of Section 3.3.2; the input recipe is the one in
paper_2503_05530_amd/workloads.py)."""
import hashlib

import numpy as np
import pytest

from oracle import proximity_oracle as po
from paper_2503_05530_amd import workloads as W

import stream_golden as SG

# hits / evictions over the whole stream, from a simulation independent of this repository's oracle
EXPECTED_COUNTS = {
    ("mid", 0.0): (0, 99_700), ("mid", 0.1): (0, 99_700),
    ("mid", 0.25): (69_624, 30_076), ("mid", 0.5): (69_624, 30_076), ("mid", 1.0): (69_624, 30_076),
    ("large", 0.5): (15_221, 4_479),
    ("lowreuse", 0.2): (435, 48_565),
}


def base_ids(w):
    if w.choice == "zipf":
        return W.zipf_choice(w.n_stream, w.n_bases, w.zipf_s, w.seed)
    return W.uniform_choice(w.n_stream, w.n_bases, w.seed)


@pytest.fixture(scope="module")
def streams():
    return {name: W.stream_for(W.WORKLOADS[name]) for name in ("mid", "large", "lowreuse")}


@pytest.mark.parametrize("name,tau", sorted(EXPECTED_COUNTS))
def test_stored_decisions_have_the_expected_counts_and_reduce_to_a_cache_over_base_ids(name, tau):
    w = W.WORKLOADS[name]
    sec = SG.read_decisions(name)[f"{name} tau={tau!r}"]
    hits, evictions = EXPECTED_COUNTS[(name, tau)]
    assert int(sec["queries"]) == w.n_stream and int(sec["capacity"]) == w.capacity
    assert (int(sec["hits"]), int(sec["evictions"])) == (hits, evictions)
    assert int(sec["misses"]) == w.n_stream - hits and int(sec["size"]) == min(w.capacity, w.n_stream - hits)
    flags = sec["flags"]
    assert len(flags) == w.n_stream and int(flags.sum()) == hits
    assert hashlib.sha256(np.packbits(flags).tobytes()).hexdigest() == sec["flags_sha256"]
    # below the rewording radius nothing ever hits: every query is its own key; above it the cache is an
    # exact-match cache over base ids
    keys = list(range(w.n_stream)) if hits == 0 else base_ids(w).tolist()
    model = SG.TextbookTrace(keys, w.capacity, w.policy)
    assert (model.flags == flags).all()
    assert SG.sha_i64(model.src) == sec["source_seq_sha256"]
    assert model.snapshots[w.n_stream] == [int(v) for v in sec["dump_seq"].split()]
    assert model.counters(w.n_stream)["evictions"] == evictions


@pytest.mark.parametrize("name,tau,stretches", [
    ("mid", 0.25, ((0, 1500), (50_000, 700), (99_300, 700))),
    ("mid", 0.0, ((0, 500), (99_600, 400))),
    ("mid", 1.0, ((70_000, 500),)),
    ("large", 0.5, ((0, 800), (10_000, 500), (19_500, 500))),
    ("lowreuse", 0.2, ((0, 1500), (25_000, 300), (49_700, 300))),
])
def test_stored_decisions_equal_the_live_oracle_at_start_middle_and_end(streams, name, tau, stretches):
    """The oracle itself, run again on stretches of each stream.  A stretch that does not begin at row 0 starts
    from the cache contents the textbook model gives for that position (keys = the queries at the resident
    inserting positions, in eviction order), which the stored final contents confirm for the whole stream."""
    w = W.WORKLOADS[name]
    q = streams[name]
    sec = SG.read_decisions(name)[f"{name} tau={tau!r}"]
    keys = list(range(w.n_stream)) if int(sec["hits"]) == 0 else base_ids(w).tolist()
    model = SG.TextbookTrace(keys, w.capacity, w.policy, snapshots=[p for p, _ in stretches])
    no_db = lambda v: (np.full(1, -1, np.int64), np.full(1, np.inf))
    for p, n in stretches:
        orc = po.FlatCacheOracle(None, w.capacity, 1, w.policy, retrieve=no_db)
        for pos in model.snapshots[p]:
            orc.entries.append(po._Entry(po.as_f64_rows(q[pos]).copy(), np.full(1, -1, np.int64), np.full(1, np.inf), pos))
        orc.n_queries = p
        _, _, hit, src = orc.lookup_stream(q[p:p + n], tau)
        assert (hit == sec["flags"][p:p + n]).all(), (name, tau, p)
        assert (src == model.src[p:p + n]).all(), (name, tau, p)
        if p + n == w.n_stream:
            assert orc.dump_seq().tolist() == [int(v) for v in sec["dump_seq"].split()]


def test_stored_probe_batches_equal_the_live_oracle():
    """The probe microbenchmark's first batch is redrawn from the seeds (same bytes as the stored digest) and the
    oracle decides its first rows again; the batch is the one whose distances straddle the tolerance."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location("make_stream_decisions",
                                                  os.path.join(SG.GOLDEN_DIR, "make_stream_decisions.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    secs = SG.read_decisions("probe")
    keys = W.probe_warm_keys(W.PROBE_KEYS, W.PROBE_DIM, 0)
    orc = gen.warm_probe_oracle(keys, po.POLICY_LRU)
    qb = W.ProbeMix(W.PROBE_DIM, 0).batch(keys, W.PROBE_BATCH)
    sec = secs["probe batch=0"]
    assert hashlib.sha256(qb.tobytes()).hexdigest() == sec["batch_sha256"]
    assert int(sec["keys"]) == W.PROBE_KEYS and int(sec["rows"]) == W.PROBE_BATCH and float(sec["tau"]) == W.PROBE_TAU
    n = 150
    hit = np.array([orc.lookup(qb[t], W.PROBE_TAU)[2] for t in range(n)], dtype=np.uint8)
    assert (hit == sec["flags"][:n]).all()
    for b in (0, 1):
        s = secs[f"probe batch={b}"]
        assert int(s["flags"].sum()) == int(s["hits_in_batch"])
        assert 0.10 < s["flags"].mean() < 0.40
    assert int(secs["probe batch=1"]["hits_total"]) == int(secs["probe batch=0"]["hits_in_batch"]) + \
        int(secs["probe batch=1"]["hits_in_batch"])
