#!/usr/bin/env python3
"""Writes tests/golden/decisions_*.txt: the CPU oracle's hit/miss decisions on the full query
streams of the benchmark workloads.

    python tests/golden/make_stream_decisions.py [mid large lowreuse probe]

Everything stored comes from ``oracle/`` alone (Algorithm 1 replayed with the database call left
out: its branch reads only query-key distances) on inputs from the seeded generators; no value
is taken from the GPU library.  The literal replay of 100 000 queries against 300 float64 keys
takes about a minute per tolerance, and of 8 192 queries against 10 000 keys a few minutes, which
is why the GPU parity tests read these files instead of repeating the replay on the GPU machine;
``tests/test_stream_golden.py`` re-runs the oracle on prefixes and checks the files against it, and
against a textbook exact-match cache over base ids where the workload's geometry makes the two agree.

File format (text): one ``[name]`` section per (workload, tolerance); ``key = value`` lines;
``flags_hex`` is the hit flags packed most-significant-bit first (row 0 = top bit of the first
byte), in hexadecimal, wrapped (``flags_all = miss``: no row hit; ``flags_same_as``: identical to the
named section's); ``*_sha256`` are digests of little-endian int64 arrays.
"""
from __future__ import annotations

import hashlib
import os
import sys
import time
from multiprocessing import Pool

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import proximity_oracle as po                      # noqa: E402
from paper_2503_05530_amd import workloads as W                # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
PROBE_BATCHES = 2


def sha_i64(a) -> str:
    return hashlib.sha256(np.ascontiguousarray(a, dtype="<i8").tobytes()).hexdigest()


def flags_to_hex(flags) -> str:
    return np.packbits(np.asarray(flags, dtype=np.uint8)).tobytes().hex()


def section(name, fields) -> str:
    out = [f"[{name}]"]
    for key, val in fields:
        if key == "flags_hex":
            out.append("flags_hex =")
            out += [val[i:i + 120] for i in range(0, len(val), 120)]
            out.append("end")
        else:
            out.append(f"{key} = {val}")
    return "\n".join(out) + "\n"


def stream_task(args):
    name, tau = args
    w = W.WORKLOADS[name]
    q = W.stream_for(w)
    t0 = time.time()
    hit, src, orc = po.simulate_decisions(q, tau, w.capacity, w.policy)
    st = orc.stats()
    fields = [("workload", name), ("tau", repr(float(tau))), ("queries", len(q)), ("capacity", w.capacity),
              ("policy", "LRU" if w.policy == po.POLICY_LRU else "FIFO"),
              ("hits", st["hits"]), ("misses", st["misses"]), ("evictions", st["evictions"]), ("size", st["size"]),
              ("source_seq_sha256", sha_i64(src)),
              ("dump_seq", " ".join(str(int(s)) for s in orc.dump_seq())),
              ("flags_sha256", hashlib.sha256(np.packbits(hit).tobytes()).hexdigest()),
              ("flags_hex", flags_to_hex(hit))]
    print(f"{name} tau={tau}: {st['hits']} hits, {st['evictions']} evictions, {time.time() - t0:.0f} s", flush=True)
    return name, tau, fields


def warm_probe_oracle(keys, policy):
    """The oracle's state after the warm-up stream of the probe microbenchmark: distinct random unit vectors
    lie about 1.41 apart, far above the tolerance, so every one of them misses and is stored, in order
    (the GPU tests check that the library's warm-up indeed missed on every row)."""
    no_db = lambda q: (np.full(1, -1, np.int64), np.full(1, np.inf))
    orc = po.FlatCacheOracle(None, len(keys), 1, policy, retrieve=no_db)
    for t, key in enumerate(keys):
        orc.entries.append(po._Entry(po.as_f64_rows(key).copy(), np.full(1, -1, np.int64), np.full(1, np.inf), t))
    orc.n_queries = orc.n_misses = orc.n_inserts = orc.n_scans = len(keys)
    return orc


def probe_task(_):
    """Two batches of the probe microbenchmark drawn against the oracle's own resident keys (each batch
    depends on which keys are resident when it starts) and decided by the oracle row by row."""
    n_keys, dim, batch, tau = W.PROBE_KEYS, W.PROBE_DIM, W.PROBE_BATCH, W.PROBE_TAU
    keys = W.probe_warm_keys(n_keys, dim, 0)
    # the warm-up keys really are farther apart than tau (checked on a sample of pairs)
    sample = po.as_f64_rows(keys[:400])
    gram = sample @ sample.T
    np.fill_diagonal(gram, -1.0)
    assert np.sqrt(np.maximum(2.0 - 2.0 * gram.max(), 0.0)) > 1.0
    orc = warm_probe_oracle(keys, po.POLICY_LRU)
    mix = W.ProbeMix(dim, 0)
    out = []
    t0 = time.time()
    for b in range(PROBE_BATCHES):
        resident = orc.dump_keys().astype(np.float32)      # keys are float32 values held in float64: exact
        qb = mix.batch(resident, batch)
        hit = np.zeros(batch, dtype=np.uint8)
        src = np.zeros(batch, dtype=np.int64)
        near = {1e-5: 0, 1e-4: 0, 1e-3: 0}
        for t in range(batch):
            dmin = po.key_distances(qb[t], orc.dump_keys()).min()
            for rel in near:
                near[rel] += int(abs(dmin - tau) <= rel * tau)
            _, _, h, s = orc.lookup(qb[t], tau)
            hit[t], src[t] = int(h), s
            assert bool(h) == bool(dmin <= tau)
        st = orc.stats()
        out.append((f"probe batch={b}", [
            ("keys", n_keys), ("rows", batch), ("tau", repr(float(tau))), ("policy", "LRU"),
            ("batch_sha256", hashlib.sha256(qb.tobytes()).hexdigest()),
            ("hits_in_batch", int(hit.sum())), ("hits_total", st["hits"]), ("evictions_total", st["evictions"]),
            ("rows_within_1e-5_of_tau", near[1e-5]), ("rows_within_1e-4_of_tau", near[1e-4]),
            ("rows_within_1e-3_of_tau", near[1e-3]),
            ("source_seq_sha256", sha_i64(src)), ("dump_seq_sha256", sha_i64(orc.dump_seq())),
            ("flags_hex", flags_to_hex(hit))]))
        print(f"probe batch {b}: {int(hit.sum())} hits, {time.time() - t0:.0f} s", flush=True)
    return "probe", None, out


def main():
    which = sys.argv[1:] or ["mid", "large", "lowreuse", "probe"]
    tasks = []
    for name in which:
        if name == "probe":
            tasks.append((probe_task, None))
        else:
            w = W.WORKLOADS[name]
            for tau in (w.taus or (w.tau,)):
                tasks.append((stream_task, (name, tau)))
    with Pool(min(len(tasks), max(1, (os.cpu_count() or 2) - 1))) as pool:
        pending = [pool.apply_async(fn, (arg,)) for fn, arg in tasks]
        results = [p.get() for p in pending]
    header = ("# Written by tests/golden/make_stream_decisions.py from the CPU oracle (Algorithm 1, decisions only)\n"
              "# on the seeded synthetic streams; see that script for the format.  Do not edit by hand.\n")
    by_file = {}
    seen = {}                                   # flags already written in a file: (file, hex) -> section name
    for name, tau, payload in results:
        if name == "probe":
            by_file.setdefault("probe", []).extend(section(n, f) for n, f in payload)
            continue
        sec = f"{name} tau={tau!r}"
        fields = []
        for key, val in payload:
            if key == "flags_hex" and set(val) == {"0"}:
                fields.append(("flags_all", "miss"))            # no row hit: nothing to store
            elif key == "flags_hex" and (name, val) in seen:
                fields.append(("flags_same_as", seen[(name, val)]))
            else:
                if key == "flags_hex":
                    seen[(name, val)] = sec
                fields.append((key, val))
        by_file.setdefault(name, []).append(section(sec, fields))
    for name, parts in by_file.items():
        path = os.path.join(HERE, f"decisions_{name}.txt")
        with open(path, "w") as f:
            f.write(header + "\n".join(parts))
        print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
