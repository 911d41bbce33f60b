"""Reader for tests/golden/decisions_*.txt (the CPU oracle's decisions on the full benchmark streams, written by
tests/golden/make_stream_decisions.py) and the textbook exact-match cache the streams reduce to.

Why a textbook cache applies: in the tiny, mid, large and low-reuse workloads two rewordings of one base question
lie about 0.14 (0.07) apart and different bases more than 1.2 apart, so for a tolerance between the two the
approximate cache hits exactly when a key of the same base is resident: a classical FIFO/LRU cache keyed by base
id.  tests/test_stream_golden.py shows the oracle's stored decisions equal to that model row for row; the GPU
tests then take flags, answering rows and cache contents at any stream position from the model.
"""
from __future__ import annotations

import collections
import hashlib
import os

import numpy as np

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def sha_i64(a) -> str:
    return hashlib.sha256(np.ascontiguousarray(a, dtype="<i8").tobytes()).hexdigest()


def read_decisions(name: str) -> dict:
    """Sections of decisions_<name>.txt as {section: {key: value}}; 'flags' is a uint8 array of 'queries' (or
    'rows') entries."""
    sections, cur, in_hex = {}, None, False
    for line in open(os.path.join(GOLDEN_DIR, f"decisions_{name}.txt")):
        line = line.rstrip("\n")
        if in_hex:
            if line == "end":
                in_hex = False
            else:
                cur["flags_hex"] += line
            continue
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = sections.setdefault(line[1:-1], {})
            continue
        key, _, val = line.partition("=")
        key, val = key.strip(), val.strip()
        if key == "flags_hex":
            cur["flags_hex"], in_hex = "", True
        else:
            cur[key] = val
    for sec in sections.values():
        n = int(sec.get("queries", sec.get("rows")))
        if sec.get("flags_all") == "miss":
            sec["flags"] = np.zeros(n, dtype=np.uint8)
        elif "flags_same_as" in sec:
            sec["flags_hex"] = sections[sec["flags_same_as"]]["flags_hex"]
        if "flags_hex" in sec:
            sec["flags"] = np.unpackbits(np.frombuffer(bytes.fromhex(sec["flags_hex"]), dtype=np.uint8))[:n]
    return sections


class TextbookTrace:
    """A classical exact-match FIFO (policy 0) or LRU (policy 1) cache over hashable keys, replayed over a key
    sequence: hit flags, the position whose insertion answers each position (itself on a miss), and the
    resident keys' inserting positions in eviction order after any prefix."""

    def __init__(self, keys, capacity: int, policy: int, snapshots=()):
        store = collections.OrderedDict()          # key -> inserting position, next victim first
        n = len(keys)
        self.flags = np.zeros(n, dtype=np.uint8)
        self.src = np.arange(n, dtype=np.int64)
        self.evictions_upto = np.zeros(n + 1, dtype=np.int64)
        self.snapshots = {}
        want = set(int(p) for p in snapshots)
        ev = 0
        for t, key in enumerate(keys):
            if t in want:
                self.snapshots[t] = list(store.values())
            if key in store:
                self.flags[t] = 1
                self.src[t] = store[key]
                if policy == 1:
                    store.move_to_end(key)
            elif capacity > 0:
                if len(store) >= capacity:
                    store.popitem(last=False)
                    ev += 1
                store[key] = t
            self.evictions_upto[t + 1] = ev
        self.snapshots[n] = list(store.values())
        self.capacity = capacity

    def counters(self, n: int) -> dict:
        """Counters of Algorithm 1 after the first n positions."""
        hits = int(self.flags[:n].sum())
        misses = n - hits
        return dict(queries=n, hits=hits, misses=misses, inserts=misses if self.capacity > 0 else 0,
                    evictions=int(self.evictions_upto[n]), size=min(self.capacity, misses))
