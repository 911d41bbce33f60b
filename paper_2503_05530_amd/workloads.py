"""Seeded synthetic inputs: document corpora and ordered query streams.

The paper evaluates on embedded text collections (768-dimensional passage
embeddings, about 24 M passages for the largest index) and on query sets whose
popularity follows a Zipf law, where each repeat of a question is a slightly
different wording of it (Section 2.3, Section 4.2 "Query workload").  None of
those collections exists here, so this module draws stand-ins with the same
shapes: unit-norm Gaussian document vectors, a pool of unit-norm "base"
questions, and a stream in which every query is a base picked by rank
popularity plus a small random displacement (a rewording), re-normalised.

This file holds input generation only.  It computes no distance, runs no cache
and selects no neighbour: both the CPU oracle's tests and the GPU path's tests
draw their inputs from here, and neither side's arithmetic lives here.

Every array is produced by ``numpy.random.default_rng([seed, tag])`` with a
fixed tag per role, drawn in row order, so a stream prefix does not depend on
the stream length and chunked generation equals one-shot generation.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, Optional

import numpy as np

TAG_CORPUS = 0
TAG_BASES = 1
TAG_CHOICE = 2
TAG_PERTURB = 3
TAG_PROBE_MIX = 4
TAG_LSH_PLANES = 5

POLICY_FIFO = 0
POLICY_LRU = 1

DTYPE_F32 = 0
DTYPE_BF16 = 1


def _rng(seed: int, tag: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(tag)])


def unit_rows(v: np.ndarray) -> np.ndarray:
    """Scale every row to Euclidean length one (float64 in, float64 out)."""
    v = np.asarray(v, dtype=np.float64)
    return v / np.sqrt(np.sum(v * v, axis=-1, keepdims=True))


def corpus_f32(n_docs: int, dim: int, seed: int, chunk_rows: int = 1 << 16) -> np.ndarray:
    """Document embeddings: rows iid N(0,1), scaled to unit length, stored as float32."""
    rng = _rng(seed, TAG_CORPUS)
    out = np.empty((n_docs, dim), dtype=np.float32)
    for r0 in range(0, n_docs, chunk_rows):
        r1 = min(n_docs, r0 + chunk_rows)
        out[r0:r1] = unit_rows(rng.standard_normal((r1 - r0, dim))).astype(np.float32)
    return out


def base_queries(n_bases: int, dim: int, seed: int) -> np.ndarray:
    """The pool of distinct questions (float64, unit length)."""
    return unit_rows(_rng(seed, TAG_BASES).standard_normal((n_bases, dim)))


def zipf_choice(n_stream: int, n_bases: int, s: float, seed: int) -> np.ndarray:
    """Index of the base each stream position repeats: rank r is drawn with weight r**-s."""
    p = np.arange(1, n_bases + 1, dtype=np.float64) ** (-float(s))
    cdf = np.cumsum(p) / np.sum(p)
    u = _rng(seed, TAG_CHOICE).random(n_stream)
    idx = np.searchsorted(cdf, u, side="right")
    return np.minimum(idx, n_bases - 1).astype(np.int64)


def uniform_choice(n_stream: int, n_bases: int, seed: int) -> np.ndarray:
    """Index of the base each stream position repeats, all bases equally likely."""
    u = _rng(seed, TAG_CHOICE).random(n_stream)
    return np.minimum(np.floor(u * n_bases).astype(np.int64), n_bases - 1)


def perturbed_stream(bases: np.ndarray, idx: np.ndarray, radius: float, seed: int,
                     chunk_rows: int = 1 << 14) -> np.ndarray:
    """Queries = unit(base[idx[t]] + radius * unit(g_t)), g_t iid N(0, I), stored as float32."""
    rng = _rng(seed, TAG_PERTURB)
    n, dim = len(idx), bases.shape[1]
    out = np.empty((n, dim), dtype=np.float32)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        g = unit_rows(rng.standard_normal((r1 - r0, dim)))
        out[r0:r1] = unit_rows(bases[idx[r0:r1]] + float(radius) * g).astype(np.float32)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@dataclass(frozen=True)
class Workload:
    """One named configuration: corpus shape, stream recipe and cache parameters."""
    name: str
    n_docs: int
    dim: int
    corpus_dtype: int
    n_bases: int
    n_stream: int
    choice: str            # "zipf" or "uniform"
    zipf_s: float
    radius: float
    capacity: int
    policy: int
    tau: float
    k: int
    batch: int
    seed: int = 0
    taus: tuple = field(default_factory=tuple)
    batches: tuple = field(default_factory=tuple)


WORKLOADS = {
    "tiny": Workload("tiny", 10_000, 768, DTYPE_F32, 200, 1_000, "zipf", 1.1, 0.1,
                     50, POLICY_FIFO, 0.25, 10, 1),
    "mid": Workload("mid", 1_000_000, 768, DTYPE_F32, 5_000, 100_000, "zipf", 1.1, 0.1,
                    300, POLICY_LRU, 0.25, 10, 1,
                    taus=(0.0, 0.1, 0.25, 0.5, 1.0), batches=(1, 64)),
    "large": Workload("large", 24_000_000, 768, DTYPE_F32, 2_000, 20_000, "zipf", 1.1, 0.1,
                      300, POLICY_LRU, 0.5, 32, 256),
    "lowreuse": Workload("lowreuse", 8_000_000, 384, DTYPE_BF16, 100_000, 50_000, "uniform", 0.0,
                         0.05, 1_000, POLICY_FIFO, 0.2, 100, 128),
}

# The cache-probe microbenchmark has no corpus: 10 000 resident keys, batches of
# 4 096 queries, tolerance 0.3, least-recently-used replacement.
PROBE_KEYS = 10_000
PROBE_DIM = 768
PROBE_BATCH = 4_096
PROBE_TAU = 0.3
PROBE_MAX_RADIUS = 0.6


def stream_for(w: Workload, n_stream: Optional[int] = None) -> np.ndarray:
    """The query stream of a workload (a prefix of it if ``n_stream`` is given)."""
    n = w.n_stream if n_stream is None else int(n_stream)
    b = base_queries(w.n_bases, w.dim, w.seed)
    if w.choice == "zipf":
        idx = zipf_choice(w.n_stream, w.n_bases, w.zipf_s, w.seed)[:n]
    else:
        idx = uniform_choice(w.n_stream, w.n_bases, w.seed)[:n]
    return perturbed_stream(b, idx, w.radius, w.seed)


def corpus_for(w: Workload, n_docs: Optional[int] = None) -> np.ndarray:
    """Host corpus of a workload as float32 (a prefix of it if ``n_docs`` is given).

    For the bfloat16 workload the caller rounds with :func:`f32_to_bf16_bits`;
    rows are not re-normalised after rounding.
    """
    return corpus_f32(w.n_docs if n_docs is None else int(n_docs), w.dim, w.seed)


def lsh_planes(n_bits: int, dim: int, seed: int) -> np.ndarray:
    """Normals of ``n_bits`` random hyperplanes through the origin (standard Gaussian), float32 [n_bits][dim].
    They are an input of the bucketed cache, handed to the oracle and to the library alike."""
    return _rng(seed, TAG_LSH_PLANES).standard_normal((n_bits, dim)).astype(np.float32)


def probe_warm_keys(n_keys: int, dim: int, seed: int) -> np.ndarray:
    """Fresh unit Gaussian vectors that fill the probe microbenchmark's cache."""
    return unit_rows(_rng(seed, TAG_CORPUS).standard_normal((n_keys, dim))).astype(np.float32)


class ProbeMix:
    """Batches for the probe microbenchmark.

    Half of the queries (by a fair coin) are a key that is resident when the
    batch starts, displaced by a random vector of length U(0, 0.6) and
    re-normalised; the other half are fresh unit Gaussian vectors.  The caller
    supplies the resident keys, because which keys are resident depends on the
    cache's history.
    """

    def __init__(self, dim: int, seed: int, max_radius: float = PROBE_MAX_RADIUS):
        self.dim = dim
        self.max_radius = float(max_radius)
        self.rng = _rng(seed, TAG_PROBE_MIX)

    def batch(self, resident_keys: np.ndarray, n: int) -> np.ndarray:
        rng = self.rng
        coin = rng.random(n) < 0.5
        pick = np.minimum(np.floor(rng.random(n) * len(resident_keys)).astype(np.int64),
                          max(len(resident_keys) - 1, 0))
        radius = self.max_radius * rng.random(n)
        g = unit_rows(rng.standard_normal((n, self.dim)))
        fresh = unit_rows(rng.standard_normal((n, self.dim)))
        out = fresh
        if len(resident_keys):
            near = unit_rows(np.asarray(resident_keys, dtype=np.float64)[pick] + radius[:, None] * g)
            out = np.where(coin[:, None], near, fresh)
        return out.astype(np.float32)


def device_corpus_chunks(n_docs: int, dim: int, seed: int, device, dtype_code: int,
                         chunk_rows: int = 1 << 20) -> Iterator:
    """Yield (row_begin, tensor) chunks of a corpus drawn on the device.

    Corpora too large to draw on the host in reasonable time are generated
    with a seeded ``torch.Generator`` on the device, one fixed-size chunk of
    rows at a time (chunk c uses seed ``seed * 1_000_003 + c``), so the same
    rows come back for the same (seed, chunk_rows) on the same software stack.
    Rows are unit-normalised in float32; bfloat16 corpora are the rounding of
    those rows.
    """
    import torch

    for c, r0 in enumerate(range(0, n_docs, chunk_rows)):
        r1 = min(n_docs, r0 + chunk_rows)
        g = torch.Generator(device=device)
        g.manual_seed(int(seed) * 1_000_003 + c)
        x = torch.randn((r1 - r0, dim), generator=g, device=device, dtype=torch.float32)
        x = x / torch.linalg.vector_norm(x, dim=1, keepdim=True)
        if dtype_code == DTYPE_BF16:
            x = x.to(torch.bfloat16)
        yield r0, x
