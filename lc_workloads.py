"""Seeded synthetic inputs for the LycheeCluster decode hot path.

This module only *draws inputs* (chunk boundaries, keys, values, queries) and
converts between bf16 bit patterns and wider floats.  It holds none of the
method's arithmetic, so both the CPU oracle's tests and the HIP path's tests
and benchmark may use it.

The workloads stand in for the long-context benchmarks the paper evaluates on
(Section 5.1): they reproduce the *shapes* the method sees at decode time --
Llama-style grouped-query attention (32 query / 8 KV heads, head_dim 128),
contexts of 4K to 128K tokens cut into variable-length chunks -- with keys that
cluster per chunk (a shared per-chunk offset plus unit noise) and queries that
lean toward a few target chunks, so that retrieval has something to find.

Recipe (all draws from numpy PCG64 streams seeded per (config, sequence)):
  * chunk lengths: drawn one by one from the config's distribution until they
    cover T tokens; the last chunk is truncated to end at T and, if that
    leaves it shorter than the minimum length, merged into the previous one.
  * keys:   k_i = z_i + o_chunk(i),  z ~ N(0, I),  o_j ~ N(0, 0.5^2 I) drawn per
            (KV head, chunk); rounded once to bf16.
  * values: N(0, I), rounded once to bf16.
  * queries: for each KV head pick `n_targets` chunks; every query head of the
            group gets q = z + beta * sum of those chunks' offsets; bf16.
  * streamed tokens (streaming config): k = z + m_t with m_t a random walk of
            step std 0.02 per dimension; chunk close lengths uniform in a range.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------
# bf16 <-> float conversions (bit-level; round-to-nearest-even)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest, ties to even); return uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int                 # enters the seed
    B: int
    H_q: int
    H_kv: int
    d: int
    T: int                      # tokens per sequence (or 0 if ragged, see T_range)
    chunk_dist: str             # "uniform" | "lognormal"
    chunk_lo: int
    chunk_hi: int
    levels: int
    fanout: int
    budget: int
    T_range: Optional[Tuple[int, int]] = None      # ragged batch: T_b ~ U{lo..hi}
    lognormal_median: float = 48.0
    lognormal_sigma: float = 0.6
    n_queries: int = 1          # independent decode queries per sequence
    n_targets: int = 3
    beta: float = 1.0
    stream_steps: int = 0       # streaming config: decode steps after prefill
    stream_close_lo: int = 16
    stream_close_hi: int = 64
    stream_drift: float = 0.02
    fanouts: Optional[Tuple[int, ...]] = None      # per-level fan-outs (entry l >= 1: children per level-l node), None = fanout
    beam: Optional[Tuple[int, ...]] = None         # nodes kept per level under the top-k policy (entry 0: chunks, 0 = no limit)

    @property
    def G(self) -> int:
        return self.H_q // self.H_kv


C1 = Workload("C1-4K", 1, 1, 32, 8, 128, 4096, "uniform", 8, 64, 2, 16, 1024)
C2 = Workload("C2-32Kx4", 2, 4, 32, 8, 128, 32768, "uniform", 16, 128, 3, 16, 2048, n_queries=64)
C3 = Workload("C3-128K", 3, 1, 32, 8, 128, 131072, "lognormal", 8, 256, 4, 16, 4096)
C4 = Workload("C4-stream", 4, 1, 32, 8, 128, 32768, "uniform", 16, 64, 3, 16, 2048,
              stream_steps=2048)
C5 = Workload("C5-ragged16", 5, 16, 28, 4, 128, 0, "uniform", 8, 128, 3, 32, 2048,
              T_range=(16384, 65536))

# The paper's own tiers at the headline context (Appendix A: chunks of 8 to 16 tokens, 2 chunks per fine
# cluster, budget 1024; 22 fine clusters per coarse unit gives about 250 coarse units): not one of the
# five configurations, used to compare the top-k policy of Algorithm 1 with the flat scan where the
# index is large.
P3 = Workload("P3-128K-paper-tiers", 6, 1, 32, 8, 128, 131072, "uniform", 8, 16, 3, 16, 1024,
              fanouts=(0, 2, 22), beam=(0, 43, 8))

WORKLOADS = {w.name: w for w in (C1, C2, C3, C4, C5, P3)}


def tiny(name: str = "tiny", **kw) -> Workload:
    """A small workload of the same structure, for tests the oracle finishes instantly."""
    base = Workload(name, 99, 1, 8, 2, 128, 512, "uniform", 4, 24, 2, 4, 128)
    return replace(base, **kw)


def _rng(w: Workload, seq: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([1000 * w.cfg_id + seq, stream]))


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------

def seq_lengths(w: Workload) -> List[int]:
    if w.T_range is None:
        return [w.T] * w.B
    r = _rng(w, 0, stream=7)
    return [int(x) for x in r.integers(w.T_range[0], w.T_range[1] + 1, size=w.B)]


def draw_chunk_bounds(w: Workload, seq: int, T: int) -> np.ndarray:
    """Chunk boundaries b_0=0 < b_1 < ... < b_M = T (int32)."""
    r = _rng(w, seq, stream=1)
    lens: List[int] = []
    total = 0
    while total < T:
        if w.chunk_dist == "uniform":
            n = int(r.integers(w.chunk_lo, w.chunk_hi + 1))
        elif w.chunk_dist == "lognormal":
            n = int(round(float(np.exp(r.normal(np.log(w.lognormal_median), w.lognormal_sigma)))))
            n = min(max(n, w.chunk_lo), w.chunk_hi)
        else:
            raise ValueError(w.chunk_dist)
        lens.append(n)
        total += n
    lens[-1] -= total - T
    if len(lens) > 1 and lens[-1] < w.chunk_lo:
        last = lens.pop()
        lens[-1] += last
    b = np.zeros(len(lens) + 1, dtype=np.int32)
    b[1:] = np.cumsum(lens)
    assert b[-1] == T
    return b


@dataclass
class SeqInputs:
    T: int
    bounds: np.ndarray          # int32 [M+1]
    K: np.ndarray               # uint16 bf16 bits [H_kv, T, d]
    V: np.ndarray               # uint16 bf16 bits [H_kv, T, d]
    offsets: np.ndarray         # float32 [H_kv, M, d]   (the per-chunk key offsets)
    Q: np.ndarray               # uint16 bf16 bits [n_queries, H_q, d]
    targets: np.ndarray         # int32 [n_queries, H_kv, n_targets]


def make_sequence(w: Workload, seq: int, T: Optional[int] = None,
                  offset_std: float = 0.5, noise_std: float = 1.0) -> SeqInputs:
    """Draw one sequence's bounds, K, V and queries."""
    if T is None:
        T = seq_lengths(w)[seq]
    bounds = draw_chunk_bounds(w, seq, T)
    M = len(bounds) - 1
    lens = np.diff(bounds)
    r = _rng(w, seq, stream=2)
    offsets = (offset_std * r.standard_normal((w.H_kv, M, w.d), dtype=np.float32))
    K = np.empty((w.H_kv, T, w.d), dtype=np.uint16)
    V = np.empty((w.H_kv, T, w.d), dtype=np.uint16)
    chunk_of = np.repeat(np.arange(M), lens)
    for h in range(w.H_kv):
        z = r.standard_normal((T, w.d), dtype=np.float32)
        if noise_std != 1.0:
            z *= np.float32(noise_std)
        z += offsets[h][chunk_of]
        K[h] = f32_to_bf16_bits(z)
        V[h] = f32_to_bf16_bits(r.standard_normal((T, w.d), dtype=np.float32))
    Q, targets = make_queries(w, seq, offsets, w.n_queries)
    return SeqInputs(T, bounds, K, V, offsets, Q, targets)


def make_queries(w: Workload, seq: int, offsets: np.ndarray, n_queries: int,
                 stream: int = 3) -> Tuple[np.ndarray, np.ndarray]:
    """Queries biased toward `n_targets` random chunks per KV head."""
    r = _rng(w, seq, stream=stream)
    H_kv, M, d = offsets.shape
    G = w.G
    nt = min(w.n_targets, M)
    Q = np.empty((n_queries, w.H_q, d), dtype=np.uint16)
    targets = np.empty((n_queries, H_kv, nt), dtype=np.int32)
    for i in range(n_queries):
        for h in range(H_kv):
            t = r.choice(M, size=nt, replace=False)
            targets[i, h] = t
            bias = w.beta * offsets[h, t].sum(axis=0)
            z = r.standard_normal((G, d), dtype=np.float32) + bias[None, :]
            Q[i, h * G:(h + 1) * G] = f32_to_bf16_bits(z)
    return Q, targets


@dataclass
class StreamInputs:
    k: np.ndarray               # uint16 [steps, H_kv, d]
    v: np.ndarray               # uint16 [steps, H_kv, d]
    q: np.ndarray               # uint16 [steps, H_q, d]
    close: np.ndarray           # uint8  [steps]  1 where the open chunk closes after this token


def make_stream(w: Workload, seq: int, steps: Optional[int] = None) -> StreamInputs:
    """Streamed decode tokens with a slowly drifting key mean, and close decisions."""
    steps = w.stream_steps if steps is None else steps
    r = _rng(w, seq, stream=4)
    drift = np.cumsum(w.stream_drift * r.standard_normal((steps, w.H_kv, w.d), dtype=np.float32), axis=0)
    k = f32_to_bf16_bits(r.standard_normal((steps, w.H_kv, w.d), dtype=np.float32) + drift)
    v = f32_to_bf16_bits(r.standard_normal((steps, w.H_kv, w.d), dtype=np.float32))
    q = f32_to_bf16_bits(r.standard_normal((steps, w.H_q, w.d), dtype=np.float32)
                         + np.repeat(drift, w.G, axis=1) * 4.0)
    close = np.zeros(steps, dtype=np.uint8)
    pos = 0
    while True:
        pos += int(r.integers(w.stream_close_lo, w.stream_close_hi + 1))
        if pos > steps:
            break
        close[pos - 1] = 1
    return StreamInputs(k, v, q, close)
