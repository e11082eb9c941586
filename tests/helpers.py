"""Shared test helpers: brute-force checkers and small builders.

Nothing here belongs to the product path.  The checkers are written from the
definitions (covering invariant, acceptance band), not from the oracle's or the
HIP library's code.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np

import lc_workloads as wl
from oracle import lychee_oracle as orc


def rand_case(seed: int, T: int = 200, d: int = 8, lo: int = 2, hi: int = 12, G: int = 2,
              offset_std: float = 0.5, noise_std: float = 1.0, tail: int = 0):
    """Random chunked keys/values/query group in float64 (bf16-representable values)."""
    r = np.random.default_rng(seed)
    lens = []
    while sum(lens) < T - tail:
        lens.append(int(r.integers(lo, hi + 1)))
    lens[-1] -= sum(lens) - (T - tail)
    if lens[-1] <= 0:
        lens.pop()
    bounds = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(bounds[-1]) + tail
    M = len(lens)
    off = offset_std * r.standard_normal((M, d))
    chunk_of = np.repeat(np.arange(M), lens)
    K = noise_std * r.standard_normal((T, d))
    K[:bounds[-1]] += off[chunk_of]
    V = r.standard_normal((T, d))
    tgt = r.choice(M, size=min(3, M), replace=False)
    q = r.standard_normal((G, d)) + off[tgt].sum(axis=0)[None, :]
    rb = lambda a: wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(a.astype(np.float32)))
    return dict(K=rb(K), V=rb(V), q=rb(q), bounds=bounds, T=T, M=M, d=d, G=G)


def check_covering_invariant(idx: orc.Index, K: np.ndarray, slack: float = 1e-9) -> None:
    """Brute force: every node's ball covers every token key beneath it (TOKEN_BALL),
    and every descendant chunk's ball: |mu_j - mu_u| + r_j <= R_u."""
    K = np.asarray(K, dtype=np.float64)
    M = idx.M
    for level in range(idx.L):
        anc = idx.ancestor(level)
        for j in range(M):
            u = int(anc[j])
            mu, R = idx.center[level][u], idx.radius[level][u]
            reach = math.sqrt(float(((idx.center[0][j] - mu) ** 2).sum())) + idx.radius[0][j]
            assert reach <= R * (1 + slack) + slack, (level, u, j, reach, R)
            if idx.geometry == orc.TOKEN_BALL:
                toks = K[idx.bounds[j]:idx.bounds[j + 1]]
                dist = np.sqrt(((toks - mu[None, :]) ** 2).sum(axis=1)).max()
                assert dist <= R * (1 + slack) + slack, (level, u, j, dist, R)


def check_counts(idx: orc.Index) -> None:
    lens = idx.lens()
    for level in range(idx.L):
        anc = idx.ancestor(level)
        n = idx.n(level)
        ntok = np.bincount(anc, weights=lens, minlength=n).astype(np.int64)
        nch = np.bincount(anc, minlength=n).astype(np.int64)
        assert np.array_equal(ntok, idx.ntok[level]), level
        assert np.array_equal(nch, idx.nchunk[level]), level
    assert int(idx.ntok[idx.L - 1].sum()) == int(idx.bounds[-1])


def accept_ids(got: Sequence[int], scores: np.ndarray, lens: np.ndarray, budget: int,
               pinned: Sequence[int] = (), rel_band: float = 1e-5,
               candidates: Optional[Sequence[int]] = None, max_count: Optional[int] = None) -> None:
    """Acceptance rule for a chunk-id set computed in lower precision.

    `scores` are the oracle's (float64) scores of all chunks.  Let s_cut be the
    oracle score of the first chunk the oracle's selection rejects.  The set is
    accepted iff every candidate chunk scoring above s_cut + band is present,
    none scoring below s_cut - band is present, the ids are ascending and
    distinct, and the total length stays within the budget.  If nothing is
    rejected the set must equal the oracle's exactly.
    """
    got = [int(x) for x in got]
    assert got == sorted(set(got)), "ids must be ascending and distinct"
    pinned = set(int(p) for p in pinned)
    M = len(scores)
    cand = [j for j in (range(M) if candidates is None else candidates) if j not in pinned]
    assert pinned <= set(got), "pinned chunks missing"
    free = [j for j in got if j not in pinned]
    assert set(free) <= set(cand), "selected a chunk outside the candidate frontier"
    assert sum(int(lens[j]) for j in free) <= budget, "budget exceeded"
    if max_count is not None:
        assert len(free) <= max_count
    order = sorted(cand, key=lambda j: (-scores[j], j))
    total, m = 0, 0
    for j in order:
        if scores[j] == -math.inf or total + int(lens[j]) > budget:
            break
        if max_count is not None and m >= max_count:
            break
        total += int(lens[j])
        m += 1
    ref = sorted(order[:m])
    if m == len(order) or scores[order[m]] == -math.inf:
        assert free == ref, "everything fits: sets must be identical"
        return
    s_cut = scores[order[m]]
    band = rel_band * max(1.0, abs(s_cut))
    must = {j for j in cand if scores[j] > s_cut + band}
    never = {j for j in cand if scores[j] < s_cut - band}
    assert must <= set(free), f"missing {sorted(must - set(free))}"
    assert not (never & set(free)), f"spurious {sorted(never & set(free))}"


def dense_attention_library(q: np.ndarray, K: np.ndarray, V: np.ndarray):
    """Textbook softmax(q K^T / sqrt(d)) V through library routines (scipy), float64."""
    from scipy.special import logsumexp, softmax
    x = (np.asarray(q, np.float64) @ np.asarray(K, np.float64).T) / math.sqrt(q.shape[1])
    return softmax(x, axis=1) @ np.asarray(V, np.float64), logsumexp(x, axis=1)


TOPOLOGY_TIE = 2e-5     # a float32 dot product of two unit vectors of 128 entries is off by up to about 1e-5


def same_topology_or_near_tie(gi, oi, levels, where, tally):
    """The GPU-built tree `gi` must have the oracle's parents at every level below `levels` unless the
    oracle's own clustering of this tree passed through a near-tie (oi.min_margin <= TOPOLOGY_TIE), in
    which case a float32 assignment may legitimately fall the other way; such trees are counted in
    tally["near_tie"], matching ones in tally["same"].  Returns whether the topology matches."""
    same = all(np.array_equal(gi.parent[l], oi.parent[l]) for l in range(levels))
    if same:
        tally["same"] = tally.get("same", 0) + 1
    else:
        assert oi.min_margin <= TOPOLOGY_TIE, \
            f"{where}: topology differs from the oracle's although its clustering never came closer to a tie than {oi.min_margin:.3g}"
        tally["near_tie"] = tally.get("near_tie", 0) + 1
    return same
