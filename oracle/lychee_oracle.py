"""CPU oracle for the LycheeCluster decode hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy implementation of what the path computes, written
from the paper so that a reader can check it against the text by eye.  It
shares no code with the HIP library and is never used by the product path:
only the tests, the smoke check and the benchmark's CPU-baseline leg import it.

What follows the paper directly
  * attention over an active token set            -- Eq. 1, Section 4.1
  * chunk representative = mean-pooled keys, and its unit direction
                                                  -- Section 4.1 / 4.3
  * node = (centroid, covering radius)            -- Section 4.1
  * score upper bound  q.mu + |q| r               -- Eq. 2
  * spherical k-means, inner-product similarity, 10 fixed iterations
                                                  -- Section 4.3, Appendix A
  * top-down pruning with per-level top-k         -- Algorithm 1 (steps 1-2)
  * lazy update: nearest fine cluster, moving-average centroid, monotone
    radius growth                                 -- Section 4.4, Algorithm 1 (step 4)
  * budget >= context degenerates to full attention -- Appendix F.1

Readings taken where the paper is silent (each is listed in the design notes):
  * a chunk is itself a node with its own (center, radius); with the default
    TOKEN_BALL geometry the center is the un-normalised mean key and the radius
    covers the chunk's token keys, so Eq. 2 bounds every token logit;
    PAPER_UNIT keeps the literal unit-norm representative with radius 0.
  * an internal node's radius covers the balls of all descendant chunks.
  * grouped-query heads sharing a KV head share one selection; the group score
    is the maximum of the per-head bounds.
  * scores are divided by sqrt(d) so that they bound the logits of Eq. 1.
  * selection: sort by (score descending, id ascending) and keep the longest
    prefix whose token total fits the budget (no skipping).
  * EXACT policy: the result is *defined* as the flat scan over all chunks; the
    hierarchical variants must reproduce it.  BEAM policy: Algorithm 1 with a
    top-k per level.
  * lazy update: count-weighted cumulative mean; the radius also grows by the
    centroid shift so that old members stay covered.
  * stored centers are float32 values (chunk-level centers optionally
    bfloat16 values), stored radii are rounded *up* to float32 and measured
    against the stored (rounded) centers.

Parity status: every function below is pinned by tests/test_oracle_*.py
(brute force, closed forms, library routines, a hand-worked example).  The
clustering is pinned by iterating a library's nearest-codeword search (which
on the unit sphere is the inner-product assignment) from the same start, and
by invariants (objective monotone, k = N, separated clusters recovered).
"""
from __future__ import annotations

import heapq
import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

TOKEN_BALL = 0
PAPER_UNIT = 1

POLICY_EXACT = 0
POLICY_BEAM = 1

CENTER_F32 = 0      # chunk-level centers stored as float32
CENTER_BF16 = 1     # chunk-level centers stored as bfloat16 (the levels above stay float32)

NEG_INF = -math.inf


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------

def store_f32(x) -> np.ndarray:
    """Round to the nearest float32 and return as float64 (a stored value)."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def store_bf16(x) -> np.ndarray:
    """Round to the nearest bfloat16 (8 significant bits, ties to even; normal range) and return as
    float64: x = m 2^e with 0.5 <= |m| < 1, and m is rounded to a multiple of 2^-8."""
    m, e = np.frexp(np.asarray(x, dtype=np.float64))
    return np.ldexp(np.round(m * 256.0) / 256.0, e)


def store_center0(x, center_dtype: int) -> np.ndarray:
    """A chunk-level center as it is stored."""
    return store_bf16(x) if center_dtype == CENTER_BF16 else store_f32(x)


def round_up_f32(x) -> np.ndarray:
    """Smallest float32 that is >= x, returned as float64."""
    x = np.asarray(x, dtype=np.float64)
    f = x.astype(np.float32)
    low = f.astype(np.float64) < x
    f = np.where(low, np.nextafter(f, np.float32(np.inf)), f)
    return f.astype(np.float64)


def unit(v: np.ndarray) -> np.ndarray:
    """Project onto the unit sphere; the zero vector maps to e_0 (paper silent)."""
    v = np.asarray(v, dtype=np.float64)
    n = math.sqrt(float(v @ v))
    if n == 0.0:
        e = np.zeros_like(v)
        e[0] = 1.0
        return e
    return v / n


def unit_rows(X: np.ndarray) -> np.ndarray:
    return np.stack([unit(x) for x in X]) if len(X) else np.zeros_like(X)


# --------------------------------------------------------------------------
# the index of one (sequence, KV head)
# --------------------------------------------------------------------------

@dataclass
class Index:
    """Stored hierarchical index.  Level 0 = chunks, level L-1 = top.

    center[l]  [N_l, d]  float64 holding float32-representable values (level 0: bfloat16-
                         representable ones when center_dtype is CENTER_BF16)
    radius[l]  [N_l]     float64 holding float32-representable values (-inf: empty node)
    parent[l]  [N_l]     int64, index into level l+1 (-1 at the top level)
    ntok[l]    [N_l]     tokens in the subtree
    nchunk[l]  [N_l]     chunks in the subtree (1 at level 0)
    bounds     [M+1]     token boundaries of the closed chunks
    T                    tokens written so far; [bounds[-1], T) is the open tail
    """
    d: int
    L: int
    F: object                      # int, or per-level sequence (see level_fanout)
    geometry: int
    bounds: np.ndarray
    T: int
    center: List[np.ndarray]
    radius: List[np.ndarray]
    parent: List[np.ndarray]
    ntok: List[np.ndarray]
    nchunk: List[np.ndarray]
    center_dtype: int = CENTER_F32
    radius_build: Optional[List[np.ndarray]] = None   # radii as the last (re)build left them: the baseline of
                                                      # radius_drift(); the lazy update never touches it
    min_margin: float = float("inf")   # build only: smallest best-vs-second-best similarity gap the
                                       # clustering passed through (how near it came to a tie); not
                                       # part of the stored index

    @property
    def M(self) -> int:
        return len(self.bounds) - 1

    def n(self, level: int) -> int:
        return len(self.radius[level])

    def lens(self) -> np.ndarray:
        return np.diff(self.bounds)

    def children(self, level: int, node: int) -> np.ndarray:
        """Ids at level-1 whose parent is `node` (ascending)."""
        return np.nonzero(self.parent[level - 1] == node)[0]

    def ancestor(self, level: int) -> np.ndarray:
        """For every chunk, its ancestor's id at `level`."""
        a = np.arange(self.M)
        for l in range(level):
            a = self.parent[l][a]
        return a


# --------------------------------------------------------------------------
# index construction (prefill)  -- Section 4.3
# --------------------------------------------------------------------------

def chunk_node(keys: np.ndarray, geometry: int,
               center_dtype: int = CENTER_F32) -> Tuple[np.ndarray, float, np.ndarray]:
    """(stored center, stored radius, mean key) of one chunk from its token keys [n, d].

    The representative is the mean-pooled key (Section 4.1).  TOKEN_BALL stores
    the mean itself and the radius that covers the chunk's token keys -- measured
    from the center as stored, whatever its storage rounding; PAPER_UNIT stores
    the unit-norm representative with radius 0.
    """
    keys = np.asarray(keys, dtype=np.float64)
    c = keys.sum(axis=0) / keys.shape[0]
    if geometry == TOKEN_BALL:
        mu = store_center0(c, center_dtype)
        diff = keys - mu[None, :]
        r = float(round_up_f32(np.sqrt((diff * diff).sum(axis=1)).max()))
    else:
        mu = store_center0(unit(c), center_dtype)
        r = 0.0
    return mu, r, c


def direction_of(center: np.ndarray) -> np.ndarray:
    """Unit direction of a stored center: what clustering and nearest-cluster search compare."""
    return unit(center)


def spherical_kmeans(X: np.ndarray, k: int, iters: int,
                     trace: Optional[list] = None, margins: Optional[list] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Spherical k-means on unit rows X [N, d] (Section 4.3; Appendix A: 10 iterations).

    Similarity is the inner product.  Initial centroid c is the point with
    index floor(c*N/k).  One iteration = assign every point to the centroid of
    largest inner product (ties -> lower centroid id), then replace each
    centroid by the normalised sum of its members; a cluster with no members
    (or a zero sum) keeps its previous centroid.  Returns (labels, centroids)
    where labels come from the last assignment and centroids from the last
    update.  `trace`, if given, receives the objective sum_i <x_i, m_label(i)>
    measured right after each assignment; `margins`, if given, receives per
    iteration the smallest gap between a point's best and second-best similarity
    (how close the assignment came to a tie; instrumentation only).
    """
    N = X.shape[0]
    m = np.stack([X[(c * N) // k] for c in range(k)]).astype(np.float64)
    labels = np.zeros(N, dtype=np.int64)
    for _ in range(iters):
        sim = X @ m.T                                   # [N, k]
        labels = np.argmax(sim, axis=1)                 # first maximum = lowest id
        if trace is not None:
            trace.append(float(sim[np.arange(N), labels].sum()))
        if margins is not None and k >= 2 and N > 0:
            top2 = np.partition(sim, k - 2, axis=1)[:, k - 2:]
            margins.append(float((top2[:, 1] - top2[:, 0]).min()))
        for c in range(k):
            members = X[labels == c]
            if len(members) == 0:
                continue
            s = members.sum(axis=0)
            if float(s @ s) == 0.0:
                continue
            m[c] = unit(s)
    return labels, m


def level_fanout(F, level: int) -> int:
    """Average number of children of a node at `level` (>= 1): F itself, or F[level] when the levels
    have fan-outs of their own (the paper's tiers: 2 chunks per fine cluster, at most 64 coarse units;
    Appendix A)."""
    if isinstance(F, (int, np.integer)):
        return int(F)
    return int(F[level])


def build_index(K: np.ndarray, bounds: Sequence[int], T: int, L: int, F,
                iters: int = 10, geometry: int = TOKEN_BALL, center_dtype: int = CENTER_F32) -> Index:
    """Build the index of one (sequence, KV head).

    K [>=T, d] float64 keys; bounds[0..M] boundaries of the closed chunks
    (bounds[0] = 0, bounds[M] <= T); tokens [bounds[M], T) are the open tail.
    Levels: 0 = chunks, then L-1 rounds of spherical k-means with
    k = ceil(N/F) clusters on the unit directions of the level below (F an int,
    or a sequence with F[level] for the level being formed).
    """
    K = np.asarray(K, dtype=np.float64)
    bounds = np.asarray(bounds, dtype=np.int64)
    M = len(bounds) - 1
    d = K.shape[1]
    assert bounds[0] == 0 and bounds[-1] <= T and np.all(np.diff(bounds) >= 1)

    center0 = np.zeros((M, d))
    radius0 = np.zeros(M)
    for j in range(M):
        center0[j], radius0[j], _ = chunk_node(K[bounds[j]:bounds[j + 1]], geometry, center_dtype)
    idx = Index(d=d, L=L, F=F, geometry=geometry, center_dtype=center_dtype, bounds=bounds.copy(), T=int(T),
                center=[center0], radius=[radius0],
                parent=[np.full(M, -1, dtype=np.int64)],
                ntok=[np.diff(bounds).astype(np.int64)],
                nchunk=[np.ones(M, dtype=np.int64)])

    anc = np.arange(M)                      # chunk -> node id at the current level
    for level in range(1, L):
        below = idx.center[level - 1]
        N = below.shape[0]
        k = max(1, -(-N // level_fanout(F, level)))
        X = np.stack([direction_of(c) for c in below]) if N else np.zeros((0, d))
        if N:
            gaps: list = []
            labels, m = spherical_kmeans(X, k, iters, margins=gaps)
            if gaps:
                idx.min_margin = min(idx.min_margin, min(gaps))
        else:
            labels, m = np.zeros(0, dtype=np.int64), np.tile(unit(np.zeros(d)), (k, 1))
        idx.parent[level - 1] = labels.astype(np.int64)
        anc = labels[anc] if N else anc
        cen = np.zeros((k, d))
        rad = np.full(k, NEG_INF)
        ntok = np.zeros(k, dtype=np.int64)
        nchunk = np.zeros(k, dtype=np.int64)
        for u in range(k):
            desc = np.nonzero(anc == u)[0]
            nchunk[u] = len(desc)
            ntok[u] = int(idx.ntok[0][desc].sum())
            if len(desc) == 0:
                cen[u] = store_f32(m[u])            # empty node: keeps its centroid, never kept
                continue
            if geometry == TOKEN_BALL:
                cen[u] = store_f32(idx.center[0][desc].sum(axis=0) / len(desc))
            else:
                cen[u] = store_f32(m[u])
            diff = idx.center[0][desc] - cen[u][None, :]
            reach = np.sqrt((diff * diff).sum(axis=1)) + idx.radius[0][desc]
            rad[u] = float(round_up_f32(reach.max()))
        idx.center.append(cen)
        idx.radius.append(rad)
        idx.parent.append(np.full(k, -1, dtype=np.int64))
        idx.ntok.append(ntok)
        idx.nchunk.append(nchunk)
    idx.radius_build = [r.copy() for r in idx.radius]
    return idx


def radius_drift(idx: Index, level: int) -> Tuple[float, float, float, int]:
    """How far the lazy update has inflated the radii of `level` (>= 1) since the last (re)build:
    (sum of the radii at build, sum of the radii now, largest growth of one node, nodes counted),
    over the nodes that held chunks at build time (finite radius then).  Radii only grow under the
    lazy update (Section 4.4), so sum now >= sum at build; the paper's limitations paragraph
    proposes re-clustering once they have inflated: a caller re-clusters when
    sum now > (1 + tau) * sum at build."""
    assert idx.radius_build is not None and level >= 1
    base = idx.radius_build[level]
    live = np.isfinite(base)
    now = idx.radius[level][: len(base)]
    if not live.any():
        return 0.0, 0.0, 0.0, 0
    return float(base[live].sum()), float(now[live].sum()), float((now[live] - base[live]).max()), int(live.sum())


# --------------------------------------------------------------------------
# scoring  -- Eq. 2
# --------------------------------------------------------------------------

def upper_bounds(q: np.ndarray, center: np.ndarray, radius: np.ndarray) -> np.ndarray:
    """UB_g(u) = (q_g . mu_u + |q_g| r_u) / sqrt(d) for a query group q [G, d]; returns [G, N]."""
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[1]
    qn = np.sqrt((q * q).sum(axis=1))
    return (q @ center.T + qn[:, None] * radius[None, :]) / math.sqrt(d)


def node_scores(idx: Index, level: int, q: np.ndarray, nodes: Optional[np.ndarray] = None) -> np.ndarray:
    """Group score s(u) = max_g UB_g(u); empty nodes score -inf."""
    if nodes is None:
        nodes = np.arange(idx.n(level))
    nodes = np.asarray(nodes, dtype=np.int64)
    if len(nodes) == 0:
        return np.zeros(0)
    s = np.full(len(nodes), NEG_INF)
    live = idx.nchunk[level][nodes] > 0
    if live.any():
        ub = upper_bounds(q, idx.center[level][nodes[live]], idx.radius[level][nodes[live]])
        s[live] = ub.max(axis=0)
    return s


# --------------------------------------------------------------------------
# selection under a token budget
# --------------------------------------------------------------------------

def order_by_score(ids: np.ndarray, scores: np.ndarray) -> np.ndarray:
    """Positions sorted by (score descending, id ascending)."""
    return np.lexsort((np.asarray(ids), -np.asarray(scores)))


def select_prefix(ids: np.ndarray, scores: np.ndarray, lens: np.ndarray, budget: int,
                  max_count: Optional[int] = None) -> np.ndarray:
    """Longest prefix of the (score desc, id asc) order whose lengths sum to <= budget
    (and, if given, holding at most max_count entries).  Stops at the first entry
    that does not fit.  Returns the chosen ids in ascending order."""
    ids = np.asarray(ids, dtype=np.int64)
    order = order_by_score(ids, scores)
    total = 0
    chosen: List[int] = []
    for pos in order:
        if scores[pos] == NEG_INF:
            break
        if max_count is not None and len(chosen) >= max_count:
            break
        if total + int(lens[pos]) > budget:
            break
        total += int(lens[pos])
        chosen.append(int(ids[pos]))
    return np.array(sorted(chosen), dtype=np.int64)


def pinned_chunks(idx: Index, sink_tokens: int) -> np.ndarray:
    """Leading chunks that cover the first `sink_tokens` tokens: always attended,
    never scored, not charged to the budget (Appendix A sets an attention sink)."""
    if sink_tokens <= 0:
        return np.zeros(0, dtype=np.int64)
    return np.nonzero(idx.bounds[:-1] < sink_tokens)[0]


def _merge_pinned(pinned: np.ndarray, chosen: np.ndarray) -> np.ndarray:
    return np.array(sorted(set(pinned.tolist()) | set(chosen.tolist())), dtype=np.int64)


# --------------------------------------------------------------------------
# retrieval  -- Algorithm 1 steps 1-2, Section 4.4
# --------------------------------------------------------------------------

def retrieve_flat(idx: Index, q: np.ndarray, budget: int, sink_tokens: int = 0,
                  return_scores: bool = False):
    """EXACT policy, by definition: score every chunk, select under the budget."""
    M = idx.M
    pinned = pinned_chunks(idx, sink_tokens)
    cand = np.setdiff1d(np.arange(M), pinned)
    s_all = node_scores(idx, 0, q)
    chosen = select_prefix(cand, s_all[cand], idx.lens()[cand], budget)
    out = _merge_pinned(pinned, chosen)
    return (out, s_all) if return_scores else out


def retrieve_best_first(idx: Index, q: np.ndarray, budget: int, sink_tokens: int = 0) -> np.ndarray:
    """EXACT policy by best-first branch and bound over the tree.

    A max-queue ordered by (score desc, internal nodes before chunks, id asc)
    starts with the top level.  Popping an internal node pushes its children;
    popping a chunk makes it the next chunk of the flat scan's order, because
    every node's score bounds the scores of the chunks beneath it (Eq. 2 with
    covering radii) and, at equal score, internal nodes are opened first so
    that a lower-id chunk hiding beneath one is seen in time.
    Stops at the first chunk that does not fit.
    """
    pinned = set(pinned_chunks(idx, sink_tokens).tolist())
    lens = idx.lens()
    top = idx.L - 1
    heap: List[Tuple[float, int, int]] = []
    s_top = node_scores(idx, top, q)
    for u in range(idx.n(top)):
        if top == 0 and u in pinned:
            continue
        if s_top[u] > NEG_INF:
            heapq.heappush(heap, (-s_top[u], -top, u))
    total = 0
    chosen: List[int] = []
    while heap:
        neg, neg_level, u = heapq.heappop(heap)
        level = -neg_level
        if level == 0:
            if total + int(lens[u]) > budget:
                break
            total += int(lens[u])
            chosen.append(u)
            continue
        kids = idx.children(level, u)
        if level - 1 == 0:
            kids = np.array([j for j in kids if j not in pinned], dtype=np.int64)
        sk = node_scores(idx, level - 1, q, kids)
        for j, sj in zip(kids, sk):
            if sj > NEG_INF:
                heapq.heappush(heap, (-sj, -(level - 1), int(j)))
    return _merge_pinned(np.array(sorted(pinned), dtype=np.int64), np.array(chosen, dtype=np.int64))


def _min_prefix_reaching(ids: np.ndarray, scores: np.ndarray, weights: np.ndarray, target: int) -> np.ndarray:
    """Shortest prefix of the (score desc, id asc) order whose weights sum to >= target
    (everything with a finite score if the total stays below target).  Returns positions."""
    order = order_by_score(ids, scores)
    total = 0
    kept: List[int] = []
    for pos in order:
        if scores[pos] == NEG_INF:
            break
        kept.append(int(pos))
        total += int(weights[pos])
        if total >= target:
            break
    return np.array(kept, dtype=np.int64)


def retrieve_level_sync(idx: Index, q: np.ndarray, budget: int, sink_tokens: int = 0,
                        stats: Optional[Dict] = None) -> np.ndarray:
    """EXACT policy, level by level (the form a GPU can run), two passes.

    All internal nodes are scored once.  Probe: going down, keep at each level
    the best frontier nodes until their subtree token counts reach the budget;
    score the chunks below them; tau0 = the score at which those chunks'
    cumulative length first reaches the budget (-inf if it never does).  At
    least `budget` tokens of chunks score >= tau0, so the flat scan's prefix
    cannot reach below tau0.  Verify: going down from the top keep every node
    scoring >= tau0 (every ancestor of a chunk scoring >= tau0 does, by Eq. 2);
    score the chunks below the kept level-1 nodes and apply the selection rule.
    """
    L = idx.L
    pinned = pinned_chunks(idx, sink_tokens)
    if L == 1:
        if stats is not None:
            stats.update(tau0=NEG_INF, leaves_scored=idx.M, internal_scored=0)
        return retrieve_flat(idx, q, budget, sink_tokens)
    lens = idx.lens()
    s = {l: node_scores(idx, l, q) for l in range(1, L)}
    internal_scored = sum(idx.n(l) for l in range(1, L))

    # probe
    frontier = np.arange(idx.n(L - 1))
    for level in range(L - 1, 0, -1):
        pos = _min_prefix_reaching(frontier, s[level][frontier], idx.ntok[level][frontier], budget)
        kept = frontier[pos]
        below = idx.parent[level - 1]
        frontier = np.nonzero(np.isin(below, kept))[0]
    probe = np.setdiff1d(frontier, pinned)
    sp = node_scores(idx, 0, q, probe)
    pos = _min_prefix_reaching(probe, sp, lens[probe], budget)
    if len(pos) and int(lens[probe[pos]].sum()) >= budget and budget > 0:
        tau0 = float(sp[pos[-1]])
    else:
        tau0 = NEG_INF if budget > 0 else math.inf
    if budget <= 0:
        if stats is not None:
            stats.update(tau0=tau0, leaves_scored=len(probe), internal_scored=internal_scored)
        return _merge_pinned(pinned, np.zeros(0, dtype=np.int64))

    # verify
    kept_mask = s[L - 1] >= tau0
    for level in range(L - 2, 0, -1):
        kept_mask = kept_mask[idx.parent[level]] & (s[level] >= tau0)
    survivors = np.nonzero(kept_mask[idx.parent[0]])[0]
    survivors = np.setdiff1d(survivors, pinned)
    ss = node_scores(idx, 0, q, survivors)
    chosen = select_prefix(survivors, ss, lens[survivors], budget)
    if stats is not None:
        stats.update(tau0=tau0, leaves_scored=len(np.union1d(survivors, probe)),
                     survivors=len(survivors), internal_scored=internal_scored)
    return _merge_pinned(pinned, chosen)


def retrieve_beam(idx: Index, q: np.ndarray, budget: int, beam: Sequence[int],
                  sink_tokens: int = 0, stats: Optional[Dict] = None) -> np.ndarray:
    """BEAM policy: Algorithm 1 generalised to L levels.

    At level l (top first) keep the beam[l] best frontier nodes by (score desc,
    id asc); the next frontier is their children.  At the chunk level the
    selection rule is applied to the best beam[0] frontier chunks.
    beam[l] <= 0 means "no limit".
    """
    L = idx.L
    pinned = pinned_chunks(idx, sink_tokens)
    lens = idx.lens()
    frontier = np.arange(idx.n(L - 1))
    scored = []
    for level in range(L - 1, 0, -1):
        sl = node_scores(idx, level, q, frontier)
        scored.append(len(frontier))
        order = order_by_score(frontier, sl)
        order = order[sl[order] > NEG_INF]
        if beam[level] > 0:
            order = order[:beam[level]]
        kept = frontier[order]
        frontier = np.nonzero(np.isin(idx.parent[level - 1], kept))[0]
    frontier = np.setdiff1d(frontier, pinned)
    s0 = node_scores(idx, 0, q, frontier)
    scored.append(len(frontier))
    chosen = select_prefix(frontier, s0, lens[frontier], budget,
                           max_count=beam[0] if beam[0] > 0 else None)
    if stats is not None:
        stats.update(scored_per_level=scored[::-1])
    return _merge_pinned(pinned, chosen)


# --------------------------------------------------------------------------
# attention  -- Eq. 1 restricted to the active set
# --------------------------------------------------------------------------

def active_tokens(idx_bounds: np.ndarray, T: int, ids: Sequence[int]) -> np.ndarray:
    """Token positions of the listed chunks plus the open tail [bounds[M], T)."""
    b = np.asarray(idx_bounds, dtype=np.int64)
    parts = [np.arange(b[j], b[j + 1]) for j in ids]
    parts.append(np.arange(b[-1], T))
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)


def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, tokens: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Softmax attention of each query row over the given token positions.

    q [G, d]; K, V [>=T, d]; returns (out [G, d], lse [G]).  Logits q.k/sqrt(d),
    softmax with the maximum subtracted.  Empty set: out = 0, lse = -inf.
    """
    q = np.asarray(q, dtype=np.float64)
    G, d = q.shape
    out = np.zeros((G, d))
    lse = np.full(G, NEG_INF)
    if len(tokens) == 0:
        return out, lse
    Ka = np.asarray(K, dtype=np.float64)[tokens]
    Va = np.asarray(V, dtype=np.float64)[tokens]
    for g in range(G):
        x = Ka @ q[g] / math.sqrt(d)
        mx = x.max()
        e = np.exp(x - mx)
        z = e.sum()
        out[g] = (e[:, None] * Va).sum(axis=0) / z
        lse[g] = mx + math.log(z)
    return out, lse


def sparse_decode(q: np.ndarray, K: np.ndarray, V: np.ndarray, bounds: np.ndarray, T: int,
                  ids: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Attention over the listed chunks and the open tail (Algorithm 1 step 3)."""
    return attend(q, K, V, active_tokens(bounds, T, ids))


# --------------------------------------------------------------------------
# lazy update  -- Section 4.4, Algorithm 1 step 4
# --------------------------------------------------------------------------

def append_token(idx: Index) -> None:
    """A new token joins the open tail (its k, v are written to the cache by the caller)."""
    idx.T += 1


def nearest_fine_cluster(idx: Index, c_x: np.ndarray) -> Tuple[int, np.ndarray]:
    """argmax over all level-1 nodes of <unit(c_x), unit(mu_p)>, ties -> lower id."""
    xh = direction_of(c_x)
    sims = np.array([float(xh @ direction_of(mu)) for mu in idx.center[1]])
    return int(np.argmax(sims)), sims


def close_chunk(idx: Index, K: np.ndarray) -> int:
    """Turn the open tail [bounds[M], T) into chunk M and graft it onto the index.

    The new chunk goes under the level-1 node whose direction is nearest to its
    own; that node and its ancestors take a count-weighted moving average of
    the new center, and their radii grow (never shrink): by the distance the
    centroid moved, and enough to cover the new chunk's ball.  Returns the
    level-1 parent (or -1 when the index has a single level).
    """
    K = np.asarray(K, dtype=np.float64)
    lo, hi = int(idx.bounds[-1]), idx.T
    assert hi > lo, "no open tokens to close"
    mu_x, r_x, _ = chunk_node(K[lo:hi], idx.geometry, idx.center_dtype)
    n_x = hi - lo
    p = -1
    if idx.L > 1:
        p, _ = nearest_fine_cluster(idx, mu_x)
        a = p
        for level in range(1, idx.L):
            n_a = int(idx.nchunk[level][a])
            mu_a = idx.center[level][a]
            new = (n_a * mu_a + mu_x) / (n_a + 1)
            if idx.geometry == PAPER_UNIT:
                new = unit(new)
            new = store_f32(new)
            shift = math.sqrt(float(((new - mu_a) ** 2).sum()))
            reach = math.sqrt(float(((mu_x - new) ** 2).sum())) + r_x
            idx.center[level][a] = new
            idx.radius[level][a] = float(round_up_f32(max(idx.radius[level][a] + shift, reach)))
            idx.ntok[level][a] += n_x
            idx.nchunk[level][a] += 1
            a = int(idx.parent[level][a])
    idx.center[0] = np.vstack([idx.center[0], mu_x[None, :]])
    idx.radius[0] = np.append(idx.radius[0], r_x)
    idx.parent[0] = np.append(idx.parent[0], p)
    idx.ntok[0] = np.append(idx.ntok[0], n_x)
    idx.nchunk[0] = np.append(idx.nchunk[0], 1)
    idx.bounds = np.append(idx.bounds, hi)
    return p


# --------------------------------------------------------------------------
# one whole decode step for a (sequence, KV head)
# --------------------------------------------------------------------------

def decode_step(idx: Index, q: np.ndarray, K: np.ndarray, V: np.ndarray, budget: int,
                policy: int = POLICY_EXACT, beam: Optional[Sequence[int]] = None,
                sink_tokens: int = 0):
    """Retrieve, then attend.  If everything fits the budget this is full attention
    (Appendix F.1)."""
    if policy == POLICY_EXACT:
        ids = retrieve_flat(idx, q, budget, sink_tokens)
    else:
        ids = retrieve_beam(idx, q, budget, beam, sink_tokens)
    out, lse = sparse_decode(q, K, V, idx.bounds, idx.T, ids)
    return ids, out, lse
