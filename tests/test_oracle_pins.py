"""Pins for the CPU oracle: closed forms, brute force, library routines, the hand example.

Each test ties one part of oracle/lychee_oracle.py to something other than
itself, chosen so that a plausible slip (dropped term, wrong sign, transposed
operand, off-by-one in the prefix rule) makes at least one of them fail.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import lychee_oracle as orc
from tests import helpers as H

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


# ---------------------------------------------------------------- hand example

def _hand():
    g = json.load(open(GOLDEN))
    d = g["d"]
    K = np.zeros((13, d))
    K[:, :2] = np.array(g["keys_xy"], dtype=np.float64)
    V = np.zeros((13, d))
    V[:, 0] = np.arange(13)
    V[:, 1] = 1.0
    q = np.zeros((1, d))
    q[0, :2] = g["q_xy"]
    idx = orc.build_index(K, g["bounds"], 13, g["levels"], g["fanout"])
    return g, K, V, q, idx


def test_hand_example_index():
    g, K, V, q, idx = _hand()
    assert np.allclose(idx.center[0][:, :2], g["chunk_centers_xy"], atol=0)
    assert np.allclose(idx.radius[0], g["chunk_radii"], rtol=1e-6)
    assert idx.parent[0].tolist() == g["parents"]
    assert np.allclose(idx.center[1][:, :2], g["cluster_centers_xy"], atol=0)
    assert np.allclose(idx.radius[1], g["cluster_radii"], rtol=1e-6)
    assert idx.ntok[1].tolist() == g["cluster_ntok"]


def test_hand_example_scores_and_selection():
    g, K, V, q, idx = _hand()
    assert np.allclose(orc.node_scores(idx, 0, q), g["chunk_scores"], rtol=1e-6)
    assert np.allclose(orc.node_scores(idx, 1, q), g["cluster_scores"], rtol=1e-6)
    for bud, want in g["exact"].items():
        for fn in (orc.retrieve_flat, orc.retrieve_best_first, orc.retrieve_level_sync):
            assert fn(idx, q, int(bud)).tolist() == want, (fn.__name__, bud)
    assert orc.retrieve_beam(idx, q, 7, [0, 1]).tolist() == g["beam_top1_budget7"]
    assert orc.retrieve_beam(idx, q, 7, [0, 2]).tolist() == g["beam_top2_budget7"]


def test_hand_example_attention():
    g, K, V, q, idx = _hand()
    out, lse = orc.sparse_decode(q, K, V, idx.bounds, idx.T, g["attn_ids"])
    assert np.allclose(out[0], g["attn_out"], rtol=1e-12, atol=1e-12)
    assert abs(lse[0] - g["attn_lse"]) < 1e-12


# ---------------------------------------------------------------- Eq. 2: the bound

@pytest.mark.parametrize("seed,d,L,F", [(1, 4, 2, 3), (2, 8, 3, 3), (3, 128, 3, 4), (4, 16, 4, 2)])
def test_bound_never_underestimates(seed, d, L, F):
    """Brute force: at every level a node's score bounds the logit of every token below it."""
    c = H.rand_case(seed, T=160, d=d, G=3)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], L, F)
    H.check_covering_invariant(idx, c["K"])
    H.check_counts(idx)
    r = np.random.default_rng(seed + 100)
    for _ in range(5):
        q = r.standard_normal((3, d)) * r.uniform(0.1, 3.0)
        true_max = np.array([(c["K"][idx.bounds[j]:idx.bounds[j + 1]] @ q.T).max() / math.sqrt(d)
                             for j in range(idx.M)])
        for level in range(L):
            s = orc.node_scores(idx, level, q)
            anc = idx.ancestor(level)
            assert np.all(s[anc] >= true_max - 1e-9), level
            # every ancestor bounds the *chunk* scores beneath it (what pruning relies
            # on); an internal child's own ball may stick out of its parent's, so
            # nothing is claimed between two internal levels.
            s_chunk = orc.node_scores(idx, 0, q)
            assert np.all(s[anc] >= s_chunk - 1e-9), level


def test_bound_is_tight_closed_form():
    """One chunk, q along (k_far - mu): the bound equals q.k_far exactly (Cauchy-Schwarz equality)."""
    d = 4
    K = np.array([[1.0, 0, 0, 0], [3.0, 0, 0, 0], [2.0, 1.0, 0, 0], [2.0, -1.0, 0, 0], [2.0, 0, 0, 0.5]])
    idx = orc.build_index(K, [0, 5], 5, 1, 4)
    mu = idx.center[0][0]
    assert np.allclose(mu, [2.0, 0, 0, 0.1])
    dist = np.sqrt(((K - mu) ** 2).sum(axis=1))
    far = int(np.argmax(dist))
    q = (K[far] - mu)[None, :] * 1.7
    s = orc.node_scores(idx, 0, q)[0]
    assert abs(s - float(q[0] @ K[far]) / 2.0) < 1e-6
    # opposite direction: bound is loose by exactly 2 |q| r / sqrt(d) relative to q.mu - |q| r
    s2 = orc.node_scores(idx, 0, -q)[0]
    assert abs(s2 - (float(-q[0] @ mu) + np.linalg.norm(q) * dist[far]) / 2.0) < 1e-6


def test_identical_keys_zero_radius_score_is_true_score():
    d = 8
    k = np.arange(1, d + 1, dtype=np.float64) / 4
    K = np.tile(k, (6, 1))
    idx = orc.build_index(K, [0, 2, 6], 6, 2, 2)
    assert np.all(idx.radius[0] == 0.0) and idx.radius[1][0] == 0.0
    q = np.array([[0.5, -1, 2, 0, 0, 1, 1, -2.0], [1, 1, 1, 1, 0, 0, 0, 0.0]])
    want = max(float(q[0] @ k), float(q[1] @ k)) / math.sqrt(d)
    assert np.allclose(orc.node_scores(idx, 0, q), want)
    assert np.allclose(orc.node_scores(idx, 1, q), want)


def test_group_score_is_max_over_heads():
    c = H.rand_case(7, T=80, d=8, G=4)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 2, 4)
    per_head = np.stack([orc.node_scores(idx, 0, c["q"][g:g + 1]) for g in range(4)])
    assert np.array_equal(orc.node_scores(idx, 0, c["q"]), per_head.max(axis=0))


def test_chunk_node_symmetric_pair():
    """Keys at +-a e_1 (+ common b): center b, radius a."""
    b = np.array([0.5, -1.0, 2.0, 0.25])
    a = 3.0
    K = np.stack([b + a * np.eye(4)[1], b - a * np.eye(4)[1]])
    mu, r, _ = orc.chunk_node(K, orc.TOKEN_BALL)
    assert np.array_equal(mu, b) and r == a
    mu_u, r_u, _ = orc.chunk_node(K, orc.PAPER_UNIT)
    assert abs(np.linalg.norm(mu_u) - 1) < 1e-6 and r_u == 0.0
    assert np.allclose(mu_u, b / np.linalg.norm(b), atol=1e-7)


def test_round_up_f32():
    x = np.array([1.0, 1.0 + 1e-12, 0.1, 3.0000001, 1e-30])
    y = orc.round_up_f32(x)
    assert np.all(y >= x)
    assert np.all(y.astype(np.float32).astype(np.float64) == y)
    assert y[0] == 1.0 and y[1] == float(np.nextafter(np.float32(1), np.float32(2)))


# ---------------------------------------------------------------- selection rule

def _brute_prefix(ids, scores, lens, budget):
    order = sorted(range(len(ids)), key=lambda p: (-scores[p], ids[p]))
    best = []
    for m in range(len(order) + 1):
        if sum(lens[p] for p in order[:m]) <= budget:
            best = order[:m]
        else:
            break
    return sorted(ids[p] for p in best)


@pytest.mark.parametrize("seed", range(8))
def test_select_prefix_brute_force(seed):
    r = np.random.default_rng(seed)
    n = int(r.integers(1, 12))
    ids = np.sort(r.choice(40, size=n, replace=False))
    scores = np.round(r.standard_normal(n), 1)          # ties on purpose
    lens = r.integers(1, 9, size=n)
    for budget in (0, 1, 5, 13, 1000):
        got = orc.select_prefix(ids, scores, lens, budget).tolist()
        assert got == _brute_prefix(ids.tolist(), scores.tolist(), lens.tolist(), budget)


def test_select_equal_lengths_is_topk():
    r = np.random.default_rng(5)
    n, ell = 50, 7
    scores = r.standard_normal(n)
    for budget in (0, 6, 7, 20, 21, 349, 350, 10 ** 6):
        k = min(n, budget // ell)
        want = np.sort(np.argsort(-scores, kind="stable")[:k])
        got = orc.select_prefix(np.arange(n), scores, np.full(n, ell), budget)
        assert np.array_equal(got, want)


def test_select_ties_prefer_lower_id_and_zero_query():
    c = H.rand_case(11, T=120, d=8, G=2)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 3, 3)
    q0 = np.zeros((2, 8))
    lens = idx.lens()
    budget = int(lens[:4].sum()) + 1
    want = []
    tot = 0
    for j in range(idx.M):
        if tot + lens[j] > budget:
            break
        tot += lens[j]
        want.append(j)
    for fn in (orc.retrieve_flat, orc.retrieve_best_first):
        assert fn(idx, q0, budget).tolist() == want
    # level-sync: with q = 0 all scores are 0 (empty nodes aside), same answer
    assert orc.retrieve_level_sync(idx, q0, budget).tolist() == want


# ---------------------------------------------------------------- EXACT retrieval == flat scan

@pytest.mark.parametrize("seed", range(12))
def test_hierarchical_equals_flat(seed):
    r = np.random.default_rng(seed)
    d = int(r.choice([4, 8, 16]))
    L = int(r.integers(1, 5))
    F = int(r.integers(2, 6))
    tight = seed % 2 == 0        # tight clusters => pruning really happens
    c = H.rand_case(seed, T=int(r.integers(60, 400)), d=d, G=int(r.integers(1, 5)),
                    offset_std=3.0 if tight else 0.5, noise_std=0.05 if tight else 1.0,
                    tail=int(r.integers(0, 5)))
    idx = orc.build_index(c["K"], c["bounds"], c["T"], L, F)
    H.check_covering_invariant(idx, c["K"])
    for budget in (0, 1, 17, 64, c["T"] // 3, c["T"], c["T"] + 50):
        for sink in (0, 5):
            flat = orc.retrieve_flat(idx, c["q"], budget, sink).tolist()
            assert orc.retrieve_best_first(idx, c["q"], budget, sink).tolist() == flat
            st = {}
            assert orc.retrieve_level_sync(idx, c["q"], budget, sink, st).tolist() == flat
            nolimit = orc.retrieve_beam(idx, c["q"], budget, [0] * L, sink).tolist()
            assert nolimit == flat
            big = orc.retrieve_beam(idx, c["q"], budget, [10 ** 6] * L, sink).tolist()
            assert big == flat


def test_level_sync_really_prunes_on_tight_clusters():
    """Chunks drawn from a few far-apart topics: whole subtrees fall below tau0."""
    r = np.random.default_rng(21)
    d, n_topics, M, ell = 8, 16, 128, 5
    topics = 6.0 * r.standard_normal((n_topics, d))
    topic_of = r.integers(0, n_topics, size=M)
    K = np.repeat(topics[topic_of], ell, axis=0) + 0.01 * r.standard_normal((M * ell, d))
    bounds = np.arange(M + 1) * ell
    idx = orc.build_index(K, bounds, M * ell, 3, 4)
    q = topics[3][None, :]
    st = {}
    ids = orc.retrieve_level_sync(idx, q, 20, 0, st)
    assert ids.tolist() == orc.retrieve_flat(idx, q, 20).tolist()
    assert set(topic_of[ids]) == {3}
    assert st["leaves_scored"] < idx.M // 2, st


def test_budget_edges():
    c = H.rand_case(31, T=150, d=8, G=2, tail=3)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 3, 4)
    for fn in (orc.retrieve_flat, orc.retrieve_best_first, orc.retrieve_level_sync):
        assert fn(idx, c["q"], 0).tolist() == []
        assert fn(idx, c["q"], int(idx.bounds[-1])).tolist() == list(range(idx.M))
        assert fn(idx, c["q"], 0, 9).tolist() == orc.pinned_chunks(idx, 9).tolist()
    assert orc.pinned_chunks(idx, 1).tolist() == [0]
    b1 = int(idx.bounds[1])
    assert orc.pinned_chunks(idx, b1).tolist() == [0]
    assert orc.pinned_chunks(idx, b1 + 1).tolist() == [0, 1]


def test_beam_binding_differs_and_is_subset_of_frontier():
    c = H.rand_case(41, T=400, d=8, G=2)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 3, 4)
    st = {}
    ids = orc.retrieve_beam(idx, c["q"], 60, [0, 2, 1], 0, st)
    # frontier: children of the best top node, then the best 2 of those
    s2 = orc.node_scores(idx, 2, c["q"])
    top = min(np.nonzero(s2 == s2.max())[0])
    kids = idx.children(2, top)
    s1 = orc.node_scores(idx, 1, c["q"], kids)
    keep = kids[np.lexsort((kids, -s1))[:2]]
    frontier = np.nonzero(np.isin(idx.parent[0], keep))[0]
    assert set(ids.tolist()) <= set(frontier.tolist())
    s0 = orc.node_scores(idx, 0, c["q"])
    assert ids.tolist() == orc.select_prefix(frontier, s0[frontier], idx.lens()[frontier], 60).tolist()
    assert st["scored_per_level"] == [len(frontier), len(kids), idx.n(2)]
    # leaf beam: at most beam[0] chunks
    ids1 = orc.retrieve_beam(idx, c["q"], 10 ** 6, [3, 0, 0])
    assert len(ids1) == 3
    assert set(ids1.tolist()) == set(np.lexsort((np.arange(idx.M), -s0))[:3].tolist())


# ---------------------------------------------------------------- attention

@pytest.mark.parametrize("seed", range(4))
def test_full_budget_equals_dense_attention(seed):
    """Budget covering the whole context: sparse decode == textbook dense attention."""
    c = H.rand_case(50 + seed, T=300, d=16, G=4, tail=seed)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 3, 4)
    ids, out, lse = orc.decode_step(idx, c["q"], c["K"], c["V"], budget=c["T"])
    assert ids.tolist() == list(range(idx.M))
    ref_out, ref_lse = H.dense_attention_library(c["q"], c["K"][:c["T"]], c["V"][:c["T"]])
    assert np.allclose(out, ref_out, rtol=1e-12, atol=1e-13)
    assert np.allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)


def test_sparse_subset_equals_library_on_gathered_rows():
    c = H.rand_case(60, T=200, d=8, G=2, tail=4)
    ids = [1, 4, 5]
    out, lse = orc.sparse_decode(c["q"], c["K"], c["V"], c["bounds"], c["T"], ids)
    rows = np.concatenate([np.arange(c["bounds"][j], c["bounds"][j + 1]) for j in ids]
                          + [np.arange(c["bounds"][-1], c["T"])])
    ref_out, ref_lse = H.dense_attention_library(c["q"], c["K"][rows], c["V"][rows])
    assert np.allclose(out, ref_out, rtol=1e-12) and np.allclose(lse, ref_lse, rtol=1e-12)


def test_attention_special_cases():
    r = np.random.default_rng(3)
    d = 8
    q = r.standard_normal((2, d))
    V = r.standard_normal((10, d))
    K_same = np.tile(r.standard_normal(d), (10, 1))
    out, lse = orc.attend(q, K_same, V, np.arange(10))
    assert np.allclose(out, V.mean(axis=0)[None, :])                 # equal logits: plain mean of V
    assert np.allclose(lse, K_same[0] @ q.T / math.sqrt(d) + math.log(10))
    K = r.standard_normal((10, d))
    out, lse = orc.attend(q, K, V, np.array([7]))
    assert np.allclose(out, V[7][None, :]) and np.allclose(lse, K[7] @ q.T / math.sqrt(d))
    out, lse = orc.attend(q, K, V, np.zeros(0, dtype=np.int64))
    assert np.all(out == 0) and np.all(lse == -math.inf)
    # huge logits do not overflow (max-subtracted)
    out, _ = orc.attend(q * 1e4, K, V, np.arange(10))
    assert np.all(np.isfinite(out))


def test_open_tail_is_always_attended():
    c = H.rand_case(70, T=100, d=8, G=1, tail=6)
    out, _ = orc.sparse_decode(c["q"], c["K"], c["V"], c["bounds"], c["T"], [])
    rows = np.arange(c["bounds"][-1], c["T"])
    ref, _ = H.dense_attention_library(c["q"], c["K"][rows], c["V"][rows])
    assert len(rows) == 6 and np.allclose(out, ref)


# ---------------------------------------------------------------- spherical k-means

def test_kmeans_objective_monotone_and_unit_centroids():
    r = np.random.default_rng(8)
    X = orc.unit_rows(r.standard_normal((120, 6)) + np.repeat(3 * r.standard_normal((6, 6)), 20, axis=0))
    tr = []
    labels, m = orc.spherical_kmeans(X, 7, 10, trace=tr)
    assert len(tr) == 10
    assert all(b >= a - 1e-12 for a, b in zip(tr, tr[1:])), tr
    assert np.allclose(np.linalg.norm(m, axis=1), 1.0)
    assert labels.min() >= 0 and labels.max() < 7


@pytest.mark.parametrize("seed,N,d,k", [(0, 60, 8, 5), (1, 200, 128, 13), (2, 33, 16, 33), (3, 500, 32, 32)])
def test_kmeans_equals_library_nearest_codeword_iterations(seed, N, d, k):
    """On the unit sphere |x - m|^2 = 2 - 2<x, m>, so the assignment step is the nearest-codeword
    search of a vector-quantisation library (Euclidean) and of a cosine-distance argmin; iterating
    those with a normalised-sum update from the same strided start must reproduce the labels and
    centroids (generic data: no exact ties, no empty clusters by construction of the check)."""
    from scipy.cluster.vq import vq
    from sklearn.metrics import pairwise_distances_argmin
    r = np.random.default_rng(100 + seed)
    n_src = max(2, k // 2)
    X = orc.unit_rows(r.standard_normal((N, d)) + 2.0 * r.standard_normal((n_src, d))[r.integers(0, n_src, size=N)])
    m = np.stack([X[(c * N) // k] for c in range(k)])
    for _ in range(10):
        lab = vq(X, m)[0]
        assert np.array_equal(lab, pairwise_distances_argmin(X, m, metric="cosine"))
        sums = np.zeros_like(m)
        np.add.at(sums, lab, X)
        hit = np.linalg.norm(sums, axis=1) > 0
        m = np.where(hit[:, None], sums / np.maximum(np.linalg.norm(sums, axis=1), 1e-300)[:, None], m)
    labels, cent = orc.spherical_kmeans(X, k, 10)
    assert np.array_equal(labels, lab)
    assert np.allclose(cent, m, rtol=0, atol=1e-12)


def test_kmeans_k_equals_n_and_separated_clusters():
    r = np.random.default_rng(9)
    X = orc.unit_rows(r.standard_normal((9, 5)))
    labels, m = orc.spherical_kmeans(X, 9, 10)
    assert labels.tolist() == list(range(9)) and np.allclose(m, X)
    # two well separated direction bundles, interleaved so the strided init sees both
    a, b = np.eye(5)[0], np.eye(5)[3]
    pts = []
    for i in range(20):
        base = a if i % 2 == 0 else b
        pts.append(base + 0.05 * r.standard_normal(5))
    X = orc.unit_rows(np.array(pts))
    labels, m = orc.spherical_kmeans(X, 2, 10)
    assert len(set(labels[0::2])) == 1 and len(set(labels[1::2])) == 1 and labels[0] != labels[1]
    assert abs(m[labels[0]] @ a) > 0.99 and abs(m[labels[1]] @ b) > 0.99


def test_kmeans_ties_go_to_lower_id_and_empty_cluster_keeps_centroid():
    e = np.eye(4)
    X = np.stack([e[0], e[0], e[1], e[1], -e[0], -e[1]])
    # k = 3: init = points 0, 2, 4 -> e0, e1, -e0.  Point 5 (-e1) ties between clusters 0 and 2 (both 0).
    labels, m = orc.spherical_kmeans(X, 3, 1)
    assert labels.tolist() == [0, 0, 1, 1, 2, 0]
    # duplicates: init picks the same point twice -> the higher-id twin stays empty
    X = np.stack([e[0], e[0], e[0], e[2]])
    labels, m = orc.spherical_kmeans(X, 4, 3)
    assert labels.tolist() == [0, 0, 0, 3]
    assert np.array_equal(m[1], e[0]) and np.array_equal(m[2], e[0])


def test_build_with_empty_cluster_is_consistent():
    e = np.eye(4)
    K = np.concatenate([np.tile(e[0], (6, 1)), np.tile(e[2], (2, 1))])
    idx = orc.build_index(K, [0, 2, 4, 6, 8], 8, 2, 1)          # F = 1 -> k = 4, clusters 1, 2 empty
    assert idx.nchunk[1].tolist() == [3, 0, 0, 1]
    assert idx.radius[1][1] == -math.inf and idx.ntok[1].tolist() == [6, 0, 0, 2]
    q = np.array([[1.0, 0, 0, 0]])
    assert orc.node_scores(idx, 1, q)[1] == -math.inf
    assert orc.node_scores(idx, 1, np.zeros((1, 4)))[1] == -math.inf   # not NaN from 0 * inf
    for bud in (0, 2, 5, 8):
        flat = orc.retrieve_flat(idx, q, bud).tolist()
        assert orc.retrieve_best_first(idx, q, bud).tolist() == flat
        assert orc.retrieve_level_sync(idx, q, bud).tolist() == flat


def test_internal_center_is_mean_of_descendant_chunk_centers():
    c = H.rand_case(81, T=300, d=8, G=1)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 4, 3)
    for level in range(1, 4):
        anc = idx.ancestor(level)
        for u in range(idx.n(level)):
            desc = np.nonzero(anc == u)[0]
            if len(desc):
                assert np.allclose(idx.center[level][u], idx.center[0][desc].mean(axis=0), rtol=1e-6, atol=1e-7)
    assert [idx.n(l) for l in range(4)] == [idx.M, -(-idx.M // 3), -(-(-(-idx.M // 3)) // 3),
                                            -(-(-(-(-(-idx.M // 3)) // 3)) // 3)]


def test_paper_unit_geometry():
    c = H.rand_case(82, T=200, d=8, G=2)
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 3, 3, geometry=orc.PAPER_UNIT)
    for level in range(3):
        live = idx.nchunk[level] > 0
        assert np.allclose(np.linalg.norm(idx.center[level][live], axis=1), 1.0, atol=1e-6)
    assert np.all(idx.radius[0] == 0)
    H.check_covering_invariant(idx, c["K"])
    # chunk score is the literal representative-key score q . kbar / sqrt(d)
    kbar = np.stack([orc.unit(c["K"][idx.bounds[j]:idx.bounds[j + 1]].mean(axis=0)) for j in range(idx.M)])
    want = (c["q"] @ kbar.T).max(axis=0) / math.sqrt(8)
    assert np.allclose(orc.node_scores(idx, 0, c["q"]), want, atol=1e-6)
    flat = orc.retrieve_flat(idx, c["q"], 50).tolist()
    assert orc.retrieve_best_first(idx, c["q"], 50).tolist() == flat
    assert orc.retrieve_level_sync(idx, c["q"], 50).tolist() == flat


# ---------------------------------------------------------------- lazy update

@pytest.mark.parametrize("geometry", [orc.TOKEN_BALL, orc.PAPER_UNIT])
@pytest.mark.parametrize("L", [1, 2, 3])
def test_append_keeps_invariants(geometry, L):
    r = np.random.default_rng(90 + L)
    c = H.rand_case(90 + L, T=120, d=8, G=2, tail=2)
    extra = 80
    K = np.vstack([c["K"], r.standard_normal((extra, 8)) + 0.02 * np.cumsum(r.standard_normal((extra, 8)), axis=0)])
    import lc_workloads as wl
    K = wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(K.astype(np.float32)))
    idx = orc.build_index(K, c["bounds"], c["T"], L, 3, geometry=geometry)
    for level in range(1, L):                               # nothing has drifted right after a build
        sb, sn, mg, n = orc.radius_drift(idx, level)
        assert sb == sn and mg == 0.0 and n == int(np.isfinite(idx.radius[level]).sum())
    prev_r = [x.copy() for x in idx.radius]
    open_len = idx.T - int(idx.bounds[-1])
    for step in range(extra):
        orc.append_token(idx)
        open_len += 1
        if open_len >= 3 and r.random() < 0.3:
            M0 = idx.M
            p = orc.close_chunk(idx, K)
            open_len = 0
            assert idx.M == M0 + 1 and int(idx.bounds[-1]) == idx.T
            H.check_covering_invariant(idx, K)
            H.check_counts(idx)
            for level in range(1, L):                       # radii never shrink
                assert np.all(idx.radius[level] >= prev_r[level])
                # ... so the drift figures are the plain differences to the radii at build
                sb, sn, mg, n = orc.radius_drift(idx, level)
                live = np.isfinite(idx.radius_build[level])
                assert sn >= sb and mg >= 0.0
                assert mg == pytest.approx(float((idx.radius[level][live] - idx.radius_build[level][live]).max()))
            prev_r = [x.copy() for x in idx.radius]
            if L > 1:
                # moving average == batch mean of descendant chunk centers (TOKEN_BALL)
                assert idx.parent[0][-1] == p
                if geometry == orc.TOKEN_BALL:
                    desc = np.nonzero(idx.parent[0] == p)[0]
                    assert np.allclose(idx.center[1][p], idx.center[0][desc].mean(axis=0), rtol=1e-5, atol=1e-6)
                # the chosen parent is the nearest by direction
                xh = orc.unit(idx.center[0][-1])
                # (centers moved after the choice; recheck against a fresh argmax is not meaningful)
            # retrieval stays exact after grafting
            flat = orc.retrieve_flat(idx, c["q"], 60).tolist()
            assert orc.retrieve_best_first(idx, c["q"], 60).tolist() == flat
            assert orc.retrieve_level_sync(idx, c["q"], 60).tolist() == flat


def test_append_picks_nearest_direction_and_first_on_tie():
    e = np.eye(4)
    K = np.concatenate([np.tile(e[0], (4, 1)), np.tile(e[1], (4, 1)), np.tile(2 * e[1] + 0.0, (2, 1))])
    idx = orc.build_index(K, [0, 2, 4, 6, 8], 8, 2, 2)         # clusters {0,1} along e0, {2,3} along e1
    assert idx.parent[0].tolist() == [0, 0, 1, 1]
    idx.T = 10
    p = orc.close_chunk(idx, K)                                 # new chunk along e1
    assert p == 1 and idx.nchunk[1].tolist() == [2, 3] and idx.ntok[1].tolist() == [4, 6]
    assert np.allclose(idx.center[1][1], (e[1] + e[1] + 2 * e[1]) / 3, atol=1e-7)
    # radius: max(old + shift, |mu_x - mu'| + r_x) = max(0 + 1/3, 2/3 + 0)
    assert abs(idx.radius[1][1] - 2 / 3) < 1e-6
    # drift since the build: both clusters had radius 0; cluster 1 grew to 2/3, cluster 0 did not move
    assert orc.radius_drift(idx, 1) == pytest.approx((0.0, 2 / 3, 2 / 3, 2), abs=1e-6)
    # a chunk equidistant (in direction) from both clusters goes to the lower id
    K2 = np.vstack([K, np.tile(e[2], (2, 1))])
    idx.T = 12
    assert orc.close_chunk(idx, K2) == 0


def test_append_into_empty_cluster():
    e = np.eye(4)
    K = np.concatenate([np.tile(e[0], (6, 1)), np.tile(e[2], (2, 1)), np.tile(e[0], (2, 1))])
    idx = orc.build_index(K, [0, 2, 4, 6, 8], 8, 2, 1)
    assert idx.nchunk[1].tolist() == [3, 0, 0, 1]
    idx.T = 10
    p = orc.close_chunk(idx, K)             # direction e0: clusters 0,1,2 all have centroid e0 -> id 0
    assert p == 0
    H.check_covering_invariant(idx, K)
    H.check_counts(idx)


# ---------------------------------------------------------------- bfloat16 chunk centers

def test_store_bf16_is_round_to_nearest_even_with_8_significant_bits():
    import torch
    # exact cases: ties go to the even neighbour, everything else to the nearer one
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -(1.0 + 2.0 ** -8),
                  0.0, 255.5, 256.5 * 2.0 ** 10, 0.1])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -1.0,
                     0.0, 256.0, 256.0 * 2.0 ** 10, 0.10009765625])
    assert np.array_equal(orc.store_bf16(x), want)
    # a library conversion of float32 inputs (no second rounding on the way) agrees bit for bit
    r = np.random.default_rng(3)
    f = (r.standard_normal(200000) * np.exp(r.uniform(-30, 30, 200000))).astype(np.float32)
    lib = torch.from_numpy(f).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.store_bf16(f.astype(np.float64)), lib)
    # stored values are fixed points, and the error is at most half a unit in the 8th bit
    assert np.array_equal(orc.store_bf16(lib), lib)
    assert np.all(np.abs(lib - f.astype(np.float64)) <= np.abs(f.astype(np.float64)) * 2.0 ** -8)


@pytest.mark.parametrize("geometry", [orc.TOKEN_BALL, orc.PAPER_UNIT])
def test_bf16_chunk_centers_keep_the_index_sound(geometry):
    """With chunk centers rounded to bfloat16 the radii are measured from the rounded centers, so the
    covering invariant, the bound and the equality of hierarchical and flat retrieval all still hold;
    the stored chunk centers are bfloat16 values next to the float32-mode ones."""
    c = H.rand_case(21, T=260, d=16, G=3)
    a = orc.build_index(c["K"], c["bounds"], c["T"], 3, 3, geometry=geometry)
    b = orc.build_index(c["K"], c["bounds"], c["T"], 3, 3, geometry=geometry, center_dtype=orc.CENTER_BF16)
    assert b.center_dtype == orc.CENTER_BF16
    assert np.array_equal(orc.store_bf16(b.center[0]), b.center[0])
    assert np.array_equal(b.center[0], orc.store_bf16(a.center[0])) or \
        np.max(np.abs(b.center[0] - a.center[0])) <= 2.0 ** -8 * np.max(np.abs(a.center[0]))
    assert not np.array_equal(a.center[0], b.center[0])
    H.check_covering_invariant(b, c["K"])
    H.check_counts(b)
    if geometry == orc.TOKEN_BALL:
        # radii grow by no more than the rounding moved the centers
        shift = np.sqrt(((a.center[0] - b.center[0]) ** 2).sum(axis=1))
        assert np.all(b.radius[0] <= a.radius[0] + shift + 1e-6) and np.all(b.radius[0] >= a.radius[0] - shift - 1e-6)
        true_max = np.array([(c["K"][b.bounds[j]:b.bounds[j + 1]] @ c["q"].T).max() / math.sqrt(16)
                             for j in range(b.M)])
        assert np.all(orc.node_scores(b, 0, c["q"]) >= true_max - 1e-9)
    for budget in (0, 17, 60, 150, 10 ** 6):
        flat = orc.retrieve_flat(b, c["q"], budget).tolist()
        assert orc.retrieve_best_first(b, c["q"], budget).tolist() == flat
        assert orc.retrieve_level_sync(b, c["q"], budget).tolist() == flat


def test_bf16_chunk_centers_survive_appends():
    import lc_workloads as wl
    r = np.random.default_rng(33)
    c = H.rand_case(33, T=150, d=8, G=2, tail=3)
    K = np.vstack([c["K"], r.standard_normal((60, 8))])
    K = wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(K.astype(np.float32)))
    idx = orc.build_index(K, c["bounds"], c["T"], 3, 3, center_dtype=orc.CENTER_BF16)
    open_len = idx.T - int(idx.bounds[-1])
    closed = 0
    for _ in range(60):
        orc.append_token(idx)
        open_len += 1
        if open_len >= 4 and r.random() < 0.4:
            orc.close_chunk(idx, K)
            open_len = 0
            closed += 1
            assert np.array_equal(orc.store_bf16(idx.center[0][-1]), idx.center[0][-1])
            H.check_covering_invariant(idx, K)
            H.check_counts(idx)
    assert closed >= 5
    flat = orc.retrieve_flat(idx, c["q"], 70).tolist()
    assert orc.retrieve_best_first(idx, c["q"], 70).tolist() == flat


# ---------------------------------------------------------------- per-level fan-outs

def test_per_level_fanouts_give_the_papers_tiers():
    """Fan-outs of their own per level (2 chunks per fine cluster, then 8 fine clusters per coarse
    unit here): level sizes are ceil(N / F_level), and everything that holds for one fan-out holds."""
    c = H.rand_case(55, T=400, d=8, G=2)
    F = [0, 2, 8]
    idx = orc.build_index(c["K"], c["bounds"], c["T"], 3, F)
    M = idx.M
    assert idx.n(1) == -(-M // 2) and idx.n(2) == -(-idx.n(1) // 8)
    same = orc.build_index(c["K"], c["bounds"], c["T"], 3, 2)
    assert np.array_equal(idx.parent[0], same.parent[0]) and np.array_equal(idx.center[1], same.center[1])
    assert same.n(2) == -(-same.n(1) // 2) and idx.n(2) < same.n(2)
    H.check_covering_invariant(idx, c["K"])
    H.check_counts(idx)
    for budget in (0, 30, 120, 10 ** 6):
        flat = orc.retrieve_flat(idx, c["q"], budget).tolist()
        assert orc.retrieve_best_first(idx, c["q"], budget).tolist() == flat
        assert orc.retrieve_level_sync(idx, c["q"], budget).tolist() == flat
    beam = [0, 6, 2]
    got = orc.retrieve_beam(idx, c["q"], 10 ** 6, beam)
    assert len(set(idx.parent[0][got].tolist())) <= 6
