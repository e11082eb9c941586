"""Do the pins bite?  Plant plausible mistakes in the oracle (on the CPU) and check
that at least one pin fails for each."""
import math

import numpy as np
import pytest

from oracle import lychee_oracle as orc
from tests import test_oracle_pins as P


def _fails(fn, *a, **kw):
    try:
        fn(*a, **kw)
    except AssertionError:
        return True
    return False


def test_dropped_radius_term_is_caught(monkeypatch):
    def bad(q, center, radius):
        return (np.asarray(q) @ center.T) / math.sqrt(q.shape[1])
    monkeypatch.setattr(orc, "upper_bounds", bad)
    assert _fails(P.test_bound_never_underestimates, 1, 4, 2, 3)
    assert _fails(P.test_hand_example_scores_and_selection)


def test_wrong_radius_sign_is_caught(monkeypatch):
    def bad(q, center, radius):
        qn = np.sqrt((q * q).sum(axis=1))
        return (q @ center.T - qn[:, None] * radius[None, :]) / math.sqrt(q.shape[1])
    monkeypatch.setattr(orc, "upper_bounds", bad)
    assert _fails(P.test_bound_is_tight_closed_form)


def test_missing_sqrt_d_is_caught(monkeypatch):
    def bad(q, center, radius):
        qn = np.sqrt((q * q).sum(axis=1))
        return q @ center.T + qn[:, None] * radius[None, :]
    monkeypatch.setattr(orc, "upper_bounds", bad)
    assert _fails(P.test_hand_example_scores_and_selection)


def test_skipping_instead_of_stopping_is_caught(monkeypatch):
    def bad(ids, scores, lens, budget, max_count=None):
        order = orc.order_by_score(ids, scores)
        total, chosen = 0, []
        for pos in order:
            if total + int(lens[pos]) > budget:
                continue                      # wrong: skips and carries on
            total += int(lens[pos])
            chosen.append(int(ids[pos]))
        return np.array(sorted(chosen), dtype=np.int64)
    monkeypatch.setattr(orc, "select_prefix", bad)
    assert _fails(P.test_hand_example_scores_and_selection)
    assert _fails(P.test_select_prefix_brute_force, 3) or _fails(P.test_select_prefix_brute_force, 1)


def test_wrong_tie_break_is_caught(monkeypatch):
    monkeypatch.setattr(orc, "order_by_score",
                        lambda ids, scores: np.lexsort((-np.asarray(ids), -np.asarray(scores))))
    assert _fails(P.test_select_ties_prefer_lower_id_and_zero_query)


def test_attention_without_scaling_is_caught(monkeypatch):
    real = orc.attend

    def bad(q, K, V, tokens):
        return real(np.asarray(q) * math.sqrt(q.shape[1]), K, V, tokens)
    monkeypatch.setattr(orc, "attend", bad)
    assert _fails(P.test_hand_example_attention)
    assert _fails(P.test_full_budget_equals_dense_attention, 0)


def test_append_without_shift_term_is_caught(monkeypatch):
    """Growing the radius only to reach the new chunk leaves old members uncovered."""
    real_round = orc.round_up_f32
    state = {"n": 0}

    def close_no_shift(idx, K):
        K = np.asarray(K, dtype=np.float64)
        lo, hi = int(idx.bounds[-1]), idx.T
        mu_x, r_x, _ = orc.chunk_node(K[lo:hi], idx.geometry)
        n_x = hi - lo
        p = -1
        if idx.L > 1:
            p, _ = orc.nearest_fine_cluster(idx, mu_x)
            a = p
            for level in range(1, idx.L):
                n_a = int(idx.nchunk[level][a])
                mu_a = idx.center[level][a]
                new = orc.store_f32((n_a * mu_a + mu_x) / (n_a + 1))
                reach = math.sqrt(float(((mu_x - new) ** 2).sum())) + r_x
                idx.center[level][a] = new
                idx.radius[level][a] = float(real_round(max(idx.radius[level][a], reach)))   # no shift
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
    monkeypatch.setattr(orc, "close_chunk", close_no_shift)
    assert _fails(P.test_append_keeps_invariants, orc.TOKEN_BALL, 2) or \
        _fails(P.test_append_keeps_invariants, orc.TOKEN_BALL, 3)


def test_kmeans_argmin_is_caught(monkeypatch):
    real_argmax = np.argmax

    def bad_kmeans(X, k, iters, trace=None, margins=None):
        N = X.shape[0]
        m = np.stack([X[(c * N) // k] for c in range(k)]).astype(np.float64)
        labels = np.argmin(X @ m.T, axis=1)
        return labels, m
    monkeypatch.setattr(orc, "spherical_kmeans", bad_kmeans)
    assert _fails(P.test_kmeans_k_equals_n_and_separated_clusters)
    assert _fails(P.test_hand_example_index)


def test_kmeans_unnormalised_update_and_wrong_start_are_caught(monkeypatch):
    """Mistakes that keep the objective monotone and still separate clear clusters: only the
    comparison with the library's nearest-codeword iterations sees them."""
    def mean_update(X, k, iters, trace=None):
        N = X.shape[0]
        m = np.stack([X[(c * N) // k] for c in range(k)]).astype(np.float64)
        labels = np.zeros(N, dtype=np.int64)
        for _ in range(iters):
            labels = np.argmax(X @ m.T, axis=1)
            for c in range(k):
                if np.any(labels == c):
                    m[c] = X[labels == c].mean(axis=0)          # wrong: not projected back onto the sphere
        return labels, m

    def first_k_start(X, k, iters, trace=None):
        m = X[:k].astype(np.float64).copy()                     # wrong: first k points instead of strided
        labels = np.zeros(X.shape[0], dtype=np.int64)
        for _ in range(iters):
            labels = np.argmax(X @ m.T, axis=1)
            for c in range(k):
                if np.any(labels == c):
                    m[c] = orc.unit(X[labels == c].sum(axis=0))
        return labels, m

    for bad in (mean_update, first_k_start):
        monkeypatch.setattr(orc, "spherical_kmeans", bad)
        assert _fails(P.test_kmeans_equals_library_nearest_codeword_iterations, 1, 200, 128, 13) or \
            _fails(P.test_kmeans_equals_library_nearest_codeword_iterations, 3, 500, 32, 32), bad.__name__
