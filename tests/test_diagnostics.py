"""Hand-checked values for the retrieval-quality metrics (recall rate, Jaccard, window hit)."""
import numpy as np

from paper_2603_08453_amd import diagnostics as D


def test_recall_rate():
    logits = np.array([0.1, 5.0, 3.0, -1.0, 4.0, 2.0])          # top-3 tokens: 1, 4, 2
    assert D.recall_rate(logits, np.array([1, 2, 3]), 3) == 2 / 3
    assert D.recall_rate(logits, np.array([1, 2, 4]), 3) == 1.0
    assert D.recall_rate(logits, np.array([], dtype=int), 3) == 0.0
    assert D.recall_rate(logits, np.arange(6), 100) == 1.0


def test_selected_tokens_and_stability_metrics():
    bounds = np.array([0, 3, 5, 9])
    assert D.selected_tokens(bounds, 11, [0, 2]).tolist() == [0, 1, 2, 5, 6, 7, 8, 9, 10]
    assert D.jaccard([1, 2, 3], [2, 3, 4]) == 2 / 4
    assert D.jaccard([], []) == 1.0
    hist = [[1], [2, 3], [9]]
    assert D.window_hit(hist, [2, 9, 7]) == 2 / 3
    assert D.window_hit(hist, [2, 9, 7], w=1) == 1 / 3
    assert D.window_hit(hist, []) == 1.0
