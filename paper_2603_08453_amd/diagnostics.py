"""Retrieval-quality diagnostics (host side, numpy): the paper's recall rate (Table 3 caption)
and its two stability metrics (Appendix D: Jaccard similarity of consecutive retrieved sets,
window hit rate with w = 32).  They read the ids that lc_retrieve returns; none of this is on
the decode hot path."""
from __future__ import annotations

from typing import Iterable, List, Sequence

import numpy as np


def selected_tokens(bounds: np.ndarray, T: int, ids: Sequence[int]) -> np.ndarray:
    """Token positions attended for a list of chunk ids: the chunks plus the open tail."""
    b = np.asarray(bounds, dtype=np.int64)
    parts = [np.arange(b[j], b[j + 1]) for j in ids] + [np.arange(b[-1], T)]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)


def recall_rate(logits: np.ndarray, attended: np.ndarray, k: int) -> float:
    """Share of the k tokens with the highest full-attention logits that were retrieved.
    logits [T] (any monotone function of the attention weight), attended = token positions."""
    k = min(k, len(logits))
    if k == 0:
        return 1.0
    top = np.argpartition(-logits, k - 1)[:k]
    return float(np.isin(top, attended).sum()) / k


def jaccard(a: Iterable[int], b: Iterable[int]) -> float:
    a, b = set(a), set(b)
    return 1.0 if not (a | b) else len(a & b) / len(a | b)


def window_hit(history: List[Iterable[int]], current: Iterable[int], w: int = 32) -> float:
    """Share of the currently retrieved ids that appeared in one of the last w retrieved sets."""
    cur = set(current)
    if not cur:
        return 1.0
    seen = set()
    for s in history[-w:]:
        seen |= set(s)
    return len(cur & seen) / len(cur)
