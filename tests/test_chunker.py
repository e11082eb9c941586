"""Structure-aware chunker: hand-worked pins for the oracle, and the library's host routine
against the oracle on synthetic token streams (no GPU involved)."""
import os

import numpy as np
import pytest

from oracle import chunker_oracle as co


def test_separator_levels():
    assert [co.separator_level(t) for t in ["}", "x] ", "\n\n", "a---", "```py"]] == [1, 1, 1, 1, 1]
    assert [co.separator_level(t) for t in [".", "end. ", "\n", "ok?", "。"]] == [2, 2, 2, 2, 2]
    assert [co.separator_level(t) for t in [",", "a; ", ":", "、"]] == [3, 3, 3, 3]
    assert [co.separator_level(t) for t in [" ", "foo ", "\t"]] == [4, 4, 4]
    assert [co.separator_level(t) for t in ["foo", "", " bar", "3.14x"]] == [0, 0, 0, 0]


def test_hand_worked_chunks():
    # a delimiter inside the window wins over the forced cut; none -> cut at the maximum; short last chunk
    t = ["a", "b", ".", "c", "d", "e", ",", "f", "g", "h", "i", "j"]
    assert co.chunk_tokens(t, 2, 4) == [0, 3, 7, 11, 12]
    # the strongest delimiter in the window wins even if a weaker one comes first
    assert co.chunk_tokens(["x", ",", "y", "\n\n", "z"], 2, 4) == [0, 4, 5]
    # among equals the earliest wins; delimiters before the minimum length are ignored
    assert co.chunk_tokens(["a", ".", "b", ".", "c"], 2, 4) == [0, 2, 4, 5]
    assert co.chunk_tokens([".", ".", "a", "b", "c", "d"], 3, 4) == [0, 4, 6]
    assert co.chunk_tokens(["foo ", "bar", "baz"], 1, 3) == [0, 1, 3]
    assert co.chunk_tokens(["你好", "，", "世界", "。"], 2, 4) == [0, 4]
    # no delimiter anywhere: fixed-size chunks of the maximum length
    assert co.chunk_tokens(["w"] * 10, 2, 4) == [0, 4, 8, 10]
    assert co.chunk_tokens([], 2, 4) == [0]


def test_invariants_on_random_streams():
    r = np.random.default_rng(0)
    vocab = ["the", " cat", ".", ",", "\n", "\n\n", "}", " ", "x", "。", "foo ", ":", "```", "y"]
    for _ in range(50):
        n = int(r.integers(0, 200))
        toks = [vocab[i] for i in r.integers(0, len(vocab), size=n)]
        mn = int(r.integers(1, 9))
        mx = mn + int(r.integers(0, 9))
        b = co.chunk_tokens(toks, mn, mx)
        lens = np.diff(b)
        assert b[0] == 0 and b[-1] == n and np.all(lens >= 1) and np.all(lens <= mx)
        assert np.all(lens[:-1] >= mn)


def test_library_chunker_matches_oracle():
    from paper_2603_08453_amd import binding as lc
    if not os.path.exists(lc.LIB_PATH):
        from paper_2603_08453_amd import build
        build.build(verbose=False)
    r = np.random.default_rng(1)
    vocab = ["the", " cat", ".", ",", "\n", "\n\n", "}", " ", "x", "。", "foo ", ":", "```", "y", "，", "a]\t",
             "", "\t", "?!", "--", "---"]
    for _ in range(100):
        n = int(r.integers(0, 300))
        toks = [vocab[i] for i in r.integers(0, len(vocab), size=n)]
        mn = int(r.integers(1, 10))
        mx = mn + int(r.integers(0, 10))
        assert lc.lc_chunk_tokens(toks, mn, mx) == co.chunk_tokens(toks, mn, mx)
    assert lc.lc_chunk_tokens(["a", "b", ".", "c", "d", "e", ",", "f", "g", "h", "i", "j"], 2, 4) == [0, 3, 7, 11, 12]
    with pytest.raises(lc.LycheeError):
        lc.lc_chunk_tokens(["a"], 3, 2)
