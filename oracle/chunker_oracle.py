"""CPU oracle for structure-aware chunking -- TEST INFRASTRUCTURE ONLY.

Section 4.3 ("Structure-Aware Chunking") and Appendix B: tokens are accumulated greedily; once
the chunk has reached the minimum length the algorithm looks, up to the maximum length, for the
natural delimiter of highest priority and cuts right after it; without any delimiter the chunk is
cut at the maximum length.  Delimiter priorities are those of the paper's separator table
(level 1 structural ... level 4 whitespace).

Readings where the paper is silent: a token's level is decided by how its text *ends* (trailing
blanks ignored for levels 1-3), except that a blank line, a horizontal rule, a code fence or a
newline anywhere in the token counts; among several delimiters of the best level inside the window
the earliest wins; the last chunk of a text may be shorter than the minimum.

Pinned by tests/test_chunker.py on hand-worked token lists.
"""
from typing import List, Sequence

LEVEL1_ENDS = ("}", "]", ">")
LEVEL1_ANY = ("\n\n", "---", "***", "```")
LEVEL2_ENDS = (".", "?", "!", "。", "？", "！")
LEVEL3_ENDS = (",", ";", ":", "，", "；", "：", "、")


def separator_level(token: str) -> int:
    """1 (strongest) .. 4 (whitespace), 0 = no delimiter."""
    body = token.rstrip(" \t")
    if any(m in token for m in LEVEL1_ANY) or body.endswith(LEVEL1_ENDS):
        return 1
    if "\n" in token or body.endswith(LEVEL2_ENDS):
        return 2
    if body.endswith(LEVEL3_ENDS):
        return 3
    if token != "" and (token[-1] in " \t" or token.strip(" \t") == ""):
        return 4
    return 0


def chunk_tokens(tokens: Sequence[str], min_len: int, max_len: int) -> List[int]:
    """Chunk boundaries b_0 = 0 < ... < b_M = len(tokens)."""
    assert 1 <= min_len <= max_len
    n = len(tokens)
    bounds = [0]
    pos = 0
    while pos < n:
        lo = pos + min_len - 1                  # last token of the shortest allowed chunk
        hi = min(pos + max_len, n) - 1          # last token of the longest allowed chunk
        cut = hi
        best = 5
        for e in range(lo, hi + 1):
            lv = separator_level(tokens[e])
            if lv != 0 and lv < best:
                best, cut = lv, e
        pos = cut + 1
        bounds.append(pos)
    return bounds
