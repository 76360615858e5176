"""Longest-suffix matching by exhaustive search, straight from the definition.

TEST INFRASTRUCTURE ONLY (like the rest of ``oracle/``): no automaton, no index,
just a scan of the corpus for a token string.  It is what the suffix automaton
computes faster (arxiv 2411.10666, Section 3.2: the longest suffix of the sequence
that occurs in the corpus, and the earliest position where it ends), and it is
affordable at any corpus size for a sample of positions, where the checker's own
automaton over a 500 M-token corpus takes minutes to build.
"""
from __future__ import annotations

import numpy as np


class CorpusScan:
    """Searches over one int32 token corpus (kept as raw little-endian bytes)."""

    def __init__(self, corpus):
        c = np.ascontiguousarray(corpus, dtype="<i4")
        self.n = int(c.size)
        self._bytes = c.tobytes()

    def first_occurrence(self, pattern) -> int:
        """Token index where `pattern` first starts in the corpus, or -1."""
        p = np.ascontiguousarray(pattern, dtype="<i4").tobytes()
        if not p:
            return 0
        start = 0
        while True:
            at = self._bytes.find(p, start)
            if at < 0:
                return -1
            if at % 4 == 0:              # a match of whole tokens, not of shifted bytes
                return at // 4
            start = at + 1

    def occurs(self, pattern) -> bool:
        return self.first_occurrence(pattern) >= 0

    def check_static_match(self, x, t, match_len):
        """Is `match_len` the length of the longest suffix of x[:t] that occurs in the
        corpus?  -> (is_longest, end) with end = the (exclusive) end of the first
        occurrence of that suffix, the paper's min_endpos; (False, -1) if the suffix
        of that length does not occur at all."""
        if match_len == 0:
            return (t == 0 or not self.occurs(x[t - 1:t])), 0
        at = self.first_occurrence(x[t - match_len:t])
        if at < 0:
            return False, -1
        longer = match_len < t and self.occurs(x[t - match_len - 1:t])
        return (not longer), at + match_len

    def draft(self, end, draft_len):
        """The draft_len tokens after a match ending at `end`, cut at the corpus end."""
        return np.frombuffer(self._bytes, dtype="<i4", count=max(0, min(draft_len, self.n - end)),
                             offset=4 * end)
