"""Brute-force definitions used to pin the CPU checker (tiny inputs only).

Nothing here builds an automaton: every quantity is computed from its plain
definition by scanning the text (Section 3.1: a node's min_endpos is the earliest
end position of its substrings; Section 3.2: the match is the exact longest
suffix of the current sequence that occurs in the reference text).
"""
from __future__ import annotations


def first_end(text, w, limit=None):
    """End (exclusive index) of the first occurrence of w in text[:limit], or -1."""
    n = len(text) if limit is None else limit
    k = len(w)
    for e in range(k, n + 1):
        if list(text[e - k:e]) == list(w):
            return e
    return -1


def longest_suffix_match(text, x, limit=None):
    """Largest k such that x[-k:] occurs in text[:limit]; -> (k, first end) ."""
    for k in range(len(x), 0, -1):
        e = first_end(text, x[len(x) - k:], limit)
        if e >= 0:
            return k, e
    return 0, -1


def substrings(text):
    """dict: distinct substring (tuple) -> sorted list of end positions."""
    occ = {}
    n = len(text)
    for i in range(n):
        for j in range(i + 1, n + 1):
            occ.setdefault(tuple(text[i:j]), []).append(j)
    return occ


def endpos_classes(text):
    """Suffix-automaton states by definition: classes of substrings with the same
    set of end positions.  -> dict keyed by (max length, first end) with fields
    minlen, link key, transitions {token: key}."""
    occ = substrings(text)
    groups = {}
    for w, ends in occ.items():
        groups.setdefault(tuple(ends), []).append(w)
    key_of = {}
    info = {}
    for ends, ws in groups.items():
        longest = max(ws, key=len)
        key = (len(longest), ends[0])
        info[key] = dict(longest=longest, minlen=min(len(w) for w in ws))
        for w in ws:
            key_of[w] = key
    root = (0, 0)
    info[root] = dict(longest=(), minlen=0)
    key_of[()] = root
    for key, d in info.items():
        w = d["longest"]
        if key == root:
            d["link"] = None
        else:
            d["link"] = key_of[w[len(w) - d["minlen"] + 1:]]
        d["next"] = {}
        for a in set(text):
            wa = w + (a,)
            if wa in key_of:
                d["next"][a] = key_of[wa]
    return info
