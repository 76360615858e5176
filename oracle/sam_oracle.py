"""ctypes wrapper over the plain-C CPU checker in ``sam_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the CPU-baseline leg
of the benchmark may import this; the GPU library never does, and this module
never imports the GPU library.  The arithmetic lives in the C file (Algorithms 1
and 2, Sections 3.2-3.3 of arxiv 2411.10666); this file only marshals arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sam_oracle.c")
_LIB = os.path.join(_HERE, "libsam_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the checker with gcc (plain C, -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_i32p = C.POINTER(C.c_int32)
_i64p = C.POINTER(C.c_int64)


def _p32(a):
    return a.ctypes.data_as(_i32p)


def _p64(a):
    return a.ctypes.data_as(_i64p)


def lib():
    global _lib
    with _lock:
        if _lib is None:
            L = C.CDLL(build())
            L.osam_new.restype = C.c_void_p
            L.osam_free.argtypes = [C.c_void_p]
            L.osam_expand.argtypes = [C.c_void_p, C.c_int32]
            L.osam_expand.restype = C.c_int
            L.osam_extend.argtypes = [C.c_void_p, _i32p, C.c_int64]
            L.osam_extend.restype = C.c_int
            L.osam_build.argtypes = [_i32p, C.c_int64]
            L.osam_build.restype = C.c_void_p
            L.osam_transfer.argtypes = [C.c_void_p, C.c_int32, _i32p, _i32p, C.c_void_p]
            L.osam_num_states.argtypes = [C.c_void_p]
            L.osam_num_states.restype = C.c_int64
            L.osam_num_trans.argtypes = [C.c_void_p]
            L.osam_num_trans.restype = C.c_int64
            L.osam_last.argtypes = [C.c_void_p]
            L.osam_last.restype = C.c_int32
            L.osam_dump_states.argtypes = [C.c_void_p, _i32p, _i32p, _i32p, _i32p]
            L.osam_dump_trans.argtypes = [C.c_void_p, _i32p, _i32p, _i32p]
            L.osam_dump_trans.restype = C.c_int64
            L.osam_counters.argtypes = [C.c_void_p, _i64p]
            L.osam_init_topk.argtypes = [C.c_void_p, C.c_int32]
            L.osam_init_topk.restype = C.c_int
            L.osam_dump_topk.argtypes = [C.c_void_p, C.c_void_p, _i32p, _i32p, C.c_void_p]
            L.osam_prim.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _i32p, _i32p,
                                    C.c_void_p]
            L.osam_prim.restype = C.c_int32
            L.oseq_new.argtypes = [C.c_void_p, _i32p, C.c_int64]
            L.oseq_new.restype = C.c_void_p
            L.oseq_free.argtypes = [C.c_void_p]
            L.oseq_feed.argtypes = [C.c_void_p, _i32p, C.c_int32]
            L.oseq_feed.restype = C.c_int
            L.oseq_draft.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _i32p, _i32p]
            L.oseq_cursors.argtypes = [C.c_void_p, _i32p]
            L.oseq_dynamic.argtypes = [C.c_void_p]
            L.oseq_dynamic.restype = C.c_void_p
            L.oseq_text_len.argtypes = [C.c_void_p]
            L.oseq_text_len.restype = C.c_int64
            L.oseq_counters.argtypes = [C.c_void_p, _i64p]
            L.obatch_step.argtypes = [C.POINTER(C.c_void_p), C.c_int32, _i32p, _i32p,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      _i32p, _i32p, _i32p, _i32p]
            L.obatch_step.restype = C.c_int
            L.obatch_run.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_int32, _i32p, _i32p,
                                     C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                     _i32p, _i32p, _i32p, _i32p]
            L.obatch_run.restype = C.c_int
            _lib = L
    return _lib


class Sam:
    """A suffix automaton (Appendix A.1).  ``Sam()`` is INIT_SAM; ``Sam.build`` is
    Build-SAM; ``expand`` is Expand (Algorithm 2); ``transfer`` is Algorithm 1."""

    def __init__(self, handle=None, owned=True):
        self._L = lib()
        self._h = handle if handle is not None else self._L.osam_new()
        self._owned = owned
        if not self._h:
            raise MemoryError("osam_new failed")

    @classmethod
    def build(cls, tokens, progress=None, chunk=1 << 24) -> "Sam":
        """Build-SAM.  With `progress` (a callable taking done, total) the tokens
        are fed in chunks and it is called between them."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        if progress is None:
            h = lib().osam_build(_p32(t), len(t))
            if not h:
                raise MemoryError("osam_build failed")
            return cls(h)
        S = cls()
        for lo in range(0, len(t), chunk):
            progress(lo, len(t))
            part = t[lo:lo + chunk]
            if S._L.osam_extend(S._h, _p32(part), len(part)) != 0:
                raise MemoryError("osam_extend failed")
        return S

    def __del__(self):
        if getattr(self, "_owned", False) and getattr(self, "_h", None):
            self._L.osam_free(self._h)
            self._h = None

    def expand(self, t: int) -> None:
        if self._L.osam_expand(self._h, int(t)) != 0:
            raise MemoryError("osam_expand failed")

    def transfer(self, t: int, s: int, l: int):
        cs, cl = C.c_int32(s), C.c_int32(l)
        self._L.osam_transfer(self._h, int(t), C.byref(cs), C.byref(cl), None)
        return cs.value, cl.value

    @property
    def num_states(self) -> int:
        return self._L.osam_num_states(self._h)

    @property
    def num_trans(self) -> int:
        return self._L.osam_num_trans(self._h)

    @property
    def last(self) -> int:
        return self._L.osam_last(self._h)

    def states(self):
        """(link, length, min_endpos, n_next), each int32 [num_states]."""
        n = self.num_states
        a = [np.empty(n, dtype=np.int32) for _ in range(4)]
        self._L.osam_dump_states(self._h, *[_p32(x) for x in a])
        return tuple(a)

    def transitions(self):
        """(src, token, dst), each int32 [num_trans], state-major, token-sorted."""
        m = self.num_trans
        a = [np.empty(m, dtype=np.int32) for _ in range(3)]
        k = self._L.osam_dump_trans(self._h, *[_p32(x) for x in a])
        assert k == m, (k, m)
        return tuple(a)

    def counters(self) -> dict:
        o = np.zeros(5, dtype=np.int64)
        self._L.osam_counters(self._h, _p64(o))
        return dict(zip(["insert", "redirect", "clone", "copy", "expand_probe"], o.tolist()))

    def init_topk(self, k: int) -> None:
        """Algorithm 3: freq per state, top-k successors and their probabilities."""
        if self._L.osam_init_topk(self._h, k) != 0:
            raise MemoryError("osam_init_topk failed")
        self._k = k

    def topk(self):
        """(freq uint64 [n], token int32 [n,k], target int32 [n,k], prob float32 [n,k]);
        unused entries have token = target = -1."""
        n, k = self.num_states, self._k
        freq = np.empty(n, dtype=np.uint64)
        tok = np.empty((n, k), dtype=np.int32)
        dst = np.empty((n, k), dtype=np.int32)
        prob = np.empty((n, k), dtype=np.float32)
        self._L.osam_dump_topk(self._h, freq.ctypes.data_as(C.c_void_p), _p32(tok), _p32(dst),
                               prob.ctypes.data_as(C.c_void_p))
        return freq, tok, dst, prob

    def prim(self, state: int, token: int, max_size: int):
        """Algorithm 4 -> (tokens, parents, probs), each of the draft's length."""
        t = np.empty(max_size, dtype=np.int32)
        p = np.empty(max_size, dtype=np.int32)
        pr = np.empty(max_size, dtype=np.float32)
        n = self._L.osam_prim(self._h, state, token, max_size, _p32(t), _p32(p),
                              pr.ctypes.data_as(C.c_void_p))
        if n < 0:
            raise MemoryError("osam_prim failed")
        return t[:n], p[:n], pr[:n]


class Sequence:
    """One decoding sequence: a cursor on the shared static automaton plus the
    sequence's own dynamic automaton, updated in the order of Section 3.3."""

    def __init__(self, static: Sam | None, corpus: np.ndarray | None):
        self._L = lib()
        self._static = static
        self._corpus = None if corpus is None else np.ascontiguousarray(corpus, dtype=np.int32)
        self._h = self._L.oseq_new(static._h if static is not None else None,
                                   _p32(self._corpus) if self._corpus is not None else None,
                                   0 if self._corpus is None else len(self._corpus))
        if not self._h:
            raise MemoryError("oseq_new failed")

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.oseq_free(self._h)
            self._h = None

    def feed(self, tokens) -> None:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        if self._L.oseq_feed(self._h, _p32(t), len(t)) != 0:
            raise MemoryError("oseq_feed failed")

    def draft(self, L: int, l_bias: int = 0, l_threshold: int = -1):
        """-> dict(match_len, source, draft_len, endpos, state, draft[L])."""
        o = np.zeros(5, dtype=np.int32)
        d = np.empty(L, dtype=np.int32)
        self._L.oseq_draft(self._h, L, l_bias, l_threshold, _p32(o), _p32(d))
        return dict(match_len=int(o[0]), source=int(o[1]), draft_len=int(o[2]),
                    endpos=int(o[3]), state=int(o[4]), draft=d)

    def cursors(self):
        """-> (s1, l1, s2, l2)."""
        o = np.zeros(4, dtype=np.int32)
        self._L.oseq_cursors(self._h, _p32(o))
        return tuple(int(v) for v in o)

    def dynamic(self) -> Sam:
        return Sam(self._L.oseq_dynamic(self._h), owned=False)

    def counters(self) -> dict:
        o = np.zeros(8, dtype=np.int64)
        self._L.oseq_counters(self._h, _p64(o))
        k = ["static_probes", "static_link_hops", "static_next_moves",
             "dynamic_probes", "dynamic_link_hops", "dynamic_next_moves",
             "identity_violations", "canon_hops"]
        d = dict(zip(k, o.tolist()))
        d.update({"dyn_" + a: b for a, b in self.dynamic().counters().items()})
        return d


class Batch:
    """B independent sequences stepped together (the shape of the GPU library's
    batch calls): ``init`` feeds the prompts, ``step`` feeds accepted tokens and
    returns (match_len, source, draft_len, draft)."""

    def __init__(self, static: Sam | None, corpus, prompts, max_accept: int,
                 draft_len: int, l_bias: int = 0, l_threshold: int = -1):
        self._L = lib()
        self.seqs = [Sequence(static, corpus) for _ in range(len(prompts))]
        for s, p in zip(self.seqs, prompts):
            s.feed(p)
        self.A, self.Ld, self.l_bias = max_accept, draft_len, l_bias
        self.l_threshold = l_threshold
        self._arr = (C.c_void_p * len(self.seqs))(*[s._h for s in self.seqs])

    def step(self, accepted, counts):
        B = len(self.seqs)
        acc = np.ascontiguousarray(accepted, dtype=np.int32).reshape(B, self.A)
        cnt = np.ascontiguousarray(counts, dtype=np.int32).reshape(B)
        ml = np.empty(B, dtype=np.int32)
        src = np.empty(B, dtype=np.int32)
        dl = np.empty(B, dtype=np.int32)
        d = np.empty((B, self.Ld), dtype=np.int32)
        rc = self._L.obatch_step(self._arr, B, _p32(acc), _p32(cnt), self.A, self.Ld,
                                 self.l_bias, self.l_threshold, _p32(ml), _p32(src), _p32(dl),
                                 _p32(d))
        if rc != 0:
            raise MemoryError("obatch_step failed")
        return ml, src, dl, d

    def run(self, accepted, counts):
        """All rows of accepted [S, B, A] and counts [S, B] one after the other in
        one call; returns (match_len, source, draft_len, draft) with a leading S."""
        B = len(self.seqs)
        cnt = np.ascontiguousarray(counts, dtype=np.int32)
        S = cnt.shape[0]
        cnt = cnt.reshape(S, B)
        acc = np.ascontiguousarray(accepted, dtype=np.int32).reshape(S, B, self.A)
        ml = np.empty((S, B), dtype=np.int32)
        src = np.empty((S, B), dtype=np.int32)
        dl = np.empty((S, B), dtype=np.int32)
        d = np.empty((S, B, self.Ld), dtype=np.int32)
        rc = self._L.obatch_run(self._arr, B, S, _p32(acc), _p32(cnt), self.A, self.Ld,
                                self.l_bias, self.l_threshold, _p32(ml), _p32(src), _p32(dl),
                                _p32(d))
        if rc != 0:
            raise MemoryError("obatch_run failed")
        return ml, src, dl, d

    def cursors(self):
        """int32 [B, 4] = (s1, l1, s2, l2) per sequence."""
        return np.array([s.cursors() for s in self.seqs], dtype=np.int32)
