"""ctypes binding over the C ABI declared in ``include/sam.h``.

Argument marshalling only: every step of the path runs in the HIP library.  The
functions carry the names of the C entry points.  Device buffers are torch
tensors (PyTorch is used for device memory and streams and nothing else); their
``data_ptr()`` is what crosses the boundary.  If the compiled library is missing
the import of this module fails loudly; there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

SAM_OK, SAM_EINVAL, SAM_ENOMEM, SAM_ECAPACITY, SAM_ETOKEN, SAM_EDEVICE = 0, -1, -2, -3, -4, -5
SAM_STATUS_CAPACITY, SAM_STATUS_TOKEN, SAM_STATUS_COUNT, SAM_STATUS_INTERNAL = 1, 2, 4, 8
SAM_SOURCE_NONE, SAM_SOURCE_DYNAMIC, SAM_SOURCE_STATIC, SAM_SOURCE_AUXILIARY = 0, 1, 2, 3

EXPORTS = [
    "sam_last_error", "sam_build", "sam_build_host_only", "sam_corpus_info",
    "sam_corpus_export", "sam_corpus_find", "sam_corpus_free", "sam_batch_init",
    "sam_batch_step", "sam_batch_debug", "sam_batch_sizes", "sam_batch_status",
    "sam_batch_info", "sam_batch_free", "sam_set_layout_override",
    "sam_batch_reset", "sam_set_progress_callback",
    "sam_batch_set_threshold", "sam_corpus_build_topk", "sam_corpus_export_topk",
    "sam_batch_tree_draft", "sam_corpus_save", "sam_corpus_load", "sam_corpus_load_host_only",
    "sam_batch_replay", "sam_membench", "sam_batch_init_noalloc", "sam_build_id",
]


PROGRESS_FN = C.CFUNCTYPE(None, C.c_char_p, C.c_int64, C.c_int64, C.c_void_p)


class SamError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("sam error %d: %s" % (code, msg))
        self.code = code


def _load():
    # PyTorch ships its own copy of the HIP runtime.  It has to be in the process
    # before this library is, so that both resolve to one runtime (two copies in
    # one process do not both find the GPU).
    import torch  # noqa: F401
    path = _build.LIB
    if not os.path.exists(path):
        _build.build()          # nothing built yet: build once
    L = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.sam_last_error.restype = C.c_char_p
    # a library older than the sources beside it must not be what gets tested or timed
    built_from = None
    if hasattr(L, "sam_build_id"):
        L.sam_build_id.restype = C.c_char_p
        built_from = L.sam_build_id().decode()
    if path == os.path.join(_build.HERE, "libsam_hip.so") and built_from != _build.source_digest():
        raise ImportError("%s was built from other sources (%s) than those in %s (%s): run "
                          "`python -m paper_2411_10666_amd.build`"
                          % (path, built_from, _build.CSRC, _build.source_digest()))
    L.sam_build.argtypes = [vp, i64, i32, C.POINTER(vp)]
    L.sam_build_host_only.argtypes = [vp, i64, i32, C.POINTER(vp)]
    L.sam_corpus_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    L.sam_corpus_export.argtypes = [vp, vp, vp, vp]
    L.sam_corpus_find.argtypes = [vp, i64, i32, C.POINTER(i64)]
    L.sam_corpus_free.argtypes = [vp]
    L.sam_corpus_free.restype = None
    L.sam_batch_init.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, C.POINTER(vp)]
    L.sam_batch_init_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp,
                                         C.POINTER(vp)]
    L.sam_batch_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.sam_set_progress_callback.argtypes = [PROGRESS_FN, vp]
    L.sam_batch_set_threshold.argtypes = [vp, i32]
    L.sam_corpus_build_topk.argtypes = [vp, i32]
    L.sam_corpus_save.argtypes = [vp, C.c_char_p]
    L.sam_corpus_load.argtypes = [C.c_char_p, C.POINTER(vp)]
    L.sam_corpus_load_host_only.argtypes = [C.c_char_p, C.POINTER(vp)]
    L.sam_corpus_export_topk.argtypes = [vp, vp, vp, vp, vp]
    L.sam_batch_tree_draft.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    L.sam_batch_replay.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
    L.sam_batch_reset.argtypes = [vp, vp, i32, vp, vp, vp]
    L.sam_batch_debug.argtypes = [vp, vp, vp, vp, vp, vp]
    L.sam_batch_sizes.argtypes = [vp, vp, vp, vp, vp]
    L.sam_batch_status.argtypes = [vp, C.POINTER(C.c_uint32), vp]
    L.sam_batch_info.argtypes = [vp, C.POINTER(i64)]
    L.sam_set_layout_override.argtypes = [C.c_int]
    L.sam_batch_free.argtypes = [vp]
    L.sam_batch_free.restype = None
    for name in EXPORTS:
        if name not in ("sam_last_error", "sam_corpus_free", "sam_batch_free", "sam_build_id"):
            getattr(L, name).restype = C.c_int
    return L


_lib = _load()
LIB_PATH = _build.LIB


def _check(rc: int):
    if rc != SAM_OK:
        raise SamError(rc, _lib.sam_last_error().decode("utf-8", "replace"))


def _dev_ptr(t, dtype, what):
    """Pointer of a contiguous device tensor of the given torch dtype (None -> NULL)."""
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % what)
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be contiguous %s" % (what, dtype))
    return C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def sam_last_error() -> str:
    return _lib.sam_last_error().decode("utf-8", "replace")


class Corpus:
    """Owner of a ``sam_corpus*``."""

    def __init__(self, handle):
        self._h = handle

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.sam_corpus_free(h)


class Batch:
    """Owner of a ``sam_batch*``; keeps the corpus alive."""

    def __init__(self, handle, corpus, batch, max_accept, draft_len):
        self._h = handle
        self._corpus = corpus
        self.batch, self.max_accept, self.draft_len = batch, max_accept, draft_len

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.sam_batch_free(h)


def _host_tokens(tokens):
    a = np.ascontiguousarray(tokens, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


def sam_build(corpus_tokens, vocab: int) -> Corpus:
    a, p = _host_tokens(corpus_tokens)
    h = C.c_void_p()
    _check(_lib.sam_build(p, a.size, vocab, C.byref(h)))
    return Corpus(h)


def sam_build_host_only(corpus_tokens, vocab: int) -> Corpus:
    a, p = _host_tokens(corpus_tokens)
    h = C.c_void_p()
    _check(_lib.sam_build_host_only(p, a.size, vocab, C.byref(h)))
    return Corpus(h)


def sam_corpus_save(corpus: Corpus, path: str) -> None:
    _check(_lib.sam_corpus_save(corpus._h, os.fsencode(path)))


def sam_corpus_load(path: str) -> Corpus:
    h = C.c_void_p()
    _check(_lib.sam_corpus_load(os.fsencode(path), C.byref(h)))
    return Corpus(h)


def sam_corpus_load_host_only(path: str) -> Corpus:
    h = C.c_void_p()
    _check(_lib.sam_corpus_load_host_only(os.fsencode(path), C.byref(h)))
    return Corpus(h)


def sam_corpus_info(corpus: Corpus):
    """-> (n_states, n_trans, device_bytes)."""
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    _check(_lib.sam_corpus_info(corpus._h, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def sam_corpus_export(corpus: Corpus):
    """-> (length, link, min_endpos) host int32 arrays [n_states]."""
    n = sam_corpus_info(corpus)[0]
    out = [np.empty(n, dtype=np.int32) for _ in range(3)]
    _check(_lib.sam_corpus_export(corpus._h, *[x.ctypes.data_as(C.c_void_p) for x in out]))
    return tuple(out)


def sam_corpus_find(corpus: Corpus, state: int, token: int) -> int:
    t = C.c_int64()
    _check(_lib.sam_corpus_find(corpus._h, state, token, C.byref(t)))
    return t.value


def sam_corpus_build_topk(corpus: Corpus, k: int) -> None:
    _check(_lib.sam_corpus_build_topk(corpus._h, k))
    corpus.top_k = k


def sam_corpus_export_topk(corpus: Corpus):
    """-> (freq uint64 [n], token int32 [n,k], target int32 [n,k], prob float32 [n,k])."""
    n, k = sam_corpus_info(corpus)[0], corpus.top_k
    freq = np.empty(n, dtype=np.uint64)
    tok = np.empty((n, k), dtype=np.int32)
    dst = np.empty((n, k), dtype=np.int32)
    prob = np.empty((n, k), dtype=np.float32)
    _check(_lib.sam_corpus_export_topk(corpus._h, *[x.ctypes.data_as(C.c_void_p)
                                                    for x in (freq, tok, dst, prob)]))
    return freq, tok, dst, prob


def sam_batch_tree_draft(batch: Batch, max_size: int, tokens, parents, probs, sizes,
                         stream=None) -> None:
    import torch
    for name, t in (("tokens", tokens), ("parents", parents), ("probs", probs)):
        if t.numel() != batch.batch * max_size:
            raise ValueError("%s must hold batch * max_size values" % name)
    if sizes.numel() != batch.batch:
        raise ValueError("sizes must hold batch values")
    _check(_lib.sam_batch_tree_draft(batch._h, max_size, _dev_ptr(tokens, torch.int32, "tokens"),
                                     _dev_ptr(parents, torch.int32, "parents"),
                                     _dev_ptr(probs, torch.float32, "probs"),
                                     _dev_ptr(sizes, torch.int32, "sizes"), _stream_ptr(stream)))


def sam_batch_init(corpus, prompt_tokens, prompt_offsets, batch: int, vocab: int,
                   max_seq_len: int, max_accept: int, draft_len: int, l_bias: int = 0,
                   stream=None) -> Batch:
    import torch
    h = C.c_void_p()
    _check(_lib.sam_batch_init(corpus._h if corpus is not None else None,
                               _dev_ptr(prompt_tokens, torch.int32, "prompt_tokens"),
                               _dev_ptr(prompt_offsets, torch.int64, "prompt_offsets"),
                               batch, vocab, max_seq_len, max_accept, draft_len, l_bias,
                               _stream_ptr(stream), C.byref(h)))
    return Batch(h, corpus, batch, max_accept, draft_len)


NOALLOC_MAX_BYTES = 32 * 1024 * 1024


def sam_batch_init_noalloc(corpus, prompt_tokens, prompt_offsets, prompt_offsets_host, batch: int,
                           vocab: int, max_seq_len: int, max_accept: int, draft_len: int,
                           l_bias: int = 0, stream=None) -> Batch:
    """prompt_offsets_host: int64 numpy array, the host copy of prompt_offsets."""
    import torch
    ho = np.ascontiguousarray(prompt_offsets_host, dtype=np.int64)
    if ho.size != batch + 1:
        raise ValueError("prompt_offsets_host must hold batch + 1 values")
    h = C.c_void_p()
    _check(_lib.sam_batch_init_noalloc(corpus._h if corpus is not None else None,
                                       _dev_ptr(prompt_tokens, torch.int32, "prompt_tokens"),
                                       _dev_ptr(prompt_offsets, torch.int64, "prompt_offsets"),
                                       ho.ctypes.data_as(C.c_void_p), batch, vocab, max_seq_len,
                                       max_accept, draft_len, l_bias, _stream_ptr(stream),
                                       C.byref(h)))
    return Batch(h, corpus, batch, max_accept, draft_len)


def sam_batch_step(batch: Batch, accepted, counts, match_len, draft, draft_len, source,
                   stream=None) -> None:
    import torch
    i32 = torch.int32
    if accepted is not None and accepted.numel() != batch.batch * batch.max_accept:
        raise ValueError("accepted must hold batch * max_accept tokens")
    if draft is not None and draft.numel() != batch.batch * batch.draft_len:
        raise ValueError("draft must hold batch * draft_len tokens")
    for name, t in (("counts", counts), ("match_len", match_len), ("draft_len", draft_len),
                    ("source", source)):
        if t is not None and t.numel() != batch.batch:
            raise ValueError("%s must hold batch values" % name)
    _check(_lib.sam_batch_step(batch._h, _dev_ptr(accepted, i32, "accepted"),
                               _dev_ptr(counts, i32, "counts"),
                               _dev_ptr(match_len, i32, "match_len"),
                               _dev_ptr(draft, i32, "draft"),
                               _dev_ptr(draft_len, i32, "draft_len"),
                               _dev_ptr(source, i32, "source"), _stream_ptr(stream)))


def sam_batch_reset(batch: Batch, slots, prompt_tokens, prompt_offsets, stream=None) -> None:
    import torch
    _check(_lib.sam_batch_reset(batch._h, _dev_ptr(slots, torch.int32, "slots"),
                                int(slots.numel()),
                                _dev_ptr(prompt_tokens, torch.int32, "prompt_tokens"),
                                _dev_ptr(prompt_offsets, torch.int64, "prompt_offsets"),
                                _stream_ptr(stream)))


def sam_batch_replay(batch: Batch, accepted, counts, match_len, draft, draft_len, source,
                     stream=None) -> None:
    """All rows of the [steps, ...] tensors in one launch."""
    import torch
    i32 = torch.int32
    S = int(counts.shape[0])
    B, A, L = batch.batch, batch.max_accept, batch.draft_len
    for t, shp, name in ((accepted, (S, B, A), "accepted"), (counts, (S, B), "counts"),
                         (match_len, (S, B), "match_len"), (draft, (S, B, L), "draft"),
                         (draft_len, (S, B), "draft_len"), (source, (S, B), "source")):
        if tuple(t.shape) != shp:
            raise ValueError("%s must have shape %s" % (name, shp))
    _check(_lib.sam_batch_replay(batch._h, S, _dev_ptr(accepted, i32, "accepted"),
                                 _dev_ptr(counts, i32, "counts"),
                                 _dev_ptr(match_len, i32, "match_len"),
                                 _dev_ptr(draft, i32, "draft"),
                                 _dev_ptr(draft_len, i32, "draft_len"),
                                 _dev_ptr(source, i32, "source"), _stream_ptr(stream)))


MEMBENCH_CHASE, MEMBENCH_GATHER, MEMBENCH_COPY, MEMBENCH_LAUNCH = 0, 1, 2, 3


def sam_membench(kind: int, size: int = 0, count: int = 1, workgroups: int = 1) -> float:
    """Memory-system measurement of the current device (see include/sam.h)."""
    out = C.c_double(0.0)
    _check(_lib.sam_membench(C.c_int32(kind), C.c_int64(size), C.c_int64(count),
                             C.c_int32(workgroups), C.byref(out)))
    return out.value


def sam_batch_set_threshold(batch: Batch, l_threshold: int) -> None:
    _check(_lib.sam_batch_set_threshold(batch._h, l_threshold))


class StepPlan:
    """Pre-marshalled arguments for a run of ``sam_batch_step`` calls, one per row
    of the given [steps, ...] device tensors, so that a tight loop pays for the
    C call only.  The tensors are kept alive by the plan."""

    def __init__(self, batch: Batch, accepted, counts, match_len, draft, draft_len, source,
                 stream=None):
        import torch
        i32 = torch.int32
        S = int(counts.shape[0])
        B, A, L = batch.batch, batch.max_accept, batch.draft_len
        shapes = ((accepted, (S, B, A), "accepted"), (counts, (S, B), "counts"),
                  (match_len, (S, B), "match_len"), (draft, (S, B, L), "draft"),
                  (draft_len, (S, B), "draft_len"), (source, (S, B), "source"))
        for t, shp, name in shapes:
            _dev_ptr(t, i32, name)
            if tuple(t.shape) != shp:
                raise ValueError("%s must have shape %s" % (name, shp))
        self._keep = [t for t, _, _ in shapes]
        self._batch = batch
        self._stream = _stream_ptr(stream)
        self.steps = S
        self._args = []
        for s in range(S):
            self._args.append(tuple(C.c_void_p(t.data_ptr() + s * t.stride(0) * 4)
                                    for t, _, _ in shapes))

    def run(self, lo: int, hi: int) -> None:
        """Enqueue steps lo .. hi-1."""
        fn, h, st, args = _lib.sam_batch_step, self._batch._h, self._stream, self._args
        for s in range(lo, hi):
            a = args[s]
            rc = fn(h, a[0], a[1], a[2], a[3], a[4], a[5], st)
            if rc != SAM_OK:
                _check(rc)


def sam_batch_debug(batch: Batch, s1, l1, s2, l2, stream=None) -> None:
    import torch
    i32 = torch.int32
    _check(_lib.sam_batch_debug(batch._h, _dev_ptr(s1, i32, "s1"), _dev_ptr(l1, i32, "l1"),
                                _dev_ptr(s2, i32, "s2"), _dev_ptr(l2, i32, "l2"),
                                _stream_ptr(stream)))


def sam_batch_sizes(batch: Batch, text_len, n_states, n_trans, stream=None) -> None:
    import torch
    i32 = torch.int32
    _check(_lib.sam_batch_sizes(batch._h, _dev_ptr(text_len, i32, "text_len"),
                                _dev_ptr(n_states, i32, "n_states"),
                                _dev_ptr(n_trans, i32, "n_trans"), _stream_ptr(stream)))


def sam_batch_status(batch: Batch, stream=None) -> int:
    st = C.c_uint32()
    _check(_lib.sam_batch_status(batch._h, C.byref(st), _stream_ptr(stream)))
    return st.value


_progress_keep = None


def sam_set_progress_callback(fn) -> None:
    """fn(phase: str, done: int, total: int) or None."""
    global _progress_keep
    if fn is None:
        _progress_keep = None
        _check(_lib.sam_set_progress_callback(PROGRESS_FN(), None))
        return
    cb = PROGRESS_FN(lambda phase, done, total, user: fn(phase.decode(), done, total))
    _progress_keep = cb
    _check(_lib.sam_set_progress_callback(cb, None))


def sam_set_layout_override(mode: int) -> None:
    _check(_lib.sam_set_layout_override(mode))


def sam_batch_info(batch: Batch) -> int:
    b = C.c_int64()
    _check(_lib.sam_batch_info(batch._h, C.byref(b)))
    return b.value
