"""Seeded synthetic inputs for the suffix-automaton draft path.

This module only draws token streams and acceptance schedules.  It contains
none of the method's arithmetic (no automaton, no matching, no draft logic) and
imports nothing from the HIP binding or from the CPU checker, so both can be fed
from it.

Stand-in for the paper's evaluation data (Section 4, "Models and Tasks" and
"Experiment Setup"): token ids follow a Zipf law, which approximates the unigram
skew of natural-language token streams, and a stated fraction of positions is
overwritten by copies of earlier spans, which reproduces the one property the
method exploits: generated text that repeats corpus or prompt text.

All draws come from ``numpy.random.default_rng([seed, purpose, index])`` so every
(workload, purpose, sequence) has its own reproducible sub-stream.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional

import numpy as np

_PURPOSE_CORPUS = 1
_PURPOSE_CORPUS_COPY = 2
_PURPOSE_SEQUENCE = 3
_PURPOSE_SCHEDULE = 4

_CHUNK = 1 << 24


@dataclass(frozen=True)
class WorkloadSpec:
    """Parameters of one synthetic workload.

    corpus_tokens == 0 means "no corpus" (dynamic automaton only); then the
    generated part of a sequence copies spans from that sequence's own prompt.
    """

    name: str
    corpus_tokens: int
    vocab: int
    zipf_s: float
    corpus_copy_frac: float
    corpus_copy_mean: float
    batch: int
    prompt_len: int
    gen_len: int
    seq_copy_frac: float
    seq_copy_mean: float
    max_accept: int
    draft_len: int
    l_bias: int = 0
    seed: int = 0

    @property
    def max_seq_len(self) -> int:
        return self.prompt_len + self.gen_len

    def scaled(self, **kw) -> "WorkloadSpec":
        return replace(self, **kw)


# The five benchmark workloads (index i here is "config i+1" in the docs).
CONFIGS = {
    "cfg1": WorkloadSpec("cfg1", 100_000, 32000, 1.1, 0.30, 20.0, 8, 256, 768,
                         0.5, 20.0, 8, 16),
    "cfg2": WorkloadSpec("cfg2", 10_000_000, 32000, 1.1, 0.30, 20.0, 64, 2048, 2048,
                         0.5, 20.0, 8, 16),
    "cfg3": WorkloadSpec("cfg3", 100_000_000, 32000, 1.05, 0.40, 32.0, 256, 1024, 4096,
                         0.5, 32.0, 12, 24),
    "cfg4": WorkloadSpec("cfg4", 0, 32000, 1.1, 0.0, 1.0, 1024, 6000, 2048,
                         0.7, 24.0, 16, 32),
    "cfg5": WorkloadSpec("cfg5", 500_000_000, 128256, 1.1, 0.35, 40.0, 1024, 2048, 4096,
                         0.5, 40.0, 16, 32),
}


def _zipf_cdf(vocab: int, s: float) -> np.ndarray:
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    cdf[-1] = 1.0
    return cdf


def zipf_tokens(rng: np.random.Generator, n: int, cdf: np.ndarray) -> np.ndarray:
    """n tokens with P(id = r-1) proportional to r**-s, by inverse CDF."""
    out = np.empty(n, dtype=np.int32)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        u = rng.random(hi - lo)
        out[lo:hi] = np.searchsorted(cdf, u, side="right").astype(np.int32)
    np.minimum(out, len(cdf) - 1, out=out)
    return out


def _copy_events(rng: np.random.Generator, length: int, frac: float, mean: float):
    """Positions and lengths of copy events over a stream of `length` slots.

    Scanning left to right, every slot that is not inside a copy starts one with
    probability q = f / (m (1 - f) + f); a copy has length Geometric(1/m) on
    {1, 2, ...}.  Returns (start, span) arrays, spans clipped to the stream end.
    """
    if frac <= 0.0 or length <= 0:
        z = np.zeros(0, dtype=np.int64)
        return z, z
    q = frac / (mean * (1.0 - frac) + frac)
    starts, spans = [], []
    pos = 0
    while pos < length:
        k = max(1024, int(1.2 * (length - pos) * q) + 64)
        gaps = rng.geometric(q, size=k).astype(np.int64) - 1   # singles before a copy
        lens = rng.geometric(1.0 / mean, size=k).astype(np.int64)
        # start_j = pos + sum_{i<=j} gaps_i + sum_{i<j} lens_i
        st = pos + np.cumsum(gaps) + np.concatenate(([0], np.cumsum(lens[:-1])))
        keep = st < length
        m = int(keep.sum())
        starts.append(st[:m])
        spans.append(lens[:m])
        if m < k:
            break
        pos = int(st[-1] + lens[-1])
    start = np.concatenate(starts)
    span = np.concatenate(spans)
    span = np.minimum(span, length - start)
    return start, span


def make_corpus(spec: WorkloadSpec) -> Optional[np.ndarray]:
    """Zipf stream with a fraction of positions overwritten by copies of earlier
    spans of the same stream (source start uniform among the spans that end at
    or before the copy's start; the event is skipped if none fits)."""
    n = spec.corpus_tokens
    if n <= 0:
        return None
    cdf = _zipf_cdf(spec.vocab, spec.zipf_s)
    c = zipf_tokens(np.random.default_rng([spec.seed, _PURPOSE_CORPUS, 0]), n, cdf)
    rng = np.random.default_rng([spec.seed, _PURPOSE_CORPUS_COPY, 0])
    start, span = _copy_events(rng, n, spec.corpus_copy_frac, spec.corpus_copy_mean)
    u = rng.random(len(start))
    src = np.floor(u * (start - span + 1)).astype(np.int64)
    for i, l, j in zip(start.tolist(), span.tolist(), src.tolist()):
        if i < l:
            continue
        c[i:i + l] = c[j:j + l]
    return c


def _mixture(rng: np.random.Generator, length: int, frac: float, mean: float,
             source: np.ndarray, cdf: np.ndarray) -> np.ndarray:
    """Zipf tokens interleaved with spans copied from uniform positions of `source`."""
    x = zipf_tokens(rng, length, cdf)
    if source is None or len(source) == 0:
        return x
    start, span = _copy_events(rng, length, frac, mean)
    span = np.minimum(span, len(source))
    u = rng.random(len(start))
    src = np.floor(u * (len(source) - span + 1)).astype(np.int64)
    for i, l, j in zip(start.tolist(), span.tolist(), src.tolist()):
        x[i:i + l] = source[j:j + l]
    return x


@dataclass
class Workload:
    spec: WorkloadSpec
    corpus: Optional[np.ndarray]          # int32 [n] or None
    prompts: np.ndarray                   # int32 [B, prompt_len]
    generated: np.ndarray                 # int32 [B, gen_len]
    counts: np.ndarray                    # int32 [steps, B]
    accepted: np.ndarray                  # int32 [steps, B, max_accept], pad 0
    prompt_offsets: np.ndarray = field(default=None)  # int64 [B+1]

    @property
    def steps(self) -> int:
        return int(self.counts.shape[0])

    @property
    def match_steps(self) -> int:
        return int(self.counts.sum())


def make_sequences(spec: WorkloadSpec, corpus: Optional[np.ndarray]):
    cdf = _zipf_cdf(spec.vocab, spec.zipf_s)
    B = spec.batch
    prompts = np.empty((B, spec.prompt_len), dtype=np.int32)
    gen = np.empty((B, spec.gen_len), dtype=np.int32)
    for b in range(B):
        rng = np.random.default_rng([spec.seed, _PURPOSE_SEQUENCE, b])
        if corpus is not None:
            both = _mixture(rng, spec.prompt_len + spec.gen_len, spec.seq_copy_frac,
                            spec.seq_copy_mean, corpus, cdf)
            prompts[b] = both[:spec.prompt_len]
            gen[b] = both[spec.prompt_len:]
        else:
            prompts[b] = zipf_tokens(rng, spec.prompt_len, cdf)
            gen[b] = _mixture(rng, spec.gen_len, spec.seq_copy_frac, spec.seq_copy_mean,
                              prompts[b], cdf)
    return prompts, gen


def make_schedule(spec: WorkloadSpec, gen: np.ndarray):
    """Per step and sequence, count ~ Uniform{1..A} clipped to what is left of the
    generated part; a finished sequence gets count 0 until all have finished."""
    B, G, A = spec.batch, spec.gen_len, spec.max_accept
    rng = np.random.default_rng([spec.seed, _PURPOSE_SCHEDULE, 0])
    done = np.zeros(B, dtype=np.int64)
    counts, accepted = [], []
    while (done < G).any():
        c = rng.integers(1, A + 1, size=B, dtype=np.int64)
        c = np.minimum(c, G - done)
        acc = np.zeros((B, A), dtype=np.int32)
        idx = done[:, None] + np.arange(A)[None, :]
        valid = np.arange(A)[None, :] < c[:, None]
        acc[valid] = gen[np.nonzero(valid)[0], idx[valid]]
        counts.append(c.astype(np.int32))
        accepted.append(acc)
        done += c
    if not counts:
        return (np.zeros((0, B), dtype=np.int32), np.zeros((0, B, A), dtype=np.int32))
    return np.stack(counts), np.stack(accepted)


def make_workload(spec: WorkloadSpec, corpus: Optional[np.ndarray] = None) -> Workload:
    """Build the whole workload.  Pass a corpus made earlier to skip regenerating it."""
    if corpus is None:
        corpus = make_corpus(spec)
    prompts, gen = make_sequences(spec, corpus)
    counts, accepted = make_schedule(spec, gen)
    offs = (np.arange(spec.batch + 1, dtype=np.int64) * spec.prompt_len)
    return Workload(spec, corpus, prompts, gen, counts, accepted, offs)
