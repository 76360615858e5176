"""Operation counts of the method on a synthetic workload, and the algorithmic
bytes per match-step derived from them (used by the benchmark's roofline line).

TEST / MEASUREMENT INFRASTRUCTURE: calls only the CPU checker and the input
generator.  Counts cover the generation phase only (the timed steps), not the
prompt ingest.

    python -m oracle.count_ops cfg2 [--corpus-limit N]

Pricing (bytes the method itself must move, at 16 B per table item, whatever a
particular layout fetches around it):
  probes        "t in s.next" tests: static Transfer (Algorithm 1) and the chain
                loops of Expand (Algorithm 2)                          16 B each
  records       state records read: one per static suffix-link move, one per
                state visited by Expand's loops, one per appended token (the
                target q or the root)                                   16 B each
  inserts, redirects                                                    16 B each
  clone copies  one read and one write per copied transition            32 B each
  states        new states and clones written                           16 B each
  tokens        accepted token read + text append                    4 + 4 B each
  gather        draft read + draft write, 4 + 4 B per draft token; 16 B of
                per-sequence step inputs/outputs (count, match_len, draft_len,
                source)
The dynamic Transfer of Section 3.3 is not priced: its result equals
(link(last), len(link(last))) after Expand, which needs no extra reads.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle.sam_oracle import Batch, Sam  # noqa: E402
from paper_2411_10666_amd.synth import CONFIGS, make_workload  # noqa: E402


def _totals(ob):
    tot = {}
    for q in ob.seqs:
        for k, v in q.counters().items():
            tot[k] = tot.get(k, 0) + v
    return tot


def count(spec, corpus_limit=None, batch_limit=None):
    w = make_workload(spec)
    corpus = w.corpus
    if corpus is not None and corpus_limit and len(corpus) > corpus_limit:
        corpus = corpus[:corpus_limit]
    nb = spec.batch if not batch_limit else min(spec.batch, batch_limit)
    def progress(done, total):          # a corpus of 500 M tokens takes minutes
        print("[count_ops] corpus automaton: %d of %d tokens" % (done, total), file=sys.stderr,
              flush=True)

    static = Sam.build(corpus, progress=progress) if corpus is not None else None
    ob = Batch(static, corpus, [w.prompts[b] for b in range(nb)], spec.max_accept,
               spec.draft_len, spec.l_bias)
    before = _totals(ob)
    n_draft = 0
    src_hist = np.zeros(3, dtype=np.int64)
    for s in range(w.steps):
        ml, src, dl, d = ob.step(np.ascontiguousarray(w.accepted[s, :nb]),
                                 np.ascontiguousarray(w.counts[s, :nb]))
        n_draft += int(dl.sum())
        src_hist += np.bincount(src, minlength=3)
    after = _totals(ob)
    c = {k: after[k] - before[k] for k in after}
    tokens = int(w.counts[:, :nb].sum())
    seq_steps = w.steps * nb
    n_probe = c["static_probes"] + c["dyn_expand_probe"]
    n_rec = c["static_link_hops"] + c["dyn_expand_probe"] + tokens
    n_state = tokens + c["dyn_clone"]
    walk_bytes = (16 * (n_probe + n_rec + c["dyn_insert"] + c["dyn_redirect"] + n_state)
                  + 32 * c["dyn_copy"] + 8 * tokens)
    gather_bytes = 8 * n_draft + 16 * seq_steps
    return dict(workload=spec.name, sequences=nb, corpus_tokens=0 if corpus is None else len(corpus),
                match_steps=tokens, sequence_steps=seq_steps, steps=w.steps,
                counters=c, draft_tokens=n_draft,
                source_hist=dict(none=int(src_hist[0]), dynamic=int(src_hist[1]),
                                 static=int(src_hist[2])),
                per_match_step=dict(
                    static_probes=c["static_probes"] / tokens,
                    static_link_hops=c["static_link_hops"] / tokens,
                    expand_probes=c["dyn_expand_probe"] / tokens,
                    inserts=c["dyn_insert"] / tokens,
                    redirects=c["dyn_redirect"] / tokens,
                    clones=c["dyn_clone"] / tokens,
                    copies=c["dyn_copy"] / tokens,
                    draft_tokens=n_draft / tokens),
                walk_bytes_per_match_step=walk_bytes / tokens,
                gather_bytes_per_match_step=gather_bytes / tokens,
                algo_bytes_per_match_step=(walk_bytes + gather_bytes) / tokens)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("config", choices=sorted(CONFIGS))
    ap.add_argument("--corpus-limit", type=int, default=0)
    ap.add_argument("--batch-limit", type=int, default=0)
    a = ap.parse_args()
    print(json.dumps(count(CONFIGS[a.config], a.corpus_limit or None, a.batch_limit or None),
                     indent=1))


if __name__ == "__main__":
    main()
