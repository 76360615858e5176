"""Drive the HIP library and the CPU checker over the same workload and compare
every output element by element (all integers: the bar is bit-exact)."""
from __future__ import annotations

import numpy as np


def run_gpu(corpus, vocab, prompts, accepted, counts, max_seq_len, max_accept, draft_len,
            l_bias=0, gpu_corpus=None, collect_every=1, l_threshold=-1):
    """prompts: list of int32 arrays.  accepted [S,B,A], counts [S,B].
    -> list over steps of dict(match_len, source, draft_len, draft, cursors[B,4], sizes[B,3])."""
    import torch
    from paper_2411_10666_amd import binding as sam
    dev = torch.device("cuda:0")
    B = len(prompts)
    if gpu_corpus is None and corpus is not None:
        gpu_corpus = sam.sam_build(corpus, vocab)
    offs = np.zeros(B + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(p) for p in prompts])
    flat = np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]) if offs[-1] else np.zeros(1, np.int32)
    d_tok = torch.from_numpy(flat).to(dev)
    d_off = torch.from_numpy(offs).to(dev)
    batch = sam.sam_batch_init(gpu_corpus, d_tok, d_off, B, vocab, max_seq_len, max_accept,
                               draft_len, l_bias)
    if l_threshold >= 0:
        sam.sam_batch_set_threshold(batch, l_threshold)
    d_acc = torch.from_numpy(np.ascontiguousarray(accepted, dtype=np.int32)).to(dev)
    d_cnt = torch.from_numpy(np.ascontiguousarray(counts, dtype=np.int32)).to(dev)
    i32 = dict(dtype=torch.int32, device=dev)
    ml = torch.empty(B, **i32); dl = torch.empty(B, **i32); src = torch.empty(B, **i32)
    dr = torch.empty(B, draft_len, **i32)
    cur = [torch.empty(B, **i32) for _ in range(4)]
    siz = [torch.empty(B, **i32) for _ in range(3)]
    out = []
    S = int(d_cnt.shape[0])
    for s in range(S):
        sam.sam_batch_step(batch, d_acc[s], d_cnt[s], ml, dr, dl, src)
        if s % collect_every == 0 or s == S - 1:
            sam.sam_batch_debug(batch, *cur)
            sam.sam_batch_sizes(batch, *siz)
            torch.cuda.synchronize()
            out.append(dict(step=s, match_len=ml.cpu().numpy(), source=src.cpu().numpy(),
                            draft_len=dl.cpu().numpy(), draft=dr.cpu().numpy(),
                            cursors=np.stack([c.cpu().numpy() for c in cur], axis=1),
                            sizes=np.stack([c.cpu().numpy() for c in siz], axis=1)))
    status = sam.sam_batch_status(batch)
    return out, status, batch


def run_oracle(corpus, prompts, accepted, counts, max_accept, draft_len, l_bias=0,
               static=None, collect_every=1, l_threshold=-1):
    from oracle.sam_oracle import Batch, Sam
    if static is None and corpus is not None:
        static = Sam.build(corpus)
    ob = Batch(static, corpus, prompts, max_accept, draft_len, l_bias, l_threshold)
    out = []
    S = len(counts)
    for s in range(S):
        ml, src, dl, d = ob.step(accepted[s], counts[s])
        if s % collect_every == 0 or s == S - 1:
            sizes = np.array([[q._L.oseq_text_len(q._h), q.dynamic().num_states,
                               q.dynamic().num_trans] for q in ob.seqs], dtype=np.int32)
            out.append(dict(step=s, match_len=ml, source=src, draft_len=dl, draft=d,
                            cursors=ob.cursors(), sizes=sizes))
    return out, ob


def assert_same(gpu_out, ref_out, has_static=True):
    assert len(gpu_out) == len(ref_out)
    for g, r in zip(gpu_out, ref_out):
        s = r["step"]
        for k in ("match_len", "source", "draft_len", "draft", "sizes"):
            assert np.array_equal(g[k], r[k]), "step %d: %s differs\n%s\n%s" % (s, k, g[k], r[k])
        gc, rc = g["cursors"], r["cursors"]
        if not has_static:
            gc, rc = gc[:, 2:], rc[:, 2:]
        assert np.array_equal(gc, rc), "step %d: cursors differ\n%s\n%s" % (s, gc, rc)
