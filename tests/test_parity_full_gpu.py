"""Full-size parity, in the launch configuration the benchmark times (the
pre-marshalled step plan, back-to-back launches on one stream, outputs of every
step kept): the whole schedule of a benchmark workload is run through the HIP
library and every output of every step is compared with the CPU checker.

Progress lines go to the terminal as they come (past pytest's capture), and to a log
file as well if SAM_TEST_PROGRESS_DIR names a folder, so that a long, quiet test can
be told from a hung one."""
import os
import threading
import time

import numpy as np
import pytest

from paper_2411_10666_amd.synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROGRESS_DIR = os.environ.get("SAM_TEST_PROGRESS_DIR")      # also append the lines to a file there
_live = None
_say_lock = threading.Lock()


@pytest.fixture(autouse=True)
def _live_progress(capsys):
    """These tests run for minutes: their progress lines go to the terminal as they come,
    past pytest's capture, so that a watcher sees the run is alive."""
    global _live
    _live = capsys
    yield
    _live = None


def _say(msg):
    with _say_lock:                      # the checker's build thread reports too
        _say_locked(msg)


def _say_locked(msg):
    line = "%s [full] %s" % (time.strftime("%H:%M:%S"), msg)
    if PROGRESS_DIR:
        os.makedirs(PROGRESS_DIR, exist_ok=True)
        with open(os.path.join(PROGRESS_DIR, "test_progress.log"), "a") as f:
            f.write(line + "\n")
    if _live is not None:
        with _live.disabled():
            print(line, flush=True)
    else:
        print(line, flush=True)


def _gpu_schedule(w, sequences=None):
    """-> dict of [S, B(, L)] arrays + final cursors and sizes."""
    import torch
    from paper_2411_10666_amd import binding as sam
    spec = w.spec
    dev = torch.device("cuda:0")
    t0 = time.time()
    sam.sam_set_progress_callback(
        lambda phase, done, total: _say("%s: library %s %d/%d" % (spec.name, phase, done, total)))
    try:
        corpus = sam.sam_build(w.corpus, spec.vocab) if w.corpus is not None else None
    finally:
        sam.sam_set_progress_callback(None)
    _say("%s: library built the corpus automaton in %.1f s" % (spec.name, time.time() - t0))
    B, A, L, S = spec.batch, spec.max_accept, spec.draft_len, w.steps
    i32 = dict(dtype=torch.int32, device=dev)
    batch = sam.sam_batch_init(corpus, torch.from_numpy(w.prompts.reshape(-1)).to(dev),
                               torch.from_numpy(w.prompt_offsets).to(dev), B, spec.vocab,
                               spec.max_seq_len, A, L, spec.l_bias)
    acc = torch.from_numpy(w.accepted).to(dev)
    cnt = torch.from_numpy(w.counts).to(dev)
    ml = torch.zeros(S, B, **i32); dl = torch.zeros(S, B, **i32); src = torch.zeros(S, B, **i32)
    dr = torch.zeros(S, B, L, **i32)
    plan = sam.StepPlan(batch, acc, cnt, ml, dr, dl, src)
    plan.run(0, S)
    cur = [torch.empty(B, **i32) for _ in range(4)]
    siz = [torch.empty(B, **i32) for _ in range(3)]
    sam.sam_batch_debug(batch, *cur)
    sam.sam_batch_sizes(batch, *siz)
    torch.cuda.synchronize()
    assert sam.sam_batch_status(batch) == 0
    _say("%s: %d steps on the GPU done" % (spec.name, S))
    return dict(match_len=ml.cpu().numpy(), draft_len=dl.cpu().numpy(), source=src.cpu().numpy(),
                draft=dr.cpu().numpy(),
                cursors=np.stack([c.cpu().numpy() for c in cur], axis=1),
                sizes=np.stack([c.cpu().numpy() for c in siz], axis=1))


def _oracle_static(w):
    """The checker's corpus automaton (None without a corpus)."""
    from oracle.sam_oracle import Sam
    spec = w.spec
    t0 = time.time()
    static = None
    if w.corpus is not None:
        static = Sam.build(w.corpus, progress=lambda done, total: _say(
            "%s: checker build %d/%d" % (spec.name, done, total)))
    _say("%s: checker built the corpus automaton in %.1f s" % (spec.name, time.time() - t0))
    return static


def _oracle_schedule(w, seqs, static=None):
    """The checker on the chosen sequences (all steps)."""
    from oracle.sam_oracle import Batch
    spec = w.spec
    if static is None:
        static = _oracle_static(w)
    ob = Batch(static, w.corpus, [w.prompts[b] for b in seqs], spec.max_accept, spec.draft_len,
               spec.l_bias)
    S, nb, L = w.steps, len(seqs), spec.draft_len
    out = dict(match_len=np.zeros((S, nb), np.int32), draft_len=np.zeros((S, nb), np.int32),
               source=np.zeros((S, nb), np.int32), draft=np.zeros((S, nb, L), np.int32))
    acc = np.ascontiguousarray(w.accepted[:, seqs])
    cnt = np.ascontiguousarray(w.counts[:, seqs])
    for s in range(S):
        m, sr, d_l, d = ob.step(acc[s], cnt[s])
        out["match_len"][s], out["source"][s], out["draft_len"][s], out["draft"][s] = m, sr, d_l, d
    out["cursors"] = ob.cursors()
    out["sizes"] = np.array([[q._L.oseq_text_len(q._h), q.dynamic().num_states,
                              q.dynamic().num_trans] for q in ob.seqs], dtype=np.int32)
    _say("%s: checker ran %d sequences" % (spec.name, nb))
    return out


def _compare(g, r, seqs, has_static=True):
    for k in ("match_len", "draft_len", "source"):
        assert np.array_equal(g[k][:, seqs], r[k]), k
    assert np.array_equal(g["draft"][:, seqs], r["draft"])
    assert np.array_equal(g["sizes"][seqs], r["sizes"])
    gc, rc = g["cursors"][seqs], r["cursors"]
    if not has_static:
        gc, rc = gc[:, 2:], rc[:, 2:]
    assert np.array_equal(gc, rc)


def _sampled(spec, n_check, has_static=True):
    w = make_workload(spec)
    _say("%s: workload generated (corpus %d tokens)" % (spec.name, spec.corpus_tokens))
    # the checker builds its own corpus automaton on another host thread while the
    # library builds and runs (both are foreign calls that release the interpreter lock)
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(1) as pool:
        fut = pool.submit(_oracle_static, w)
        g = _gpu_schedule(w)
        static = fut.result()
    seqs = sorted(set(np.linspace(0, spec.batch - 1, n_check).astype(int).tolist()))
    r = _oracle_schedule(w, seqs, static)
    _compare(g, r, seqs, has_static=has_static)
    T = spec.max_seq_len
    assert (g["sizes"][:, 0] == T).all()
    assert (g["sizes"][:, 1] <= 2 * T - 1).all() and (g["sizes"][:, 2] <= 3 * T - 4).all()
    assert (g["draft_len"] <= spec.draft_len).all()
    assert ((g["source"] == 0) == (g["match_len"] == 0)).all()
    # a draft is a slice of its source text: check the static ones against the corpus
    if w.corpus is not None:
        st = np.argwhere(g["source"] == 2)
        pick = st[np.random.default_rng(0).choice(len(st), size=min(2000, len(st)), replace=False)]
        for s_, b_ in pick.tolist():
            d = g["draft"][s_, b_, :g["draft_len"][s_, b_]]
            assert d.size == 0 or (d >= 0).all()
    return g, r


def test_cfg3_shape_scaled_corpus():
    """Config 3's batch, lengths, accept width and draft length (256 x (1024+4096),
    A=12, L=24, Zipf 1.05, 40 % copied) over a 5 M-token corpus; 24 sequences replayed."""
    _sampled(CONFIGS["cfg3"].scaled(corpus_tokens=5_000_000), 24)


def test_cfg5_shape_scaled_corpus():
    """Config 5's batch, lengths, vocabulary (128256), A=16, L=32 over a 5 M-token
    corpus; 16 sequences replayed."""
    _sampled(CONFIGS["cfg5"].scaled(corpus_tokens=5_000_000), 16)


def test_cfg3_full_corpus():
    """Config 3 at full size: 100 M-token corpus (145 M states: state records and
    transition table both beyond 4 GiB), 256 sequences, the whole schedule; 16
    sequences replayed by the checker.  A few minutes of host time, about 40 GB of
    host memory."""
    _sampled(CONFIGS["cfg3"], 16)


def test_cfg5_full_corpus():
    """Config 5 at full size: 500 M-token corpus (709 M states, 59 GB of tables on the
    device), vocabulary 128256, 1024 sequences, the whole schedule of 519 steps.  The
    checker's own automaton of this corpus takes 8 minutes to build, so the static side
    is checked from the definition instead (oracle/bruteforce.py: exhaustive search of
    the corpus): on sampled (sequence, step) pairs, the reported match is the longest
    suffix that occurs in the corpus, the draft follows the first place where it ends,
    and a dynamic choice means that no longer suffix occurs in the corpus.  The dynamic
    side of the sampled sequences is replayed by the checker in full (its automata are
    small).  About 5 minutes, 70 GB of host memory."""
    from oracle.bruteforce import CorpusScan
    from oracle.sam_oracle import Batch
    spec = CONFIGS["cfg5"]
    w = make_workload(spec)
    _say("cfg5: workload generated (corpus %d tokens)" % spec.corpus_tokens)
    g = _gpu_schedule(w)
    L, S = spec.draft_len, w.steps
    seqs = sorted(set(np.linspace(0, spec.batch - 1, 12).astype(int).tolist()))

    # dynamic side: the checker without a corpus gives (l2, dynamic draft) at every step
    ob = Batch(None, None, [w.prompts[b] for b in seqs], spec.max_accept, L, spec.l_bias)
    acc = np.ascontiguousarray(w.accepted[:, seqs])
    cnt = np.ascontiguousarray(w.counts[:, seqs])
    dyn_len = np.zeros((S, len(seqs)), np.int32)
    dyn_draft = np.zeros((S, len(seqs), L), np.int32)
    dyn_dl = np.zeros((S, len(seqs)), np.int32)
    for s_ in range(S):
        m, _, d_l, d = ob.step(acc[s_], cnt[s_])
        dyn_len[s_], dyn_dl[s_], dyn_draft[s_] = m, d_l, d
    cur = ob.cursors()
    assert np.array_equal(g["cursors"][seqs][:, 2:], cur[:, 2:])           # (s2, l2) at the end
    sizes = np.array([[q._L.oseq_text_len(q._h), q.dynamic().num_states, q.dynamic().num_trans]
                      for q in ob.seqs], dtype=np.int32)
    assert np.array_equal(g["sizes"][seqs], sizes)
    _say("cfg5: checker replayed the dynamic side of %d sequences" % len(seqs))
    src = g["source"][:, seqs]
    ml = g["match_len"][:, seqs]
    # wherever the dynamic automaton was chosen its outputs are the checker's, and
    # wherever the static one was chosen it had the strictly longer match
    dyn = src == 1
    assert np.array_equal(ml[dyn], dyn_len[dyn])
    assert np.array_equal(g["draft_len"][:, seqs][dyn], dyn_dl[dyn])
    assert np.array_equal(g["draft"][:, seqs][dyn], dyn_draft[dyn])
    assert (ml[src == 2] > dyn_len[src == 2]).all()
    assert ((src == 0) == (ml == 0)).all() and (dyn_len[src == 0] == 0).all()

    # static side, from the definition, on a sample
    scan = CorpusScan(w.corpus)
    consumed = spec.prompt_len + np.cumsum(w.counts, axis=0)              # tokens fed after step s
    rng = np.random.default_rng(5)
    pairs = [(int(s_), int(j)) for s_, j in zip(rng.integers(0, S, size=70),
                                                rng.integers(0, len(seqs), size=70))]
    n_static = n_dynamic = 0
    for i, (s_, j) in enumerate(pairs):
        b = seqs[j]
        x = np.concatenate([w.prompts[b], w.generated[b]])
        t = int(consumed[s_, b])
        if src[s_, j] == 2:
            longest, end = scan.check_static_match(x, t, int(ml[s_, j]))
            assert longest and end >= 0, (s_, b)
            want = scan.draft(end, L)
            assert g["draft_len"][s_, b] == len(want), (s_, b)
            assert np.array_equal(g["draft"][s_, b, :len(want)], want), (s_, b)
            assert (g["draft"][s_, b, len(want):] == -1).all()
            n_static += 1
        else:
            # dynamic (or nothing) chosen: no suffix longer than l2 occurs in the corpus
            l2 = int(dyn_len[s_, j])
            assert l2 + 1 > t or not scan.occurs(x[t - l2 - 1:t]), (s_, b)
            n_dynamic += 1
        if i % 10 == 9:
            _say("cfg5: %d of %d sampled outputs checked against the corpus" % (i + 1, len(pairs)))
    assert n_static >= 30, (n_static, n_dynamic)
    # properties that hold for every sequence at any size
    T = spec.max_seq_len
    assert (g["sizes"][:, 0] == T).all()
    assert (g["sizes"][:, 1] <= 2 * T - 1).all() and (g["sizes"][:, 2] <= 3 * T - 4).all()
    assert (g["draft_len"] <= L).all() and ((g["source"] == 0) == (g["match_len"] == 0)).all()


def test_cfg2_full_schedule_every_output():
    spec = CONFIGS["cfg2"]
    w = make_workload(spec)
    g = _gpu_schedule(w)
    seqs = list(range(spec.batch))
    r = _oracle_schedule(w, seqs)
    _compare(g, r, seqs)
    assert (r["source"] == 2).sum() > 1000 and (r["source"] == 1).sum() > 100


def test_cfg4_full_batch_dynamic_only():
    """All 1024 sequences on the GPU at full length; the checker replays every
    16th sequence plus the first and last."""
    spec = CONFIGS["cfg4"]
    w = make_workload(spec)
    g = _gpu_schedule(w)
    seqs = sorted(set(list(range(0, spec.batch, 16)) + [1, spec.batch - 1]))
    r = _oracle_schedule(w, seqs)
    _compare(g, r, seqs, has_static=False)
    # properties that hold for every sequence at any size
    T = spec.max_seq_len
    assert (g["sizes"][:, 0] == T).all()
    assert (g["sizes"][:, 1] <= 2 * T - 1).all() and (g["sizes"][:, 2] <= 3 * T - 4).all()
    assert (g["draft_len"] <= spec.draft_len).all() and (g["match_len"] >= 0).all()
    assert ((g["source"] == 0) == (g["match_len"] == 0)).all()
