"""Parity of the HIP path with the CPU checker, element by element, through the
C ABI.  Everything compared is an integer: match lengths, canonical state ids,
sources, draft lengths, draft tokens and automaton sizes must be identical."""
import numpy as np
import pytest

from parity_util import assert_same, run_gpu, run_oracle
from paper_2411_10666_amd.synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[parity] " + msg, flush=True)


def _random_case(seed, vocab, n_corpus, B, T, A, L, steps, ragged=True):
    rng = np.random.default_rng(seed)
    corpus = rng.integers(0, vocab, size=n_corpus).astype(np.int32) if n_corpus else None
    prompts = []
    for b in range(B):
        pl = int(rng.integers(0, T // 3)) if ragged else T // 4
        p = rng.integers(0, vocab, size=pl).astype(np.int32)
        if corpus is not None and pl > 10:
            j = int(rng.integers(0, n_corpus - 8))
            p[2:10] = corpus[j:j + 8]
        prompts.append(p)
    used = np.array([len(p) for p in prompts])
    counts = np.zeros((steps, B), dtype=np.int32)
    acc = rng.integers(0, vocab, size=(steps, B, A)).astype(np.int32)
    for s in range(steps):
        c = rng.integers(0, A + 1, size=B)
        c = np.minimum(c, T - used)
        counts[s] = c
        used += c
        if corpus is not None:
            for b in range(B):
                if c[b] >= 3 and rng.random() < 0.5:
                    j = int(rng.integers(0, n_corpus - c[b]))
                    acc[s, b, :c[b]] = corpus[j:j + c[b]]
    return corpus, prompts, acc, counts


@pytest.mark.parametrize("seed,vocab", [(0, 2), (1, 3), (2, 4), (3, 7), (4, 40), (5, 32000)])
def test_small_random_static_and_dynamic(seed, vocab):
    B, T, A, L, steps = 13, 300, 6, 9, 40
    _say("small random seed=%d vocab=%d B=%d T=%d" % (seed, vocab, B, T))
    corpus, prompts, acc, counts = _random_case(seed, vocab, 2000, B, T, A, L, steps)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L, l_bias=seed % 3)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L, l_bias=seed % 3)
    assert status == 0
    assert_same(g, r)


@pytest.mark.parametrize("seed,vocab", [(10, 2), (11, 3), (12, 30)])
def test_dynamic_only(seed, vocab):
    B, T, A, L, steps = 9, 500, 16, 32, 30
    _say("dynamic only seed=%d vocab=%d" % (seed, vocab))
    _, prompts, acc, counts = _random_case(seed, vocab, 0, B, T, A, L, steps)
    g, status, _ = run_gpu(None, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(None, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r, has_static=False)


@pytest.mark.parametrize("seed,vocab", [(30, 2), (31, 3), (32, 50)])
def test_wide_layout_forced(seed, vocab):
    """The 32-bit table layout (used for long sequences) on the same small cases."""
    from paper_2411_10666_amd import binding as sam
    B, T, A, L, steps = 11, 300, 6, 9, 40
    _say("wide layout seed=%d vocab=%d" % (seed, vocab))
    corpus, prompts, acc, counts = _random_case(seed, vocab, 1500, B, T, A, L, steps)
    sam.sam_set_layout_override(1)
    try:
        g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    finally:
        sam.sam_set_layout_override(0)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


@pytest.mark.parametrize("mode,T", [(2, 300), (3, 300), (2, 3000)])
@pytest.mark.parametrize("seed,vocab", [(40, 3), (41, 50), (42, 32000)])
def test_tight_slot_tables(seed, vocab, mode, T):
    """Slot tables sized to the bare minimum (a testing mode of the library), both
    layouts, sequences grown to exactly max_seq_len: buckets fill up, lookups and
    inserts sweep on into the next bucket, and the slot an insert takes is often in
    the bucket that was fetched ahead for the next state -- paths that the normal
    sizing makes rare."""
    from paper_2411_10666_amd import binding as sam
    B, A, L = 9, 7, 5
    rng = np.random.default_rng(seed)
    corpus = rng.integers(0, vocab, size=800).astype(np.int32)
    prompts = [rng.integers(0, vocab, size=int(rng.integers(0, T // 5))).astype(np.int32)
               for _ in range(B)]
    used = np.array([len(p) for p in prompts])
    rows_c, rows_a = [], []
    while (used < T).any():
        c = np.minimum(rng.integers(0, A + 1, size=B), T - used)
        a = rng.integers(0, vocab, size=(B, A)).astype(np.int32)
        for b in range(B):                      # now and then repeat what the sequence just said
            if c[b] >= 2 and rng.random() < 0.3:
                a[b, 1:] = a[b, 0]
        rows_c.append(c)
        rows_a.append(a)
        used += c
    counts = np.array(rows_c, dtype=np.int32)
    acc = np.array(rows_a, dtype=np.int32)
    _say("tight tables seed=%d vocab=%d mode=%d T=%d steps=%d" % (seed, vocab, mode, T, len(counts)))
    sam.sam_set_layout_override(mode)
    try:
        g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    finally:
        sam.sam_set_layout_override(0)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


def test_static_table_beyond_4_gib():
    """A corpus automaton whose transition table is 4.5 GiB (testing mode, bit 3): a
    ninth of the lookups land in buckets whose byte offset does not fit 32 bits, so the
    64-bit address arithmetic of Transfer runs with a corpus that builds in a moment.
    Run with the assembly token loops and with the C++ ones on the same automaton."""
    import torch
    from paper_2411_10666_amd import binding as sam
    spec = CONFIGS["cfg1"].scaled(corpus_tokens=40_000, batch=24, prompt_len=300, gen_len=500)
    w = make_workload(spec)
    prompts = [w.prompts[b] for b in range(spec.batch)]
    r, _ = run_oracle(w.corpus, prompts, w.accepted, w.counts, spec.max_accept, spec.draft_len)
    assert sum(int((x["source"] == 2).sum()) for x in r) > 200
    _say("static table beyond 4 GiB: build")
    sam.sam_set_layout_override(8)
    try:
        corpus = sam.sam_build(w.corpus, spec.vocab)
        assert sam.sam_corpus_info(corpus)[2] > (1 << 32) + (1 << 28)
        for mode in (8, 12):
            _say("static table beyond 4 GiB: steps, mode=%d" % mode)
            sam.sam_set_layout_override(mode)
            g, status, _ = run_gpu(w.corpus, spec.vocab, prompts, w.accepted, w.counts,
                                   spec.max_seq_len, spec.max_accept, spec.draft_len,
                                   gpu_corpus=corpus)
            assert status == 0
            assert_same(g, r)
    finally:
        sam.sam_set_layout_override(0)
    del corpus
    torch.cuda.empty_cache()


def _degree_corpus(kind, n, rng):
    if kind == "all_distinct":        # every state but the root has at most one transition
        return rng.permutation(n).astype(np.int32), n
    if kind == "periodic":            # abcabc...: one successor everywhere
        return (np.arange(n) % 7).astype(np.int32), 7
    if kind == "two_way":             # binary: no state can have more than two
        return rng.integers(0, 2, size=n).astype(np.int32), 2
    if kind == "three_way":           # the smallest alphabet with wide states
        return rng.integers(0, 3, size=n).astype(np.int32), 3
    assert kind == "dense"            # short contexts followed by most of the alphabet
    return rng.integers(0, 12, size=n).astype(np.int32), 12


@pytest.mark.parametrize("kind", ["all_distinct", "periodic", "two_way", "three_way", "dense"])
def test_corpora_by_out_degree(kind):
    """The device keeps a state's first two transitions in its record and only those of
    states with more in its table: corpora whose states have none, some or mostly more."""
    from paper_2411_10666_amd import binding as sam
    rng = np.random.default_rng(len(kind))
    n = 6000
    corpus, vocab = _degree_corpus(kind, n, rng)
    B, T, A, L, steps = 11, 400, 7, 10, 40
    _say("corpus by out-degree: %s vocab=%d" % (kind, vocab))
    prompts = []
    for b in range(B):
        j = int(rng.integers(0, n - 40))
        p = corpus[j:j + 30].copy()
        p[rng.integers(0, 30, size=3)] = rng.integers(0, vocab, size=3)
        prompts.append(p.astype(np.int32))
    acc = rng.integers(0, vocab, size=(steps, B, A)).astype(np.int32)
    counts = rng.integers(0, A + 1, size=(steps, B)).astype(np.int32)
    for s_ in range(steps):
        for b in range(B):
            c = int(counts[s_, b])
            if c >= 2 and rng.random() < 0.7:
                j = int(rng.integers(0, n - c))
                acc[s_, b, :c] = corpus[j:j + c]
    gc = sam.sam_build(corpus, vocab)
    n_states, n_trans, dev_bytes = sam.sam_corpus_info(gc)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L, gpu_corpus=gc)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)
    if kind in ("periodic", "two_way"):
        # nothing but (at most) the root is wide: text, 32-byte records, and next to no table
        assert dev_bytes < 4 * n + 32 * n_states + 16 * vocab + 4096


@pytest.mark.parametrize("mode", [0, 16])
def test_steps_replayed_from_a_hip_graph(mode):
    """sam_batch_step allocates nothing, reads nothing back and enqueues one kernel, so a
    step can be captured in a HIP graph: the graph is captured once over fixed input and
    output buffers and replayed for every step of the schedule, the step's tokens copied
    into the input buffers in between; every replay is compared with the checker.
    mode 16: the step kernel with its scout waves."""
    import torch
    from paper_2411_10666_amd import binding as sam
    spec = CONFIGS["cfg1"].scaled(corpus_tokens=30_000, batch=9, prompt_len=120, gen_len=260)
    w = make_workload(spec)
    prompts = [w.prompts[b] for b in range(spec.batch)]
    r, _ = run_oracle(w.corpus, prompts, w.accepted, w.counts, spec.max_accept, spec.draft_len)
    dev = torch.device("cuda:0")
    B, A, L = spec.batch, spec.max_accept, spec.draft_len
    corpus = sam.sam_build(w.corpus, spec.vocab)
    sam.sam_set_layout_override(mode)
    try:
        batch = sam.sam_batch_init(corpus, torch.from_numpy(w.prompts.reshape(-1)).to(dev),
                                   torch.from_numpy(w.prompt_offsets).to(dev), B, spec.vocab,
                                   spec.max_seq_len, A, L, spec.l_bias)
    finally:
        sam.sam_set_layout_override(0)
    i32 = dict(dtype=torch.int32, device=dev)
    acc = torch.zeros(B, A, **i32); cnt = torch.zeros(B, **i32)
    ml = torch.zeros(B, **i32); dl = torch.zeros(B, **i32); src = torch.zeros(B, **i32)
    dr = torch.zeros(B, L, **i32)
    d_acc = torch.from_numpy(w.accepted).to(dev)
    d_cnt = torch.from_numpy(w.counts).to(dev)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    # capture records the launch without running it: the batch is not advanced here
    with torch.cuda.graph(graph):
        sam.sam_batch_step(batch, acc, cnt, ml, dr, dl, src)
    _say("graph captured; replaying %d steps" % w.steps)
    for s_ in range(w.steps):
        acc.copy_(d_acc[s_]); cnt.copy_(d_cnt[s_])
        graph.replay()
        torch.cuda.synchronize()
        for got, key in ((ml, "match_len"), (dl, "draft_len"), (src, "source"), (dr, "draft")):
            assert np.array_equal(got.cpu().numpy(), r[s_][key]), "step %d: %s" % (s_, key)
    assert sam.sam_batch_status(batch) == 0


def test_multi_document_corpus_with_separators():
    """Section 3.1: the documents of a corpus are joined by a separator token into one
    string and one automaton.  40 documents joined by token vocab-1; sequences copy
    stretches that run across a separator, so matches and drafts cross document ends
    (nothing is special-cased: the separator is a token like any other)."""
    rng = np.random.default_rng(4242)
    vocab, sep = 500, 499
    docs = [rng.integers(0, sep, size=int(rng.integers(20, 400))).astype(np.int32) for _ in range(40)]
    corpus = np.concatenate([np.concatenate([d, [sep]]).astype(np.int32) for d in docs])
    sep_at = np.flatnonzero(corpus == sep)
    B, T, A, L, steps = 20, 600, 6, 12, 60
    prompts, acc, counts = [], np.zeros((steps, B, A), np.int32), np.zeros((steps, B), np.int32)
    for b in range(B):
        x = rng.integers(0, sep, size=T).astype(np.int32)
        for _ in range(12):                      # stretches that straddle a separator
            at = int(sep_at[rng.integers(0, len(sep_at) - 1)])
            lo, hi = max(0, at - int(rng.integers(2, 15))), min(len(corpus), at + int(rng.integers(2, 15)))
            pos = int(rng.integers(0, T - (hi - lo)))
            x[pos:pos + hi - lo] = corpus[lo:hi]
        pl = int(rng.integers(50, 200))
        prompts.append(x[:pl])
        used = pl
        for s_ in range(steps):
            c = min(int(rng.integers(0, A + 1)), T - used)
            counts[s_, b] = c
            acc[s_, b, :c] = x[used:used + c]
            used += c
    _say("multi-document corpus: %d documents, %d tokens" % (len(docs), len(corpus)))
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)
    crossing_drafts = sum(int(((x["draft"] == sep).any(axis=1) & (x["source"] == 2)).sum()) for x in r)
    assert crossing_drafts > 20, crossing_drafts
    # a match that itself contains a separator: longer than the distance back to it
    long_static = sum(int(((x["source"] == 2) & (x["match_len"] >= 8)).sum()) for x in r)
    assert long_static > 20, long_static


@pytest.mark.parametrize("mode", [16, 17, 18, 20])
@pytest.mark.parametrize("seed,vocab,A", [(90, 2, 5), (91, 4, 30), (92, 300, 70), (93, 32000, 16)])
def test_scout_waves_change_nothing(seed, vocab, A, mode):
    """The step kernel with its two prefetching waves (testing mode bit 4; by default they
    join at 128 sequences): rows shorter and longer than the scouts reach (64 lanes),
    empty and very short prompts (less history than the scouts look back), every table
    layout, both forms of the token loops.  The scouts only read, so every output must
    be what it is without them."""
    from paper_2411_10666_amd import binding as sam
    B, T, L, steps = 12, 900, 9, 25
    _say("scout waves seed=%d vocab=%d A=%d mode=%d" % (seed, vocab, A, mode))
    corpus, prompts, acc, counts = _random_case(seed, vocab, 3000, B, T, A, L, steps)
    prompts[0] = prompts[0][:0]
    prompts[1] = prompts[1][:2]
    used = np.array([len(p) for p in prompts])
    for s_ in range(steps):                       # shorter prompts leave the counts valid
        counts[s_] = np.minimum(counts[s_], T - used)
        used += counts[s_]
    sam.sam_set_layout_override(mode)
    try:
        g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    finally:
        sam.sam_set_layout_override(0)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


@pytest.mark.parametrize("mode", [4, 6])
@pytest.mark.parametrize("seed,vocab", [(50, 2), (51, 5), (52, 300), (53, 32000)])
def test_cxx_token_loops(seed, vocab, mode):
    """The C++ form of Transfer and Expand (what runs for the wide layout, for a
    sequence's first token and for corpora beyond 2^32 buckets) on the compact
    layout, where the assembly form runs otherwise; also with tight slot tables."""
    from paper_2411_10666_amd import binding as sam
    B, T, A, L, steps = 10, 400, 7, 8, 60
    _say("C++ token loops seed=%d vocab=%d mode=%d" % (seed, vocab, mode))
    corpus, prompts, acc, counts = _random_case(seed, vocab, 3000, B, T, A, L, steps)
    sam.sam_set_layout_override(mode)
    try:
        g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    finally:
        sam.sam_set_layout_override(0)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


def test_wide_layout_chosen_for_large_vocab():
    """A vocabulary above 2^17 does not fit the compact slot key."""
    vocab = 200_000
    B, T, A, L, steps = 6, 400, 8, 8, 30
    _say("large vocab -> wide layout")
    rng = np.random.default_rng(40)
    corpus, prompts, acc, counts = _random_case(40, 5, 1500, B, T, A, L, steps)
    # spread the five symbols over the whole vocabulary, top id included
    remap = np.array([0, 131071, 131072, 199_999, 77], dtype=np.int32)
    corpus = remap[corpus]; prompts = [remap[p] for p in prompts]; acc = remap[acc]
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


def test_compact_layout_top_token_ids():
    """Token ids at the top of the 17-bit range in the compact slot key."""
    vocab = 131072
    B, T, A, L, steps = 6, 400, 8, 8, 30
    _say("compact layout, vocab 2^17")
    corpus, prompts, acc, counts = _random_case(41, 4, 1500, B, T, A, L, steps)
    remap = np.array([0, 131071, 65536, 131070], dtype=np.int32)
    corpus = remap[corpus]; prompts = [remap[p] for p in prompts]; acc = remap[acc]
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


def test_long_rows_and_wide_drafts():
    """max_accept above one wavefront of tokens and draft_len above 64 lanes."""
    B, T, A, L, steps, vocab = 5, 1500, 150, 200, 8, 3
    _say("long rows A=%d L=%d" % (A, L))
    corpus, prompts, acc, counts = _random_case(21, vocab, 3000, B, T, A, L, steps)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


@pytest.mark.parametrize("block", range(4))
def test_many_random_shapes(block):
    """Forty small workloads with random batch, capacity, row width, draft length,
    vocabulary, bias and layout; repeated tokens and periodic texts are common at
    these vocabulary sizes, which exercises clones, redirects and list copies."""
    from paper_2411_10666_amd import binding as sam
    rng = np.random.default_rng(1234 + block)
    for case in range(10):
        vocab = int(rng.choice([2, 2, 3, 3, 4, 6, 11]))
        B = int(rng.integers(1, 70))
        T = int(rng.integers(20, 400))
        A = int(rng.integers(1, 20))
        L = int(rng.integers(1, 40))
        steps = int(rng.integers(3, 30))
        n_corpus = int(rng.integers(40, 3000))
        wide = bool(rng.integers(0, 4) == 0)
        l_bias = int(rng.integers(0, 4))
        seed = int(rng.integers(0, 1 << 30))
        _say("random shape %d.%d: vocab=%d B=%d T=%d A=%d L=%d steps=%d corpus=%d wide=%d seed=%d"
             % (block, case, vocab, B, T, A, L, steps, n_corpus, wide, seed))
        corpus, prompts, acc, counts = _random_case(seed, vocab, n_corpus, B, T, A, L, steps)
        use_corpus = corpus if rng.integers(0, 5) else None
        sam.sam_set_layout_override(1 if wide else 0)
        try:
            g, status, _ = run_gpu(use_corpus, vocab, prompts, acc, counts, T, A, L, l_bias=l_bias,
                                   collect_every=int(rng.integers(1, 4)))
        finally:
            sam.sam_set_layout_override(0)
        r, _ = run_oracle(use_corpus, prompts, acc, counts, A, L, l_bias=l_bias,
                          collect_every=1)
        r = [x for x in r if x["step"] in {y["step"] for y in g}]
        assert status == 0
        assert_same(g, r, has_static=use_corpus is not None)


@pytest.mark.parametrize("vocab,n_corpus,B,T,A,L", [(1, 1, 1, 8, 1, 1), (1, 50, 2, 40, 3, 5),
                                                   (2, 1, 1, 30, 1, 1), (2, 2, 3, 12, 2, 2),
                                                   (5, 3, 1, 2, 1, 4)])
def test_smallest_shapes(vocab, n_corpus, B, T, A, L):
    """One-token alphabet (the text is a^n: every Expand but the first links to the state
    before), one-token corpus, one sequence, rows and drafts of one token, capacity 2."""
    rng = np.random.default_rng(vocab * 100 + n_corpus)
    _say("smallest shapes vocab=%d corpus=%d B=%d T=%d A=%d L=%d" % (vocab, n_corpus, B, T, A, L))
    corpus = rng.integers(0, vocab, size=n_corpus).astype(np.int32)
    prompts = [rng.integers(0, vocab, size=int(rng.integers(0, 2))).astype(np.int32) for _ in range(B)]
    steps = 4 * T
    used = np.array([len(p) for p in prompts])
    acc = rng.integers(0, vocab, size=(steps, B, A)).astype(np.int32)
    counts = np.zeros((steps, B), dtype=np.int32)
    for s_ in range(steps):
        c = np.minimum(rng.integers(0, A + 1, size=B), T - used)
        counts[s_] = c
        used += c
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)
    assert used.min() == T                   # every sequence filled to the last token


def test_maximum_row_and_draft_sizes():
    """max_accept and draft_len at the largest values the library accepts."""
    B, T, A, L, steps, vocab = 3, 9000, 4096, 1024, 3, 3
    _say("maximum sizes A=%d L=%d" % (A, L))
    rng = np.random.default_rng(90)
    corpus = rng.integers(0, vocab, size=4000).astype(np.int32)
    prompts = [rng.integers(0, vocab, size=n).astype(np.int32) for n in (0, 100, 700)]
    acc = rng.integers(0, vocab, size=(steps, B, A)).astype(np.int32)
    acc[1, 1, :3000] = np.tile(corpus[100:1100], 3)      # long copies: long static matches
    counts = np.array([[4096, 1, 17], [0, 3000, 4096], [2000, 4096, 64]], dtype=np.int32)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)
    assert max(int(x["draft_len"].max()) for x in r) == L


@pytest.mark.parametrize("T", [16366, 16367])
def test_layout_switch_at_the_compact_limit(T):
    """max_seq_len 16366 is the last compact-layout size, 16367 the first wide one;
    one sequence is filled to the very end (state ids reach 2T)."""
    B, A, L, vocab = 2, 4096, 8, 2
    _say("layout limit T=%d" % T)
    rng = np.random.default_rng(91)
    corpus = rng.integers(0, vocab, size=1000).astype(np.int32)
    prompts = [rng.integers(0, vocab, size=T - 3 * 4096).astype(np.int32),
               np.zeros(10, np.int32)]
    acc = rng.integers(0, vocab, size=(3, B, A)).astype(np.int32)
    acc[:, 1] = 0                                          # one token repeated
    counts = np.array([[4096, 4096]] * 3, dtype=np.int32)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)
    assert g[-1]["sizes"][0, 0] == T


def test_single_token_sequences_fill_to_capacity():
    """Sequences grown exactly to max_seq_len (the worst-case table sizes), one
    repeated token and a two-token alternation included."""
    vocab, T, A, L = 3, 256, 8, 4
    prompts = [np.zeros(0, np.int32), np.zeros(5, np.int32), np.array([0, 1] * 10, np.int32)]
    B = len(prompts)
    rng = np.random.default_rng(3)
    steps = T // 1
    counts = np.zeros((steps, B), dtype=np.int32)
    acc = np.zeros((steps, B, A), dtype=np.int32)
    used = np.array([len(p) for p in prompts])
    for s in range(steps):
        c = np.minimum(rng.integers(1, A + 1, size=B), T - used)
        counts[s] = c
        used += c
        acc[s, 2] = np.tile([0, 1], A // 2) if s % 2 == 0 else rng.integers(0, vocab, size=A)
    assert (used == T).all()
    _say("fill to capacity T=%d" % T)
    corpus = rng.integers(0, vocab, size=500).astype(np.int32)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


def test_cfg1_full():
    spec = CONFIGS["cfg1"]
    _say("cfg1 full workload")
    w = make_workload(spec)
    prompts = [w.prompts[b] for b in range(spec.batch)]
    g, status, _ = run_gpu(w.corpus, spec.vocab, prompts, w.accepted, w.counts, spec.max_seq_len,
                           spec.max_accept, spec.draft_len)
    r, _ = run_oracle(w.corpus, prompts, w.accepted, w.counts, spec.max_accept, spec.draft_len)
    assert status == 0
    assert_same(g, r)
    assert sum(int((x["source"] == 2).sum()) for x in r) > 0
    assert sum(int((x["source"] == 1).sum()) for x in r) > 0


def test_cfg4_scaled_dynamic_only():
    spec = CONFIGS["cfg4"].scaled(batch=24, prompt_len=1500, gen_len=512)
    _say("cfg4 scaled B=24 T=%d" % spec.max_seq_len)
    w = make_workload(spec)
    prompts = [w.prompts[b] for b in range(spec.batch)]
    g, status, _ = run_gpu(None, spec.vocab, prompts, w.accepted, w.counts, spec.max_seq_len,
                           spec.max_accept, spec.draft_len)
    r, _ = run_oracle(None, prompts, w.accepted, w.counts, spec.max_accept, spec.draft_len)
    assert status == 0
    assert_same(g, r, has_static=False)


def test_device_side_faults_leave_other_sequences_intact():
    import torch
    from paper_2411_10666_amd import binding as sam
    vocab, T, A, L, B = 5, 46, 4, 3, 4
    rng = np.random.default_rng(8)
    corpus = rng.integers(0, vocab, size=200).astype(np.int32)
    prompts = [rng.integers(0, vocab, size=16 if b == 2 else 10).astype(np.int32)
               for b in range(B)]
    steps = 12
    acc = rng.integers(0, vocab, size=(steps, B, A)).astype(np.int32)
    counts = np.full((steps, B), 3, dtype=np.int32)
    # sequence 0: a bad token in step 2 (position 1); sequence 1: a bad count in
    # step 3; sequence 2: runs out of room after step 9 (16 + 3*10 = 46);
    # sequence 3: clean and ends exactly at capacity
    acc_g = acc.copy(); cnt_g = counts.copy()
    acc_g[2, 0, 1] = vocab + 3
    cnt_g[3, 1] = A + 1
    _say("device-side faults")
    g, status, _ = run_gpu(corpus, vocab, prompts, acc_g, cnt_g, T, A, L)
    assert status == (sam.SAM_STATUS_TOKEN | sam.SAM_STATUS_COUNT | sam.SAM_STATUS_CAPACITY)
    # what the checker sees: the faulty part of each row is simply not fed
    cnt_r = counts.copy()
    cnt_r[2, 0] = 1
    cnt_r[3, 1] = 0
    cnt_r[10:, 2] = 0
    r, _ = run_oracle(corpus, prompts, acc, cnt_r, A, L)
    assert_same(g, r)


@pytest.mark.parametrize("l_threshold,l_bias", [(0, 0), (2, 2), (5, 5)])
def test_auxiliary_threshold_hook(l_threshold, l_bias):
    B, T, A, L, steps, vocab = 9, 300, 6, 8, 40, 3
    _say("auxiliary threshold %d" % l_threshold)
    corpus, prompts, acc, counts = _random_case(50 + l_threshold, vocab, 2000, B, T, A, L, steps)
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L, l_bias=l_bias,
                           l_threshold=l_threshold)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L, l_bias=l_bias, l_threshold=l_threshold)
    assert status == 0
    assert_same(g, r)
    srcs = np.concatenate([x["source"] for x in r])
    assert (srcs != 3).any()
    if l_threshold > 0:
        assert (srcs == 3).any()


@pytest.mark.parametrize("seed,vocab,k,max_size", [(60, 2, 2, 40), (61, 3, 3, 16), (62, 6, 4, 70),
                                                   (63, 32000, 4, 40), (64, 3, 8, 128), (65, 4, 1, 5),
                                                   # equal frequencies everywhere (ties in the rows
                                                   # and in the queue), full rows, the largest sizes
                                                   (66, 2, 8, 128), (67, 8, 8, 128), (68, 5, 5, 100),
                                                   (69, 12, 3, 128), (70, 2, 1, 128), (71, 300, 8, 60)])
def test_tree_draft_matches_checker(seed, vocab, k, max_size):
    """Algorithm 4 on the GPU against the checker: tokens, parents, probability bits."""
    import torch
    from oracle.sam_oracle import Sam, Sequence
    from paper_2411_10666_amd import binding as sam
    dev = torch.device("cuda:0")
    B, T, A, L, steps = 10, 200, 6, 4, 12
    _say("tree draft seed=%d vocab=%d k=%d max_size=%d" % (seed, vocab, k, max_size))
    corpus, prompts, acc, counts = _random_case(seed, vocab, 3000, B, T, A, L, steps)
    prompts[0] = np.zeros(0, np.int32)
    counts[:, 0] = 0                                  # one sequence stays empty: size 0
    st = Sam.build(corpus)
    st.init_topk(k)
    gc = sam.sam_build(corpus, vocab)
    sam.sam_corpus_build_topk(gc, k)
    for got, want in zip(sam.sam_corpus_export_topk(gc), st.topk()):
        assert np.array_equal(got, want)
    offs = np.zeros(B + 1, np.int64); offs[1:] = np.cumsum([len(p) for p in prompts])
    batch = sam.sam_batch_init(gc, torch.from_numpy(np.concatenate(prompts)).to(dev),
                               torch.from_numpy(offs).to(dev), B, vocab, T, A, L)
    seqs = [Sequence(st, corpus) for _ in range(B)]
    last = [-1] * B
    for b, p in enumerate(prompts):
        seqs[b].feed(p)
        if len(p):
            last[b] = int(p[-1])
    i32 = dict(dtype=torch.int32, device=dev)
    ml = torch.empty(B, **i32); dl = torch.empty(B, **i32); src = torch.empty(B, **i32)
    dr = torch.empty(B, L, **i32)
    tt = torch.empty(B, max_size, **i32); tp = torch.empty(B, max_size, **i32)
    tpr = torch.empty(B, max_size, dtype=torch.float32, device=dev); ts = torch.empty(B, **i32)
    for s in range(steps):
        sam.sam_batch_step(batch, torch.from_numpy(acc[s]).to(dev), torch.from_numpy(counts[s]).to(dev),
                           ml, dr, dl, src)
        sam.sam_batch_tree_draft(batch, max_size, tt, tp, tpr, ts)
        torch.cuda.synchronize()
        gt, gp, gpr, gs = tt.cpu().numpy(), tp.cpu().numpy(), tpr.cpu().numpy(), ts.cpu().numpy()
        for b in range(B):
            seqs[b].feed(acc[s, b, :counts[s, b]])
            if counts[s, b]:
                last[b] = int(acc[s, b, counts[s, b] - 1])
            if last[b] < 0:
                assert gs[b] == 0 and (gt[b] == -1).all()
                continue
            wt, wp, wpr = st.prim(seqs[b].cursors()[0], last[b], max_size)
            n = len(wt)
            assert gs[b] == n, (s, b)
            assert np.array_equal(gt[b, :n], wt) and np.array_equal(gp[b, :n], wp), (s, b)
            assert np.array_equal(gpr[b, :n].view(np.uint32), wpr.view(np.uint32)), (s, b)
            assert (gt[b, n:] == -1).all() and (gp[b, n:] == -1).all() and (gpr[b, n:] == 0).all()
    # no table, bad size
    plain = sam.sam_build(corpus, vocab)
    b2 = sam.sam_batch_init(plain, torch.from_numpy(np.concatenate(prompts)).to(dev),
                            torch.from_numpy(offs).to(dev), B, vocab, T, A, L)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_tree_draft(b2, max_size, tt, tp, tpr, ts)
    assert e.value.code == sam.SAM_EINVAL
    big = torch.empty(B, 129, **i32)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_tree_draft(batch, 129, big, big, torch.empty(B, 129, device=dev), ts)
    assert e.value.code == sam.SAM_EINVAL


def test_loaded_corpus_behaves_like_a_built_one(tmp_path):
    from paper_2411_10666_amd import binding as sam
    B, T, A, L, steps, vocab = 6, 300, 6, 8, 25, 5
    _say("corpus saved, loaded, used")
    corpus, prompts, acc, counts = _random_case(70, vocab, 3000, B, T, A, L, steps)
    built = sam.sam_build_host_only(corpus, vocab)
    path = str(tmp_path / "c.sam")
    sam.sam_corpus_save(built, path)
    loaded = sam.sam_corpus_load(path)
    assert sam.sam_corpus_info(loaded)[2] > 0
    g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L, gpu_corpus=loaded)
    r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
    assert status == 0
    assert_same(g, r)


@pytest.mark.parametrize("seed,vocab,with_corpus", [(80, 2, True), (81, 3, True), (82, 5, False),
                                                    (83, 32000, True)])
def test_replay_equals_stepwise(seed, vocab, with_corpus):
    """The single-launch replay of a schedule gives the outputs of the step calls,
    including rows with faults, and can be continued by ordinary steps."""
    import torch
    from paper_2411_10666_amd import binding as sam
    dev = torch.device("cuda:0")
    B, T, A, L, steps = 12, 260, 7, 10, 30
    _say("replay seed=%d vocab=%d corpus=%s" % (seed, vocab, with_corpus))
    corpus, prompts, acc, counts = _random_case(seed, vocab, 2500, B, T, A, L, steps)
    if not with_corpus:
        corpus = None
    acc_g, cnt_g = acc.copy(), counts.copy()
    cnt_r = counts.copy()
    cnt_g[5, 2] = A + 3; cnt_r[5, 2] = 0                  # a bad count: row skipped
    if counts[7, 4] >= 2:
        acc_g[7, 4, 1] = vocab + 9; cnt_r[7, 4] = 1        # a bad token: row cut there
    r, _ = run_oracle(corpus, prompts, acc, cnt_r, A, L)
    gc = sam.sam_build(corpus, vocab) if corpus is not None else None
    offs = np.zeros(B + 1, np.int64); offs[1:] = np.cumsum([len(p) for p in prompts])
    flat = np.concatenate(prompts) if offs[-1] else np.zeros(1, np.int32)
    batch = sam.sam_batch_init(gc, torch.from_numpy(flat).to(dev), torch.from_numpy(offs).to(dev),
                               B, vocab, T, A, L)
    i32 = dict(dtype=torch.int32, device=dev)
    first = 20                                            # replay 20 rows, then step the rest
    ml = torch.zeros(first, B, **i32); dl = torch.zeros(first, B, **i32)
    src = torch.zeros(first, B, **i32); dr = torch.zeros(first, B, L, **i32)
    sam.sam_batch_replay(batch, torch.from_numpy(acc_g[:first]).to(dev),
                         torch.from_numpy(cnt_g[:first]).to(dev), ml, dr, dl, src)
    torch.cuda.synchronize()
    for s_ in range(first):
        assert np.array_equal(ml[s_].cpu().numpy(), r[s_]["match_len"]), s_
        assert np.array_equal(src[s_].cpu().numpy(), r[s_]["source"]), s_
        assert np.array_equal(dl[s_].cpu().numpy(), r[s_]["draft_len"]), s_
        assert np.array_equal(dr[s_].cpu().numpy(), r[s_]["draft"]), s_
    m1 = torch.empty(B, **i32); d1 = torch.empty(B, **i32); s1 = torch.empty(B, **i32)
    r1 = torch.empty(B, L, **i32)
    cur = [torch.empty(B, **i32) for _ in range(4)]
    siz = [torch.empty(B, **i32) for _ in range(3)]
    for s_ in range(first, steps):
        sam.sam_batch_step(batch, torch.from_numpy(acc_g[s_]).to(dev),
                           torch.from_numpy(cnt_g[s_]).to(dev), m1, r1, d1, s1)
        sam.sam_batch_debug(batch, *cur)
        sam.sam_batch_sizes(batch, *siz)
        torch.cuda.synchronize()
        assert np.array_equal(m1.cpu().numpy(), r[s_]["match_len"]), s_
        assert np.array_equal(r1.cpu().numpy(), r[s_]["draft"]), s_
        gcur = np.stack([c.cpu().numpy() for c in cur], axis=1)
        rcur = r[s_]["cursors"]
        if corpus is None:
            gcur, rcur = gcur[:, 2:], rcur[:, 2:]
        assert np.array_equal(gcur, rcur), s_
        assert np.array_equal(np.stack([c.cpu().numpy() for c in siz], axis=1), r[s_]["sizes"]), s_
    want = sam.SAM_STATUS_COUNT | (sam.SAM_STATUS_TOKEN if counts[7, 4] >= 2 else 0)
    assert sam.sam_batch_status(batch) == want


def test_reset_recycles_sequences():
    """Continuous batching: some sequences are replaced by new requests in the
    middle of a run; the others carry on untouched."""
    import torch
    from oracle.sam_oracle import Sam, Sequence
    from paper_2411_10666_amd import binding as sam
    dev = torch.device("cuda:0")
    vocab, T, A, L, B = 4, 200, 5, 6, 7
    rng = np.random.default_rng(77)
    corpus = rng.integers(0, vocab, size=1500).astype(np.int32)
    st = Sam.build(corpus)
    gc = sam.sam_build(corpus, vocab)
    prompts = [rng.integers(0, vocab, size=int(rng.integers(0, 40))).astype(np.int32) for _ in range(B)]
    offs = np.zeros(B + 1, np.int64); offs[1:] = np.cumsum([len(p) for p in prompts])
    batch = sam.sam_batch_init(gc, torch.from_numpy(np.concatenate(prompts)).to(dev),
                               torch.from_numpy(offs).to(dev), B, vocab, T, A, L)
    seqs = [Sequence(st, corpus) for _ in range(B)]
    for q, p in zip(seqs, prompts):
        q.feed(p)
    i32 = dict(dtype=torch.int32, device=dev)
    ml = torch.empty(B, **i32); dl = torch.empty(B, **i32); src = torch.empty(B, **i32)
    dr = torch.empty(B, L, **i32)
    cur = [torch.empty(B, **i32) for _ in range(4)]
    siz = [torch.empty(B, **i32) for _ in range(3)]
    used = np.array([len(p) for p in prompts])
    _say("reset / recycle sequences")
    for step in range(60):
        if step in (10, 25, 40):
            pick = sorted(rng.choice(B, size=int(rng.integers(1, 4)), replace=False).tolist())
            newp = [rng.integers(0, vocab, size=int(rng.integers(0, 50))).astype(np.int32) for _ in pick]
            no = np.zeros(len(pick) + 1, np.int64); no[1:] = np.cumsum([len(p) for p in newp])
            flat = np.concatenate(newp) if no[-1] else np.zeros(1, np.int32)
            sam.sam_batch_reset(batch, torch.tensor(pick, **i32), torch.from_numpy(flat).to(dev),
                                torch.from_numpy(no).to(dev))
            for b, p in zip(pick, newp):
                seqs[b] = Sequence(st, corpus)
                seqs[b].feed(p)
                used[b] = len(p)
        c = np.minimum(rng.integers(0, A + 1, size=B), T - used)
        used += c
        acc = rng.integers(0, vocab, size=(B, A)).astype(np.int32)
        sam.sam_batch_step(batch, torch.from_numpy(acc).to(dev), torch.from_numpy(c.astype(np.int32)).to(dev),
                           ml, dr, dl, src)
        sam.sam_batch_debug(batch, *cur)
        sam.sam_batch_sizes(batch, *siz)
        torch.cuda.synchronize()
        for b in range(B):
            seqs[b].feed(acc[b, :c[b]])
            r = seqs[b].draft(L, 0)
            got = (int(ml[b]), int(src[b]), int(dl[b]))
            assert got == (r["match_len"], r["source"], r["draft_len"]), (step, b)
            assert (dr[b].cpu().numpy() == r["draft"]).all(), (step, b)
            assert tuple(int(x[b]) for x in cur) == seqs[b].cursors(), (step, b)
            dyn = seqs[b].dynamic()
            assert (int(siz[0][b]), int(siz[1][b]), int(siz[2][b])) == (used[b], dyn.num_states, dyn.num_trans)
    assert sam.sam_batch_status(batch) == 0
    # argument errors
    two = torch.tensor([1, 1], **i32)
    o3 = torch.tensor([0, 1, 2], dtype=torch.int64, device=dev)
    tok = torch.zeros(4, **i32)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_reset(batch, two, tok, o3)
    assert e.value.code == sam.SAM_EINVAL and "twice" in str(e.value)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_reset(batch, torch.tensor([B], **i32), tok, o3[:2].contiguous())
    assert e.value.code == sam.SAM_EINVAL
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_reset(batch, torch.tensor([0], **i32), torch.zeros(T + 5, **i32),
                            torch.tensor([0, T + 1], dtype=torch.int64, device=dev))
    assert e.value.code == sam.SAM_ECAPACITY


def test_init_errors():
    import torch
    from paper_2411_10666_amd import binding as sam
    dev = torch.device("cuda:0")
    tok = torch.zeros(10, dtype=torch.int32, device=dev)
    off = torch.tensor([0, 10], dtype=torch.int64, device=dev)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_init(None, tok, off, 1, 5, 8, 4, 4)
    assert e.value.code == sam.SAM_ECAPACITY
    bad = torch.tensor([5, 3], dtype=torch.int64, device=dev)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_init(None, tok, bad, 1, 5, 8, 4, 4)
    assert e.value.code == sam.SAM_EINVAL
    tok[4] = 77
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_init(None, tok, off, 1, 5, 16, 4, 4)
    assert e.value.code == sam.SAM_ETOKEN
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_init(None, tok, off, 0, 5, 16, 4, 4)
    assert e.value.code == sam.SAM_EINVAL
    host_only = sam.sam_build_host_only(np.array([1, 2, 3], np.int32), 5)
    with pytest.raises(sam.SamError) as e:
        sam.sam_batch_init(host_only, tok, off, 1, 5, 16, 4, 4)
    assert e.value.code == sam.SAM_EINVAL


def test_membench_gives_plausible_figures():
    """The measurement aid runs and its figures have the right order of magnitude
    (wide brackets: this is no performance test)."""
    from paper_2411_10666_amd import binding as sam
    l2 = sam.sam_membench(sam.MEMBENCH_CHASE, 1 << 20, 4000)
    far = sam.sam_membench(sam.MEMBENCH_CHASE, 1 << 30, 4000)
    assert 20.0 < l2 < 2000.0 and l2 < far < 5000.0
    reads = sam.sam_membench(sam.MEMBENCH_GATHER, 256 << 20, 64, 4096)
    assert 1e9 < reads < 1e12
    copy = sam.sam_membench(sam.MEMBENCH_COPY, 256 << 20)
    assert 2e11 < copy < 8.5e12
    launch = sam.sam_membench(sam.MEMBENCH_LAUNCH, 0, 500, 64)
    assert 0.2 < launch < 200.0
    for args in ((sam.MEMBENCH_CHASE, 3 << 20, 10), (sam.MEMBENCH_GATHER, 1 << 20, 0, 1),
                 (sam.MEMBENCH_COPY, 16), (7, 1 << 20, 1)):
        with pytest.raises(sam.SamError) as e:
            sam.sam_membench(*args)
        assert e.value.code == sam.SAM_EINVAL


@pytest.mark.parametrize("block", range(3))
def test_random_cases_in_every_mode(block):
    """50 small random cases per block: vocabulary, batch, lengths, row and draft sizes
    drawn at random, tokens that repeat themselves, copy the corpus or copy the prompt,
    and the library mode (assembly or C++ token loops, compact or wide tables, normal
    or tight slot tables, with or without the step kernel's scout waves) drawn at random
    too."""
    from paper_2411_10666_amd import binding as sam
    for seed in range(7000 + 50 * block, 7050 + 50 * block):
        rng = np.random.default_rng(seed)
        vocab = int(rng.choice([2, 3, 4, 6, 20, 200, 5000, 32000, 100000]))
        B, T = int(rng.integers(1, 40)), int(rng.integers(20, 1200))
        A, L = int(rng.integers(1, 20)), int(rng.integers(1, 40))
        ncorp = int(rng.integers(0, 4000))
        mode = int(rng.choice([0, 0, 1, 2, 3, 4, 6])) | (16 if rng.random() < 0.5 else 0)
        corpus = rng.integers(0, vocab, size=ncorp).astype(np.int32) if ncorp > 10 else None
        prompts = [rng.integers(0, vocab, size=int(rng.integers(0, T // 2 + 1))).astype(np.int32)
                   for _ in range(B)]
        used = np.array([len(p) for p in prompts])
        rows_c, rows_a = [], []
        for _ in range(int(rng.integers(5, 80))):
            c = np.minimum(rng.integers(0, A + 1, size=B), T - used)
            a = rng.integers(0, vocab, size=(B, A)).astype(np.int32)
            for b in range(B):
                r = rng.random()
                if c[b] >= 2 and r < 0.25:
                    a[b, 1:] = a[b, 0]
                elif corpus is not None and 2 <= c[b] < len(corpus) and r < 0.6:
                    j = int(rng.integers(0, len(corpus) - c[b]))
                    a[b, :c[b]] = corpus[j:j + c[b]]
                elif 2 <= c[b] <= len(prompts[b]) and r < 0.8:
                    j = int(rng.integers(0, len(prompts[b]) - c[b] + 1))
                    a[b, :c[b]] = prompts[b][j:j + c[b]]
            rows_c.append(c)
            rows_a.append(a)
            used += c
        counts = np.array(rows_c, dtype=np.int32)
        acc = np.array(rows_a, dtype=np.int32)
        _say("random case seed=%d vocab=%d B=%d T=%d A=%d L=%d mode=%d" % (seed, vocab, B, T, A, L, mode))
        sam.sam_set_layout_override(mode)
        try:
            g, status, _ = run_gpu(corpus, vocab, prompts, acc, counts, T, A, L)
        finally:
            sam.sam_set_layout_override(0)
        r, _ = run_oracle(corpus, prompts, acc, counts, A, L)
        assert status == 0, seed
        assert_same(g, r)
