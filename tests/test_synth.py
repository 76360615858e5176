"""The seeded input generator: determinism, shapes, and the statistics the
workload recipe states (Zipf head mass, copied fraction, schedule coverage)."""
import numpy as np

from paper_2411_10666_amd.synth import CONFIGS, make_corpus, make_workload


def test_cfg1_shapes_and_determinism():
    spec = CONFIGS["cfg1"]
    w1 = make_workload(spec)
    w2 = make_workload(spec)
    assert w1.corpus.dtype == np.int32 and w1.corpus.shape == (100_000,)
    assert (w1.corpus == w2.corpus).all() and (w1.accepted == w2.accepted).all()
    assert w1.prompts.shape == (8, 256) and w1.generated.shape == (8, 768)
    assert w1.corpus.min() >= 0 and w1.corpus.max() < spec.vocab
    assert w1.prompts.max() < spec.vocab and w1.generated.max() < spec.vocab
    # schedule replays the generated part exactly, 1..A tokens at a time
    assert w1.counts.sum(axis=0).tolist() == [768] * 8
    assert w1.counts.max() <= spec.max_accept and w1.counts.min() >= 0
    for b in range(8):
        fed = np.concatenate([w1.accepted[s, b, :w1.counts[s, b]] for s in range(w1.steps)])
        assert (fed == w1.generated[b]).all()
    assert (w1.counts[:-1].max(axis=1) >= 1).all()
    assert w1.prompt_offsets.tolist() == [256 * i for i in range(9)]


def test_zipf_head_and_copied_fraction():
    spec = CONFIGS["cfg1"].scaled(corpus_tokens=400_000)
    c = make_corpus(spec)
    w = np.arange(1, spec.vocab + 1, dtype=np.float64) ** (-spec.zipf_s)
    p0 = w[0] / w.sum()
    assert abs((c == 0).mean() - p0) < 0.01
    # copied spans make long repeats common: a plain Zipf stream has almost no
    # repeated 8-grams, the corpus has them at about the copied fraction
    g = np.lib.stride_tricks.sliding_window_view(c, 8)
    h = (g.astype(np.int64) * np.array([1, 31, 961, 29791, 923521, 28629151, 887503681, 27512614111])).sum(axis=1)
    _, cnt = np.unique(h, return_counts=True)
    repeated = (cnt[cnt > 1].sum() - (cnt > 1).sum()) / len(h)
    assert 0.10 < repeated < 0.40


def test_dynamic_only_workload_copies_prompt():
    spec = CONFIGS["cfg4"].scaled(batch=4, prompt_len=600, gen_len=200)
    w = make_workload(spec)
    assert w.corpus is None
    assert w.prompts.shape == (4, 600) and w.generated.shape == (4, 200)
    assert w.counts.max() <= 16
    # most generated 4-grams occur in the prompt
    hit = 0
    tot = 0
    for b in range(4):
        grams = {tuple(w.prompts[b, i:i + 4]) for i in range(600 - 3)}
        for i in range(200 - 3):
            tot += 1
            hit += tuple(w.generated[b, i:i + 4]) in grams
    assert hit / tot > 0.4
