"""Pins for the CPU checker: brute force, automaton invariants, the worked
example, the closed-form identity for the dynamic cursor and the amortised move
bound.  None of these retypes the checker's own procedure."""
import os

import numpy as np
import pytest

from bruteforce import endpos_classes, first_end, longest_suffix_match, substrings
from oracle.sam_oracle import Batch, Sam, Sequence

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "abcbc.txt")


def _rand_text(rng, n, vocab, copy=True):
    x = rng.integers(0, vocab, size=n).tolist()
    if copy and n > 8:
        for _ in range(max(1, n // 12)):
            l = int(rng.integers(2, 7))
            i = int(rng.integers(l, n - l + 1)) if n - l + 1 > l else l
            j = int(rng.integers(0, i - l + 1))
            x[i:i + l] = x[j:j + l]
    return x[:n]


def _cases():
    out = []
    for seed in range(60):
        rng = np.random.default_rng(1000 + seed)
        vocab = [2, 3, 4, 32000][seed % 4]
        n = int(rng.integers(1, 70))
        out.append((seed, vocab, n))
    return out


def _parse_golden():
    sec, data = None, {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            sec = line.strip("[]")
            data[sec] = []
            continue
        data[sec].append(line.split())
    return data


def _structure(sam):
    link, length, endpos, n_next = sam.states()
    src, tok, dst = sam.transitions()
    nxt = [dict() for _ in range(sam.num_states)]
    for s, t, d in zip(src.tolist(), tok.tolist(), dst.tolist()):
        nxt[s][t] = d
    return link.tolist(), length.tolist(), endpos.tolist(), nxt


# --------------------------------------------------------------------------
# worked example (Figure 2's string)

def test_abcbc_table():
    g = _parse_golden()
    text = [0, 1, 2, 1, 2]
    sam = Sam.build(text)
    link, length, endpos, nxt = _structure(sam)
    assert sam.num_states == int(g["totals"][0][0])
    assert sam.num_trans == int(g["totals"][0][1])
    for row in g["states"]:
        i = int(row[0])
        assert (length[i], link[i], endpos[i]) == (int(row[1]), int(row[2]), int(row[3]))
        want = {int(a.split(":")[0]): int(a.split(":")[1]) for a in row[4:]}
        assert nxt[i] == want
    distinct = sum(length[v] - length[link[v]] for v in range(1, sam.num_states))
    assert distinct == int(g["totals"][0][2]) == len(substrings(text))


def _draft_of(field):
    return [] if field == "-" else [int(v) for v in field.split(",")]


def test_abcbc_dynamic_and_static_walks():
    g = _parse_golden()
    text = [0, 1, 2, 1, 2]
    seq = Sequence(None, None)
    for tok, row in zip(text, g["dynamic"]):
        seq.feed([tok])
        d = seq.draft(2)
        assert d["match_len"] == int(row[0])
        assert seq.cursors()[2] == int(row[1])
        assert d["draft"][:d["draft_len"]].tolist() == _draft_of(row[2])
        assert (d["draft"][d["draft_len"]:] == -1).all()
    corpus = np.array(text, dtype=np.int32)
    st = Sam.build(corpus)
    link, length, endpos, _ = _structure(st)
    seq = Sequence(st, corpus)
    # l_bias large and negative is not needed: read the static cursor directly
    for tok, row in zip([2, 1, 2, 0], g["static CBCA"]):
        seq.feed([tok])
        s1, l1, _, _ = seq.cursors()
        assert (l1, s1, endpos[s1]) == (int(row[0]), int(row[1]), int(row[2]))
        want = _draft_of(row[3])
        assert corpus[endpos[s1]:endpos[s1] + 4].tolist() == want


# --------------------------------------------------------------------------
# the automaton against the definition of its states

@pytest.mark.parametrize("seed,vocab,n", _cases())
def test_states_are_endpos_classes(seed, vocab, n):
    rng = np.random.default_rng(seed)
    text = _rand_text(rng, n, vocab)
    sam = Sam.build(text)
    link, length, endpos, nxt = _structure(sam)
    info = endpos_classes(text)
    # identity of a state that does not depend on numbering: (length, first end)
    keys = [(length[v], endpos[v]) for v in range(sam.num_states)]
    assert len(set(keys)) == len(keys)
    assert set(keys) == set(info.keys())
    for v, key in enumerate(keys):
        d = info[key]
        assert (None if link[v] < 0 else keys[link[v]]) == d["link"]
        assert {t: keys[u] for t, u in nxt[v].items()} == d["next"]
        # the longest string of the state is text[endpos-len : endpos)
        assert tuple(text[endpos[v] - length[v]:endpos[v]]) == d["longest"]
    # counting bounds
    if n >= 2:
        assert sam.num_states <= 2 * n - 1
    if n >= 3:
        assert sam.num_trans <= 3 * n - 4
    assert all(length[link[v]] < length[v] for v in range(1, sam.num_states))
    assert sum(length[v] - length[link[v]] for v in range(1, sam.num_states)) == len(substrings(text))
    assert sum(len(d) for d in nxt) == sam.num_trans


@pytest.mark.parametrize("seed,vocab,n", _cases()[:24])
def test_invariants_hold_after_every_expand(seed, vocab, n):
    rng = np.random.default_rng(50 + seed)
    text = _rand_text(rng, n, vocab)
    sam = Sam()
    for k, t in enumerate(text, 1):
        sam.expand(t)
        link, length, endpos, nxt = _structure(sam)
        assert length[sam.last] == k and endpos[sam.last] == k
        for v in range(1, sam.num_states):
            assert length[link[v]] < length[v] <= endpos[v] <= k
            w = text[endpos[v] - length[v]:endpos[v]]
            assert first_end(text[:k], w) == endpos[v]
            # shortest string of the class first ends there as well
            ws = w[len(w) - length[link[v]] - 1:]
            assert first_end(text[:k], ws) == endpos[v]


# --------------------------------------------------------------------------
# matching against the definition of the result

@pytest.mark.parametrize("seed,vocab,n", _cases())
def test_static_and_dynamic_match_brute_force(seed, vocab, n):
    rng = np.random.default_rng(77 + seed)
    corpus = _rand_text(rng, n, vocab)
    m = int(rng.integers(1, 60))
    x = _rand_text(rng, m, vocab)
    # make the sequence share material with the corpus
    if n > 6 and m > 6:
        l = min(6, n, m)
        i = int(rng.integers(0, m - l + 1))
        j = int(rng.integers(0, n - l + 1))
        x[i:i + l] = corpus[j:j + l]
    L = int(rng.integers(1, 9))
    l_bias = int(rng.integers(0, 3))
    carr = np.array(corpus, dtype=np.int32)
    st = Sam.build(carr)
    _, _, endpos1, _ = _structure(st)
    seq = Sequence(st, carr)
    for t in range(1, m + 1):
        seq.feed([x[t - 1]])
        s1, l1, s2, l2 = seq.cursors()
        k1, e1 = longest_suffix_match(corpus, x[:t])
        k2, e2 = longest_suffix_match(x, x[:t], limit=t - 1)
        assert l1 == k1
        assert l2 == k2
        if k1:
            assert endpos1[s1] == e1
        d = seq.draft(L, l_bias)
        if k1 > k2 + l_bias:
            want_src, ml, T, p, Tn = 2, k1, corpus, e1, n
        else:
            want_src, ml, T, p, Tn = 1, k2, x, e2, t
        if ml == 0:
            assert (d["source"], d["match_len"], d["draft_len"]) == (0, 0, 0)
            assert (d["draft"] == -1).all()
            continue
        want = list(T[p:min(p + L, Tn)])
        assert d["source"] == want_src and d["match_len"] == ml and d["endpos"] == p
        assert d["draft"][:d["draft_len"]].tolist() == want
        assert (d["draft"][d["draft_len"]:] == -1).all()
    c = seq.counters()
    assert c["identity_violations"] == 0
    # amortised bound of Appendix A.3: link moves <= tokens, next moves <= tokens
    assert c["static_link_hops"] <= m and c["static_next_moves"] <= m
    assert c["dynamic_link_hops"] <= m and c["dynamic_next_moves"] <= m


@pytest.mark.parametrize("seed", range(12))
def test_dynamic_equals_static_on_prefix(seed):
    """The dynamic result at time t equals a static walk of x[0..t) over an
    automaton built on x[0..t-1)."""
    rng = np.random.default_rng(300 + seed)
    x = _rand_text(rng, int(rng.integers(2, 40)), [2, 3, 5][seed % 3])
    seq = Sequence(None, None)
    for t in range(1, len(x) + 1):
        seq.feed([x[t - 1]])
        _, _, s2, l2 = seq.cursors()
        ref = Sam.build(x[:t - 1])
        _, _, ep, _ = _structure(ref)
        s, l = 0, 0
        for tok in x[:t]:
            s, l = ref.transfer(tok, s, l)
        assert l == l2
        if l:
            dl, dn, de, _ = _structure(seq.dynamic())
            assert de[s2] == ep[s]


def test_dynamic_cursor_is_link_of_last_on_long_input():
    rng = np.random.default_rng(5)
    x = _rand_text(rng, 4000, 3)
    seq = Sequence(None, None)
    seq.feed(x)
    c = seq.counters()
    assert c["identity_violations"] == 0 and c["canon_hops"] > 0
    dyn = seq.dynamic()
    link, length, _, _ = _structure(dyn)
    _, _, s2, l2 = seq.cursors()
    assert s2 == link[dyn.last] and l2 == length[s2]
    assert dyn.num_states <= 2 * len(x) - 1 and dyn.num_trans <= 3 * len(x) - 4


def test_unseen_token_resets_to_root_and_empty_cases():
    corpus = np.array([1, 2, 3, 1, 2], dtype=np.int32)
    st = Sam.build(corpus)
    seq = Sequence(st, corpus)
    seq.feed([1, 2])
    assert seq.cursors()[:2][1] == 2
    seq.feed([9])
    assert seq.cursors()[:2] == (0, 0)
    d = seq.draft(4)
    assert d["source"] == 0 and d["draft_len"] == 0
    # feeding nothing changes nothing
    before = seq.cursors()
    seq.feed([])
    assert seq.cursors() == before
    # empty corpus automaton is just a root
    assert Sam.build([]).num_states == 1


def test_auxiliary_threshold_rule():
    """Section 3.4: the auxiliary drafter has virtual length l_threshold; the
    automaton's draft is kept only for strictly longer matches."""
    corpus = np.array([1, 2, 3, 4, 5, 1, 2, 9], dtype=np.int32)
    st = Sam.build(corpus)
    seq = Sequence(st, corpus)
    seq.feed([7, 1, 2, 3])                       # static match "1 2 3", length 3
    for thr, want in [(-1, 2), (0, 2), (2, 2), (3, 3), (4, 3)]:
        d = seq.draft(4, 0, thr)
        assert d["match_len"] == 3 and d["source"] == want
        assert d["draft"].tolist() == [4, 5, 1, 2]
    seq.feed([8])                                # no match at all
    assert seq.draft(4, 0, -1)["source"] == 0
    assert seq.draft(4, 0, 0)["source"] == 3


def test_batch_matches_single_sequences():
    rng = np.random.default_rng(9)
    corpus = np.array(_rand_text(rng, 300, 6), dtype=np.int32)
    st = Sam.build(corpus)
    B, A, L = 5, 4, 6
    prompts = [np.array(_rand_text(rng, 20, 6), dtype=np.int32) for _ in range(B)]
    batch = Batch(st, corpus, prompts, A, L, 0)
    singles = [Sequence(st, corpus) for _ in range(B)]
    for s, p in zip(singles, prompts):
        s.feed(p)
    for _ in range(10):
        counts = rng.integers(0, A + 1, size=B).astype(np.int32)
        acc = rng.integers(0, 6, size=(B, A)).astype(np.int32)
        ml, src, dl, d = batch.step(acc, counts)
        for b in range(B):
            singles[b].feed(acc[b, :counts[b]])
            r = singles[b].draft(L, 0)
            assert (ml[b], src[b], dl[b]) == (r["match_len"], r["source"], r["draft_len"])
            assert (d[b] == r["draft"]).all()


def test_batch_run_is_the_loop_over_steps():
    rng = np.random.default_rng(19)
    corpus = np.array(_rand_text(rng, 300, 5), dtype=np.int32)
    st = Sam.build(corpus)
    B, A, L, S = 4, 5, 7, 12
    prompts = [np.array(_rand_text(rng, 15, 5), dtype=np.int32) for _ in range(B)]
    counts = rng.integers(0, A + 1, size=(S, B)).astype(np.int32)
    acc = rng.integers(0, 5, size=(S, B, A)).astype(np.int32)
    whole = Batch(st, corpus, prompts, A, L, 0).run(acc, counts)
    stepped = Batch(st, corpus, prompts, A, L, 0)
    for i in range(S):
        for got, want in zip(stepped.step(acc[i], counts[i]), whole):
            assert (got == want[i]).all()


# --------------------------------------------------------------------------
# tree drafts: Algorithm 3 (freq, top-k, probabilities) and Algorithm 4 (Prim)

def _freq_closed_form(text):
    """freq(v) counted from the definition: a path from v that ends in the state
    of the whole prefix T[0..j) contributes 1.  Such a path spells T[e..j) for an
    end position e of v, and it lands in that state iff the string it completes,
    of length j - e + len(v), is longer than the longest suffix of T[0..j) that
    ends at more places than that prefix does (those suffixes are other states)."""
    n = len(text)
    occ = substrings(text)
    other = [0] * (n + 1)        # other[j]: longest suffix of T[:j] with more end positions
    for j in range(1, n + 1):
        for L in range(j - 1, 0, -1):
            if len(occ[tuple(text[j - L:j])]) > len(occ[tuple(text[:j])]):
                other[j] = L
                break
    info = endpos_classes(text)
    out = {}
    for key, d in info.items():
        length = key[0]
        ends = occ[d["longest"]] if length else list(range(0, n + 1))
        f = 0
        for e in ends:
            for j in range(max(e, 1), n + 1):
                if j - e + length > other[j]:
                    f += 1
        out[key] = f
    return out


@pytest.mark.parametrize("seed,vocab,n", _cases()[:32])
def test_freq_and_topk_against_definition(seed, vocab, n):
    rng = np.random.default_rng(400 + seed)
    text = _rand_text(rng, min(n, 40), vocab)
    sam = Sam.build(text)
    k = 1 + seed % 3
    sam.init_topk(k)
    freq, tok, dst, prob = sam.topk()
    link, length, endpos, nxt = _structure(sam)
    want = _freq_closed_form(text)
    for v in range(sam.num_states):
        assert int(freq[v]) == want[(length[v], endpos[v])], (v, text)
        # top-k: successors ranked by (freq desc, token asc)
        ranked = sorted(nxt[v].items(), key=lambda kv: (-int(freq[kv[1]]), kv[0]))[:k]
        for i in range(k):
            if i < len(ranked):
                assert (tok[v, i], dst[v, i]) == ranked[i]
                assert prob[v, i] == np.float32(float(freq[ranked[i][1]]) / float(freq[v]))
            else:
                assert tok[v, i] == -1 and dst[v, i] == -1
        if v:
            assert freq[v] >= 1
        # successors partition what is left after the state's own start value
        own = 0 if (v == 0 or length[v] != endpos[v]) else 1
        assert int(freq[v]) == own + sum(int(freq[u]) for u in nxt[v].values())


def test_freq_worked_example_abcbc():
    """"ABCBC": freq by hand.  Prefix states 1,2,3,4,6 start at 1, clones 5,7 at 0.
    6:{} -> 1; 4:{C:6} -> 2; 7:{B:4} -> 2; 3:{B:4} -> 3; 5:{C:7} -> 2;
    2:{C:3} -> 4; 1:{B:2} -> 5; root:{A:1,B:5,C:7} -> 9."""
    sam = Sam.build([0, 1, 2, 1, 2])
    sam.init_topk(2)
    freq, tok, dst, prob = sam.topk()
    assert freq.tolist() == [9, 5, 4, 3, 2, 2, 1, 2]
    assert tok[0].tolist() == [0, 1] and dst[0].tolist() == [1, 5]      # A (5), then B before C (2 = 2)
    assert prob[0].tolist() == [np.float32(5 / 9), np.float32(2 / 9)]
    t, p, pr = sam.prim(0, 7, 5)
    # start token 7; then A (5/9), AB (5/9 * 4/5), ABC (* 3/4), then B (2/9) vs ABCB (1/3*2/3=2/9):
    assert t.tolist()[:4] == [7, 0, 1, 2] and p.tolist()[:4] == [-1, 0, 1, 2]
    assert pr[0] == np.float32(1.0) and pr[1] == np.float32(5 / 9)


def test_prim_tie_goes_to_the_entry_pushed_first():
    """Hand-worked "AAAB" (tests/golden/aaab_prim.txt): two queue entries with the
    probability 1/4, exact in float, pushed at different pops; the one pushed first is
    expanded first.  Fixes the whole token / parent / probability sequence."""
    rows = [ln.split() for ln in open(os.path.join(os.path.dirname(GOLDEN), "aaab_prim.txt"))
            if ln.strip() and not ln.startswith("#")]
    text = [int(x) for x in rows[0]]
    want_freq = [int(x) for x in rows[1]]
    start_state, start_token, max_size = (int(x) for x in rows[2])
    draft = rows[3:]
    sam = Sam.build(text)
    sam.init_topk(2)
    freq, tok, dst, prob = sam.topk()
    assert freq.tolist() == want_freq
    t, par, pr = sam.prim(start_state, start_token, max_size)
    assert t.tolist() == [int(r[0]) for r in draft]
    assert par.tolist() == [int(r[1]) for r in draft]
    assert pr.tolist() == [np.float32(float(r[2])) for r in draft]
    # a shorter draft is a prefix of the longer one
    t3, par3, _ = sam.prim(start_state, start_token, 3)
    assert t3.tolist() == t.tolist()[:3] and par3.tolist() == par.tolist()[:3]


@pytest.mark.parametrize("seed", range(16))
def test_prim_is_best_first_over_the_topk_tree(seed):
    rng = np.random.default_rng(500 + seed)
    vocab = [2, 3, 6][seed % 3]
    text = _rand_text(rng, int(rng.integers(5, 60)), vocab)
    sam = Sam.build(text)
    k = 1 + seed % 3
    sam.init_topk(k)
    freq, tok, dst, prob = sam.topk()
    max_size = int(rng.integers(1, 24))
    start_state = int(rng.integers(0, sam.num_states))
    t, par, pr = sam.prim(start_state, 99, max_size)
    assert t[0] == 99 and par[0] == -1 and pr[0] == np.float32(1.0)
    # every entry is a top-k successor of its parent's state, with the product probability
    state = [start_state]
    for i in range(1, len(t)):
        ps = state[par[i]]
        j = tok[ps].tolist().index(t[i])
        state.append(int(dst[ps, j]))
        assert pr[i] == np.float32(pr[par[i]]) * prob[ps, j]
        assert par[i] < i
    assert all(pr[i] >= pr[i + 1] for i in range(len(pr) - 1))
    # nothing outside the draft beats anything inside it: enumerate the whole
    # top-k tree to the depth the draft can reach and compare the probability multisets
    best = []
    frontier = [(np.float32(1.0), start_state)]
    for depth in range(max_size):
        nxt_frontier = []
        for p0, s0 in frontier:
            best.append(float(p0))
            for j in range(k):
                if dst[s0, j] >= 0:
                    nxt_frontier.append((np.float32(p0) * prob[s0, j], int(dst[s0, j])))
        frontier = nxt_frontier
        if len(best) > 4000:
            break
    best.sort(reverse=True)
    assert sorted((float(x) for x in pr), reverse=True) == best[:len(pr)]
    assert len(t) == min(max_size, len(best)) or len(best) > 4000


# --------------------------------------------------------------------------
# the exhaustive corpus scan (oracle/bruteforce.py), used where the checker's own
# automaton is too slow to build

@pytest.mark.parametrize("seed,vocab", [(0, 2), (1, 3), (2, 5), (3, 40), (4, 128256)])
def test_corpus_scan_agrees_with_the_automaton(seed, vocab):
    from oracle.bruteforce import CorpusScan
    rng = np.random.default_rng(800 + seed)
    corpus = rng.integers(0, vocab, size=2500).astype(np.int32)
    if vocab > 100:                          # give large vocabularies something to match
        corpus[1200:1300] = corpus[100:200]
    scan = CorpusScan(corpus)
    st = Sam.build(corpus)
    x = rng.integers(0, vocab, size=300).astype(np.int32)
    x[50:120] = corpus[130:200]
    x[200:260] = corpus[2440:2500]           # a match that runs into the end of the corpus
    L = 7
    ob = Batch(st, corpus, [x[:0]], 1, L, 10 ** 6)        # l_bias so large that the draft is never static...
    ob2 = Batch(st, corpus, [x[:0]], 1, L, -10 ** 6)      # ...and so small that it always is
    for t in range(1, len(x) + 1):
        ob.step(x[t - 1:t].reshape(1, 1), np.array([1], np.int32))
        m2, src2, dl2, d2 = ob2.step(x[t - 1:t].reshape(1, 1), np.array([1], np.int32))
        l1 = int(ob.cursors()[0][1])
        longest, end = scan.check_static_match(x, t, l1)
        assert longest, t
        if l1 >= 1:
            assert not scan.check_static_match(x, t, l1 - 1)[0] or l1 == 0      # a shorter suffix is not the longest
            assert int(m2[0]) == l1 and int(src2[0]) == 2
            want = scan.draft(end, L)
            assert int(dl2[0]) == len(want) and np.array_equal(d2[0, :len(want)], want)
        if l1 < t:
            assert not scan.occurs(x[t - l1 - 1:t])


def test_corpus_scan_ignores_matches_of_shifted_bytes():
    from oracle.bruteforce import CorpusScan
    # bytes of the corpus: 00 00 00 02 | 00 00 00 00; the token 0x00020000 (bytes 00 00 02 00)
    # appears at byte offset 1 but is no token of the corpus
    scan = CorpusScan(np.array([0x02000000, 0], dtype=np.int32))
    assert scan.first_occurrence(np.array([0x00020000], dtype=np.int32)) == -1
    assert scan.first_occurrence(np.array([0], dtype=np.int32)) == 1
    assert scan.first_occurrence(np.array([0x02000000, 0], dtype=np.int32)) == 0
    assert scan.draft(1, 5).tolist() == [0] and scan.draft(2, 5).tolist() == []
