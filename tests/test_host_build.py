"""Host logic of the library without a GPU: the shared library loads and exports
every declared symbol, argument checks, and the host-built corpus automaton
against the CPU checker (states, links, end positions, every transition)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle.sam_oracle import Sam
from paper_2411_10666_amd import binding as sam
from paper_2411_10666_amd.synth import CONFIGS, make_corpus

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sam.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sam_[a-z_]+)\s*\(", hdr))
    assert declared == set(sam.EXPORTS)
    lib = ctypes.CDLL(sam.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def _compare(corpus_tokens, vocab):
    c = sam.sam_build_host_only(corpus_tokens, vocab)
    ref = Sam.build(corpus_tokens)
    ns, nt, dev = sam.sam_corpus_info(c)
    assert dev == 0
    assert ns == ref.num_states and nt == ref.num_trans
    length, link, endpos = sam.sam_corpus_export(c)
    rlink, rlen, rend, _ = ref.states()
    assert (length == rlen).all() and (link == rlink).all() and (endpos == rend).all()
    return c, ref


@pytest.mark.parametrize("seed", range(8))
def test_host_build_matches_checker_small(seed):
    rng = np.random.default_rng(seed)
    vocab = [2, 3, 5, 50][seed % 4]
    n = int(rng.integers(1, 400))
    x = rng.integers(0, vocab, size=n).astype(np.int32)
    c, ref = _compare(x, vocab)
    src, tok, dst = ref.transitions()
    for s, t, d in zip(src.tolist(), tok.tolist(), dst.tolist()):
        assert sam.sam_corpus_find(c, s, t) == d
    # transitions that do not exist are reported as such (counts already agree)
    for s in range(min(ref.num_states, 50)):
        have = set(tok[src == s].tolist())
        for t in range(vocab):
            if t not in have:
                assert sam.sam_corpus_find(c, s, t) == -1


def test_host_build_matches_checker_cfg1_corpus():
    spec = CONFIGS["cfg1"]
    x = make_corpus(spec)
    c, ref = _compare(x, spec.vocab)
    src, tok, dst = ref.transitions()
    rng = np.random.default_rng(0)
    pick = rng.choice(len(src), size=20000, replace=False)
    for i in pick.tolist():
        assert sam.sam_corpus_find(c, int(src[i]), int(tok[i])) == int(dst[i])


def test_argument_errors():
    with pytest.raises(sam.SamError) as e:
        sam.sam_build_host_only(np.zeros(0, dtype=np.int32), 10)
    assert e.value.code == sam.SAM_EINVAL
    with pytest.raises(sam.SamError) as e:
        sam.sam_build_host_only(np.array([1, 2, 10], dtype=np.int32), 10)
    assert e.value.code == sam.SAM_ETOKEN and "position 2" in str(e.value)
    with pytest.raises(sam.SamError) as e:
        sam.sam_build_host_only(np.array([1, -2], dtype=np.int32), 10)
    assert e.value.code == sam.SAM_ETOKEN
    c = sam.sam_build_host_only(np.array([1, 2, 3], dtype=np.int32), 10)
    with pytest.raises(sam.SamError) as e:
        sam.sam_corpus_find(c, 99, 1)
    assert e.value.code == sam.SAM_EINVAL
    lib = ctypes.CDLL(sam.LIB_PATH)
    assert lib.sam_corpus_info(None, None, None, None) == sam.SAM_EINVAL
    assert lib.sam_batch_step(None, None, None, None, None, None, None, None) == sam.SAM_EINVAL
    assert lib.sam_batch_status(None, None, None) == sam.SAM_EINVAL
    lib.sam_corpus_free(None)
    lib.sam_batch_free(None)


@pytest.mark.parametrize("seed,k", [(0, 1), (1, 2), (2, 3), (3, 4), (4, 8)])
def test_host_topk_matches_checker(seed, k):
    """Algorithm 3 in the library (edge-ordered, no recursion) against the checker's dfs."""
    rng = np.random.default_rng(900 + seed)
    vocab = [2, 3, 5, 9, 40][seed]
    x = rng.integers(0, vocab, size=int(rng.integers(5, 500))).astype(np.int32)
    c = sam.sam_build_host_only(x, vocab)
    sam.sam_corpus_build_topk(c, k)
    ref = Sam.build(x)
    ref.init_topk(k)
    for got, want in zip(sam.sam_corpus_export_topk(c), ref.topk()):
        assert got.dtype == want.dtype and np.array_equal(got, want)


def test_host_topk_cfg1_corpus():
    spec = CONFIGS["cfg1"]
    x = make_corpus(spec)
    c = sam.sam_build_host_only(x, spec.vocab)
    sam.sam_corpus_build_topk(c, 4)
    ref = Sam.build(x)
    ref.init_topk(4)
    for got, want in zip(sam.sam_corpus_export_topk(c), ref.topk()):
        assert np.array_equal(got, want)
    with pytest.raises(sam.SamError) as e:
        sam.sam_corpus_build_topk(c, 9)
    assert e.value.code == sam.SAM_EINVAL


def test_save_and_load_round_trip(tmp_path):
    rng = np.random.default_rng(5)
    x = rng.integers(0, 7, size=5000).astype(np.int32)
    c = sam.sam_build_host_only(x, 7)
    path = str(tmp_path / "corpus.sam")
    sam.sam_corpus_save(c, path)
    d = sam.sam_corpus_load_host_only(path)
    assert sam.sam_corpus_info(d) == sam.sam_corpus_info(c)
    for a, b in zip(sam.sam_corpus_export(c), sam.sam_corpus_export(d)):
        assert np.array_equal(a, b)
    n_states = sam.sam_corpus_info(c)[0]
    for s in rng.integers(0, n_states, size=300).tolist():
        for t in range(7):
            assert sam.sam_corpus_find(c, s, t) == sam.sam_corpus_find(d, s, t)
    # the top-k table is rebuilt from a loaded automaton
    sam.sam_corpus_build_topk(c, 3)
    sam.sam_corpus_build_topk(d, 3)
    for a, b in zip(sam.sam_corpus_export_topk(c), sam.sam_corpus_export_topk(d)):
        assert np.array_equal(a, b)


def test_load_refuses_damaged_files(tmp_path):
    x = np.random.default_rng(6).integers(0, 5, size=800).astype(np.int32)
    c = sam.sam_build_host_only(x, 5)
    path = str(tmp_path / "corpus.sam")
    sam.sam_corpus_save(c, path)
    raw = bytearray(open(path, "rb").read())

    def expect_refused(data):
        bad = str(tmp_path / "bad.sam")
        open(bad, "wb").write(bytes(data))
        with pytest.raises(sam.SamError) as e:
            sam.sam_corpus_load_host_only(bad)
        assert e.value.code == sam.SAM_EINVAL

    expect_refused(raw[:-16])                      # truncated
    expect_refused(raw + b"x")                     # trailing bytes
    expect_refused(b"NOTACORP" + raw[8:])          # wrong magic
    flipped = bytearray(raw)
    off = 64 + 4 * 800 + 4 * 3                     # length of state 3
    flipped[off:off + 4] = (10 ** 6).to_bytes(4, "little")
    expect_refused(flipped)
    # a transition whose target is out of range: first used slot of the table
    n_states = sam.sam_corpus_info(c)[0]
    slots_at = 64 + 4 * 800 + 12 * n_states + 8 * 5
    slots = np.frombuffer(bytes(raw[slots_at:]), dtype=np.uint32).reshape(-1, 4)
    j = int(np.flatnonzero(slots[:, 0] != 0xFFFFFFFF)[0])
    bad_slot = bytearray(raw)
    bad_slot[slots_at + 16 * j + 8:slots_at + 16 * j + 12] = (4 * 10 ** 6).to_bytes(4, "little")
    expect_refused(bad_slot)
    with pytest.raises(sam.SamError):
        sam.sam_corpus_load_host_only(str(tmp_path / "missing.sam"))


def test_loaded_library_was_built_from_the_sources_in_the_tree():
    from paper_2411_10666_amd import build
    lib = ctypes.CDLL(sam.LIB_PATH)
    lib.sam_build_id.restype = ctypes.c_char_p
    assert lib.sam_build_id().decode() == build.source_digest()
