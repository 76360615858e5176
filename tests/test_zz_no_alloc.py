"""sam_batch_init_noalloc (the entry point for callers that cannot allocate device
memory) against sam_batch_init, through the C ABI: the batch state right after
the call and every output of the steps that follow must be identical, on two
calls in a row that share the device's fixed buffer, the second one smaller."""
import numpy as np
import pytest

from paper_2411_10666_amd.synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _state(sam, torch, batch, B):
    i32 = dict(dtype=torch.int32, device="cuda:0")
    cur = [torch.empty(B, **i32) for _ in range(4)]
    siz = [torch.empty(B, **i32) for _ in range(3)]
    sam.sam_batch_debug(batch, *cur)
    sam.sam_batch_sizes(batch, *siz)
    torch.cuda.synchronize()
    return np.stack([c.cpu().numpy() for c in cur + siz], axis=1)


def _steps(sam, torch, batch, acc, cnt, L):
    S, B = cnt.shape
    i32 = dict(dtype=torch.int32, device="cuda:0")
    ml = torch.empty(B, **i32); dl = torch.empty(B, **i32); src = torch.empty(B, **i32)
    dr = torch.empty(B, L, **i32)
    out = []
    for s in range(S):
        sam.sam_batch_step(batch, acc[s], cnt[s], ml, dr, dl, src)
        torch.cuda.synchronize()
        out.append((ml.cpu().numpy(), dl.cpu().numpy(), src.cpu().numpy(), dr.cpu().numpy(),
                    _state(sam, torch, batch, B)))
    return out


def _both_ways(sam, torch, corpus, spec, w, B, steps, first_call=False):
    """Init + `steps` steps with each entry point on the first B sequences -> the two records."""
    dev = torch.device("cuda:0")
    prompts = [w.prompts[b] for b in range(B)]
    offs = np.zeros(B + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(p) for p in prompts])
    d_tok = torch.from_numpy(np.concatenate(prompts).astype(np.int32)).to(dev)
    d_off = torch.from_numpy(offs).to(dev)
    acc = torch.from_numpy(np.ascontiguousarray(w.accepted[:steps, :B])).to(dev)
    cnt = torch.from_numpy(np.ascontiguousarray(w.counts[:steps, :B])).to(dev)
    T, A, L = spec.max_seq_len, spec.max_accept, spec.draft_len
    print("[noalloc] B=%d T=%d A=%d L=%d steps=%d static=%s" % (B, T, A, L, steps, corpus is not None),
          flush=True)

    ref = sam.sam_batch_init(corpus, d_tok, d_off, B, spec.vocab, T, A, L, spec.l_bias)
    r0 = _state(sam, torch, ref, B)
    r = _steps(sam, torch, ref, acc, cnt, L)
    assert sam.sam_batch_status(ref) == 0

    free_before = torch.cuda.mem_get_info()[0]
    nb = sam.sam_batch_init_noalloc(corpus, d_tok, d_off, offs, B, spec.vocab, T, A, L, spec.l_bias)
    # (sam_build has already looked the fixed buffer up; a very first lookup makes the
    # runtime load the part of the device code that holds it)
    assert first_call or torch.cuda.mem_get_info()[0] == free_before, "the call took device memory"
    assert 0 < sam.sam_batch_info(nb) <= sam.NOALLOC_MAX_BYTES
    # one batch per device at a time
    with pytest.raises(sam.SamError) as ei:
        sam.sam_batch_init_noalloc(corpus, d_tok, d_off, offs, B, spec.vocab, T, A, L, spec.l_bias)
    assert ei.value.code == sam.SAM_EINVAL and "in use" in str(ei.value)
    g0 = _state(sam, torch, nb, B)
    g = _steps(sam, torch, nb, acc, cnt, L)
    assert sam.sam_batch_status(nb) == 0
    del nb                                   # sam_batch_free: the buffer is free again
    assert np.array_equal(g0, r0), "state after init differs"
    for s, (a, b) in enumerate(zip(g, r)):
        for x, y, name in zip(a, b, ("match_len", "draft_len", "source", "draft", "state")):
            assert np.array_equal(x, y), "step %d: %s differs" % (s, name)
    return r


def test_noalloc_init_matches_init_twice_in_a_row():
    import torch
    from paper_2411_10666_amd import binding as sam
    spec = CONFIGS["cfg1"].scaled(corpus_tokens=60_000, batch=12, prompt_len=200, gen_len=300)
    w = make_workload(spec)
    corpus = sam.sam_build(w.corpus, spec.vocab)
    r1 = _both_ways(sam, torch, corpus, spec, w, 12, 40)
    assert sum(int((x[2] == 2).sum()) for x in r1) > 0 and sum(int((x[2] == 1).sum()) for x in r1) > 0
    # second call: fewer and shorter sequences in the same buffer, which still holds
    # the tables of the first
    spec2 = CONFIGS["cfg1"].scaled(corpus_tokens=60_000, batch=5, prompt_len=70, gen_len=120)
    w2 = make_workload(spec2)
    _both_ways(sam, torch, corpus, spec2, w2, 5, 25)
    # and without a corpus automaton
    spec3 = CONFIGS["cfg4"].scaled(batch=3, prompt_len=150, gen_len=100)
    w3 = make_workload(spec3)
    _both_ways(sam, torch, None, spec3, w3, 3, 12)


def test_noalloc_init_refuses_sizes_beyond_the_buffer():
    import torch
    from paper_2411_10666_amd import binding as sam
    dev = torch.device("cuda:0")
    B, T = 64, 16000                        # about 70 MB of tables
    offs = np.zeros(B + 1, dtype=np.int64)
    d_tok = torch.zeros(1, dtype=torch.int32, device=dev)
    d_off = torch.from_numpy(offs).to(dev)
    with pytest.raises(sam.SamError) as ei:
        sam.sam_batch_init_noalloc(None, d_tok, d_off, offs, B, 100, T, 4, 8)
    assert ei.value.code == sam.SAM_EINVAL and "fixed buffer" in str(ei.value)
    # the refusal left the buffer free
    b = sam.sam_batch_init_noalloc(None, d_tok, d_off[:3].contiguous(), offs[:3], 2, 100, 64, 4, 8)
    assert sam.sam_batch_status(b) == 0
    # bad host offsets are argument errors
    del b
    bad = offs[:3].copy(); bad[1] = 100
    with pytest.raises(sam.SamError) as ei:
        sam.sam_batch_init_noalloc(None, d_tok, d_off[:3].contiguous(), bad, 2, 100, 64, 4, 8)
    assert ei.value.code in (sam.SAM_EINVAL, sam.SAM_ECAPACITY)
