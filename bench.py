#!/usr/bin/env python3
"""Benchmark of the batched suffix-automaton draft path on one MI355X.

A "step" is one ``sam_batch_step`` call over the whole batch: for every sequence
the accepted tokens go through the static Transfer and the dynamic Expand, then
source selection and the draft gather (one kernel launch).  The workload is a
seeded synthetic one (``paper_2411_10666_amd.synth``); the corpus automaton is
built and the prompts are ingested before the clock starts, and all inputs and
outputs of the timed steps are already resident in device memory.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5]

The default workload is the largest of the five benchmark configurations (500 M-token
corpus, vocabulary 128256, 1024 sequences); building its corpus automaton on the host
takes a few minutes, during which progress lines go to stderr.

Prints one JSON line.  ``value`` is match-steps per second (one match-step = one
accepted token of one sequence pushed through both automata).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2411_10666_amd.synth import CONFIGS, make_workload  # noqa: E402

HBM_PEAK_GBPS = 8000.0
HOST_THREADS = 16          # upper limit of worker threads of the CPU leg

# Algorithmic bytes one match-step moves, per workload: the operation counts of
# the method (probes, suffix-link reads, inserts, redirects, clone copies, state
# writes, text appends) and the draft gather, each priced at the element size of
# the device layout (16 B per probe, record read, insert, redirect and state write,
# 32 B per copied transition, 8 B per token, 8 B per draft token, 16 B of per-sequence
# step inputs/outputs).  Computed by oracle/count_ops.py.
# Split into the walk (Transfer and Expand: random accesses) and the gather (draft read
# and write, step inputs and outputs: streaming).  "corpus": the corpus the counts were
# taken on (tokens; the static probe and suffix-link counts depend mildly on it).
ALGO_BYTES_PER_MATCH_STEP = {
    "cfg1": {"walk": 203.7, "gather": 32.1, "corpus": 100_000},
    "cfg2": {"walk": 211.1, "gather": 34.0, "corpus": 10_000_000},
    "cfg3": {"walk": 206.8, "gather": 34.2, "corpus": 100_000_000},
    "cfg4": {"walk": 249.6, "gather": 33.8, "corpus": 0},
    # (counted once, apart from the benchmark runs: the checker's automaton of the whole
    # 500 M-token corpus takes 8 minutes and 100 GB of host memory to build)
    "cfg5": {"walk": 207.0, "gather": 34.5, "corpus": 500_000_000},
}


# HBM bytes of sam_feed_kernel per match-step from rocprofv3 counter runs over a whole
# schedule (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a
# copy kernel of known size; per launch = this figure x the launch's match-steps), with
# the digest of the kernel sources they were taken on: the figure is reported only
# while those sources are unchanged.
MEASURED_TRAFFIC = {
    # config 5, all 519 step launches of one schedule pass (8081.5 match-steps per launch):
    # FETCH_SIZE mean 4145.76, WRITE_SIZE mean 995.16; the same counters read 131089.00
    # and 262144.00 for a copy kernel that reads and writes 262144 KiB, i.e. 2.000 and
    # 1.000 KiB per count: (4145.76 x 2.000 + 995.16) KiB = 9.510 MB per launch
    "cfg5": {"bytes_per_match_step": 1176.7, "sources": "c150325d700c1347"},
    # config 3, 673 launches (1558.1 match-steps each): FETCH_SIZE 938.57 x 2.000 +
    # WRITE_SIZE 204.75 x 1.000 KiB = 2.132 MB per launch
    "cfg3": {"bytes_per_match_step": 1368.3, "sources": "c150325d700c1347"},
    # config 4 (no corpus), 273 launches (7681.9 match-steps each): 2537.59 x 2.000 +
    # 1011.09 x 1.000 KiB = 6.232 MB per launch
    "cfg4": {"bytes_per_match_step": 811.3, "sources": "c150325d700c1347"},
}

KERNEL_SOURCES = ["sam_kernels.hip", "sam_layout.h", "sam_device.h"]


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2411_10666_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(name, match_steps_per_launch):
    """HBM bytes per launch, or None if never measured or measured on other kernels."""
    m = MEASURED_TRAFFIC.get(name)
    if not m or m["sources"] != kernel_sources_digest():
        return None
    return m["bytes_per_match_step"] * match_steps_per_launch


def _log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def gpu_leg(w, steps, warmup, tree=None, replay=True, before_timing=None):
    import torch
    from paper_2411_10666_amd import binding as sam

    spec = w.spec
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    t0 = time.time()
    said = [t0]

    def progress(phase, done, total):       # a line now and then during long builds
        if time.time() - said[0] > 20.0:
            said[0] = time.time()
            _log("corpus build, %s: %d of %d" % (phase, done, total))

    sam.sam_set_progress_callback(progress)
    try:
        corpus = sam.sam_build(w.corpus, spec.vocab) if w.corpus is not None else None
    finally:
        sam.sam_set_progress_callback(None)
    build_s = time.time() - t0
    info = sam.sam_corpus_info(corpus) if corpus is not None else (0, 0, 0)
    _log("corpus automaton: %d states, %d transitions, %.1f MB on device, built in %.1f s"
         % (info[0], info[1], info[2] / 1e6, build_s))

    if before_timing is not None:
        before_timing()        # host work started earlier must be over before anything is timed
    B, A, L = spec.batch, spec.max_accept, spec.draft_len
    S = w.steps
    d_prompts = torch.from_numpy(w.prompts.reshape(-1)).to(dev)
    d_offs = torch.from_numpy(w.prompt_offsets).to(dev)
    d_acc = torch.from_numpy(w.accepted).to(dev)
    d_cnt = torch.from_numpy(w.counts).to(dev)
    i32 = dict(dtype=torch.int32, device=dev)
    ml = torch.zeros(S, B, **i32)
    dl = torch.zeros(S, B, **i32)
    src = torch.zeros(S, B, **i32)
    dr = torch.zeros(S, B, L, **i32)
    stream = torch.cuda.current_stream()

    def new_batch():
        torch.cuda.synchronize()
        t = time.time()
        b = sam.sam_batch_init(corpus, d_prompts, d_offs, B, spec.vocab, spec.max_seq_len, A, L,
                               spec.l_bias, stream)
        torch.cuda.synchronize()
        dt = time.time() - t
        b.plan = sam.StepPlan(b, d_acc, d_cnt, ml, dr, dl, src, stream)
        return b, dt

    def run(batch, lo, hi):
        batch.plan.run(lo, hi)

    # The schedule is replayed from its start as often as needed; each replay
    # starts from freshly ingested prompts (untimed).
    batch, init_s = new_batch()
    pos = 0
    left = warmup
    while left > 0:
        n = min(left, S - pos)
        run(batch, pos, pos + n)
        pos += n
        left -= n
        if pos == S:
            batch, _ = new_batch()
            pos = 0
    torch.cuda.synchronize()

    segs = []
    timed_match_steps = 0
    timed_draft_tokens = 0
    wall = 0.0
    left = steps
    while left > 0:
        if pos == S:
            batch, _ = new_batch()
            pos = 0
        n = min(left, S - pos)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t = time.perf_counter()
        e0.record(stream)
        run(batch, pos, pos + n)
        e1.record(stream)
        torch.cuda.synchronize()
        wall += time.perf_counter() - t
        segs.append((e0, e1))
        timed_match_steps += int(w.counts[pos:pos + n].sum())
        timed_draft_tokens += int(dl[pos:pos + n].sum().item())
        pos += n
        left -= n
    ev_ms = sum(a.elapsed_time(b) for a, b in segs)
    status = sam.sam_batch_status(batch)
    if status != 0:
        raise RuntimeError("device status word is %d after the timed steps" % status)
    if timed_draft_tokens <= 0:
        raise RuntimeError("no draft tokens were produced")
    # Upper bound, reported beside the main metric and clearly apart from it: the
    # whole schedule in ONE launch (no launch gaps, no sequence waits for another's
    # longest row).  Not how a serving loop calls the library.
    replay_out = None
    if replay:
        best = None
        for _ in range(3):
            rb, _ = new_batch()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            sam.sam_batch_replay(rb, d_acc, d_cnt, ml, dr, dl, src, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
            if sam.sam_batch_status(rb) != 0:
                raise RuntimeError("device status word is not 0 after the replay")
        total = int(w.counts.sum())
        replay_out = {"steps": S, "ms": best, "match_steps_per_s": total / (best * 1e-3),
                      "draft_tokens_per_s": int(dl.sum().item()) / (best * 1e-3)}

    tree_out = None
    if tree and corpus is not None:
        # Tree drafts (Algorithms 3 and 4) from the state the timed steps ended in;
        # reported beside the main metric, not part of it.
        k, max_size = tree
        t = time.time()
        sam.sam_corpus_build_topk(corpus, k)
        topk_s = time.time() - t
        tt = torch.empty(B, max_size, **i32)
        tp = torch.empty(B, max_size, **i32)
        tpr = torch.empty(B, max_size, dtype=torch.float32, device=dev)
        ts = torch.empty(B, **i32)
        for _ in range(20):
            sam.sam_batch_tree_draft(batch, max_size, tt, tp, tpr, ts, stream)
        torch.cuda.synchronize()
        calls = 500
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(calls):
            sam.sam_batch_tree_draft(batch, max_size, tt, tp, tpr, ts, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms_warm = e0.elapsed_time(e1) / calls
        # The figure that counts: every call on cursor states it has not seen (one step of
        # the schedule between two calls moves every sequence on), so the table rows come
        # from HBM, not from the caches a repeated call would find them in.
        fb, _ = new_batch()
        n_fresh = min(200, S)
        evs = []
        for i in range(n_fresh):
            run(fb, i, i + 1)
            a = torch.cuda.Event(enable_timing=True)
            b_ = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            sam.sam_batch_tree_draft(fb, max_size, tt, tp, tpr, ts, stream)
            b_.record(stream)
            evs.append((a, b_))
        torch.cuda.synchronize()
        ms = sum(a.elapsed_time(b_) for a, b_ in evs) / n_fresh
        entries = int(ts.sum().item())           # of the last call; drafts nearly always fill up
        # dependent-load floor: the pops of one draft are a chain of table reads
        tree_out = {"k": k, "max_size": max_size, "ms_per_call": ms,
                    "ms_per_call_same_states_repeated": ms_warm, "calls": n_fresh,
                    "entries_per_call": entries, "entries_per_s": entries / (ms * 1e-3),
                    "us_per_entry_of_one_draft": ms * 1e3 / max(1.0, entries / B),
                    "topk_build_s": topk_s,
                    # per entry: one k x 12 B table read and 12 B of output
                    "algo_gbps": entries * (12.0 * k + 12.0) / (ms * 1e-3) / 1e9}
    return dict(tree=tree_out, replay=replay_out, wall_s=wall, event_ms=ev_ms, match_steps=timed_match_steps,
                draft_tokens=timed_draft_tokens, init_s=init_s, build_s=build_s,
                states=info[0], trans=info[1], static_bytes=info[2],
                batch_bytes=sam.sam_batch_info(batch))


# The checker's corpus automaton is built inside the benchmark run: 1 minute for 100 M
# tokens, 8 minutes for 500 M.  Corpora beyond this many tokens are cut for the CPU leg
# (stated in its "sample" text); all smaller ones are used whole.
CPU_CORPUS_LIMIT = 100_000_000


class CpuCorpus:
    """The checker's own corpus automaton, built on a host thread of its own while the
    library builds its one (two foreign calls that release the interpreter lock); it is
    waited for before anything is timed."""

    def __init__(self, w):
        import threading
        self.corpus, self.note, self.static, self.build_s, self.error = w.corpus, "", None, 0.0, None
        if self.corpus is not None and len(self.corpus) > CPU_CORPUS_LIMIT:
            self.corpus = self.corpus[:CPU_CORPUS_LIMIT]
            self.note = ("; corpus CUT to its first %d of %d tokens (the checker needs 8 minutes "
                         "to build the whole one)" % (CPU_CORPUS_LIMIT, len(w.corpus)))
        self._thread = threading.Thread(target=self._build, daemon=True)
        self._thread.start()

    def _build(self):
        from oracle.sam_oracle import Sam
        t0 = time.time()
        said = [t0]

        def progress(done, total):
            if time.time() - said[0] > 20.0:
                said[0] = time.time()
                _log("CPU checker, corpus build: %d of %d" % (done, total))

        try:
            if self.corpus is not None:
                self.static = Sam.build(self.corpus, progress=progress)
        except BaseException as e:      # reported by wait()
            self.error = e
        self.build_s = time.time() - t0

    def wait(self):
        self._thread.join()
        if self.error is not None:
            raise self.error


def cpu_leg(w, cc):
    """The CPU checker as it stands, timed on the steps only: once on one thread and
    once with the sequences dealt out to the host's cores (the reported value)."""
    from oracle.sam_oracle import Batch
    spec = w.spec
    cc.wait()
    corpus, static, note, build_s = cc.corpus, cc.static, cc.note, cc.build_s
    nb = min(spec.batch, 256)
    ob = Batch(static, corpus, [w.prompts[b] for b in range(nb)], spec.max_accept,
               spec.draft_len, spec.l_bias)
    acc = np.ascontiguousarray(w.accepted[:, :nb])
    cnt = np.ascontiguousarray(w.counts[:, :nb])
    t0 = time.perf_counter()
    for s in range(w.steps):
        ob.step(acc[s], cnt[s])
    dt = time.perf_counter() - t0
    ms = int(cnt.sum())
    one = dict(value=ms / dt, unit="match-steps/s", cores=1)
    out = dict(value=ms / dt, unit="match-steps/s", cores=1, kind="oracle",
               sample="%d of %d sequences, whole %d-step schedule (%d match-steps); "
                      "corpus build (%.1f s) and prompt ingest not timed%s"
                      % (nb, spec.batch, w.steps, ms, build_s, note),
               corpus_tokens=0 if corpus is None else int(len(corpus)))
    # The same work once more with the sequences dealt out to one thread per host
    # core (the checker itself is unchanged: its calls release the interpreter lock
    # and share the read-only corpus automaton).
    threads = max(1, min(nb, HOST_THREADS, os.cpu_count() or 1))
    if threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        del ob
        groups = [list(range(t, nb, threads)) for t in range(threads)]
        parts = [(Batch(static, corpus, [w.prompts[b] for b in g], spec.max_accept,
                        spec.draft_len, spec.l_bias),
                  np.ascontiguousarray(acc[:, g]), np.ascontiguousarray(cnt[:, g]))
                 for g in groups]

        def work(part):
            b, a, c = part
            b.run(a, c)       # the same steps, looped inside one foreign call

        with ThreadPoolExecutor(threads) as pool:
            t0 = time.perf_counter()
            list(pool.map(work, parts))
            dt = time.perf_counter() - t0
        out["value"], out["cores"] = ms / dt, threads
        out["one_core"] = one
    return out


def memory_leg(table_bytes):
    """What the device's memory system gives for the path's access patterns."""
    from paper_2411_10666_amd import binding as sam
    chase = {name: sam.sam_membench(sam.MEMBENCH_CHASE, size, hops)
             for name, size, hops in (("l2_1MiB", 1 << 20, 20000), ("mall_64MiB", 64 << 20, 20000),
                                      ("hbm_4GiB", 4 << 30, 20000))}
    table = 4096
    while table < max(table_bytes, 1 << 30):
        table *= 2
    return {
        "dependent_line_load_ns": chase,
        "random_16B_reads_per_s": sam.sam_membench(sam.MEMBENCH_GATHER, table, 256, 16384),
        "random_read_table_bytes": table,
        "copy_bytes_per_s": sam.sam_membench(sam.MEMBENCH_COPY, 1 << 30),
        "empty_launch_us": sam.sam_membench(sam.MEMBENCH_LAUNCH, 0, 2000, 64),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="cfg5", choices=sorted(CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-memory-system", action="store_true",
                    help="skip the memory-system measurements (memory_system, latency_bound)")
    ap.add_argument("--tree-draft", default="",
                    help="K,MAX_SIZE: also time sam_batch_tree_draft (reported as tree_draft)")
    ap.add_argument("--library-mode", type=int, default=0,
                    help="sam_set_layout_override mode for the batches of this run (a testing "
                         "and measuring aid, e.g. 32: step kernel without its scout waves)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the timed "
                         "steps (a kernel of known traffic to scale profiler counters by)")

    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (sequences are independent and "
              "would be sharded without communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be >= 1 and --warmup >= 0", file=sys.stderr)
        sys.exit(2)

    spec = CONFIGS[args.config]
    t0 = time.time()
    w = make_workload(spec)
    _log("%s: corpus %d tokens, batch %d, %d+%d tokens per sequence, %d steps in the schedule "
         "(generated in %.1f s)" % (spec.name, spec.corpus_tokens, spec.batch, spec.prompt_len,
                                    spec.gen_len, w.steps, time.time() - t0))
    if args.copy_probe_mib > 0:
        import torch
        n = args.copy_probe_mib * (1 << 20) // 4
        src_t = torch.ones(n, dtype=torch.int32, device="cuda:0")
        dst_t = torch.empty_like(src_t)
        torch.cuda.synchronize()
        dst_t.copy_(src_t)
        torch.cuda.synchronize()
        _log("copy probe: %d MiB read + %d MiB written by one copy kernel"
             % (args.copy_probe_mib, args.copy_probe_mib))
        del src_t, dst_t
    tree = tuple(int(v) for v in args.tree_draft.split(",")) if args.tree_draft else None
    if args.library_mode:
        from paper_2411_10666_amd import binding as sam
        sam.sam_set_layout_override(args.library_mode)
        _log("library mode %d" % args.library_mode)
    cc = None if args.no_cpu_baseline else CpuCorpus(w)
    g = gpu_leg(w, args.steps, args.warmup, tree, before_timing=cc.wait if cc else None)

    # one clock for everything: HIP events on the stream the steps are launched on
    per_step_ms = g["event_ms"] / args.steps
    value = g["match_steps"] / (g["event_ms"] * 1e-3)
    ab = ALGO_BYTES_PER_MATCH_STEP[spec.name]
    per_launch = g["match_steps"] / args.steps
    walk_bytes_per_launch = ab["walk"] * per_launch
    gather_bytes_per_launch = ab["gather"] * per_launch
    algo_bytes_per_launch = walk_bytes_per_launch + gather_bytes_per_launch
    achieved = algo_bytes_per_launch / (per_step_ms * 1e-3) / 1e9
    out = {
        "metric": "SAM match-steps/sec + draft tokens/sec (1 GPU), % of HBM roofline",
        "value": value,
        "unit": "match-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": per_step_ms,
        "host_wall_ms_per_step": g["wall_s"] * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {
            "workload": spec.name,
            "corpus_tokens": spec.corpus_tokens,
            "vocab": spec.vocab,
            "batch": spec.batch,
            "prompt_len": spec.prompt_len,
            "gen_len": spec.gen_len,
            "max_accept": spec.max_accept,
            "draft_len": spec.draft_len,
            "l_bias": spec.l_bias,
            "seed": spec.seed,
            **({"library_mode": args.library_mode} if args.library_mode else {}),
        },
        "draft_tokens_per_s": g["draft_tokens"] / (g["event_ms"] * 1e-3),
        "sequence_steps_per_s": spec.batch * args.steps / (g["event_ms"] * 1e-3),
        "match_steps_timed": g["match_steps"],
        "prompt_ingest_tokens_per_s": spec.batch * spec.prompt_len / g["init_s"],
        "corpus_build_s": g["build_s"],
        "device_bytes": {"static": g["static_bytes"], "batch": g["batch_bytes"]},
        "roofline": {
            "bound": "hbm",
            "kernel": "sam_feed_kernel",
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": measured_traffic(spec.name, per_launch),
            "algo_bytes_per_launch": algo_bytes_per_launch,
            "walk_bytes_per_launch": walk_bytes_per_launch,
            "gather_bytes_per_launch": gather_bytes_per_launch,
            "algo_bytes_counted_on_corpus_tokens": ab["corpus"],
            "avg_launch_ms": per_step_ms,
        },
    }
    if not args.no_memory_system:
        m = memory_leg(g["static_bytes"])
        out["memory_system"] = m
        # Little's law: each walking wavefront has one dependent line load in flight
        # (two wavefronts per sequence, one when there is no corpus automaton).
        chains = spec.batch * (2 if w.corpus is not None else 1)
        r = out["roofline"]
        traffic = r["traffic"]
        sec = per_step_ms * 1e-3
        all_hbm = chains / (m["dependent_line_load_ns"]["hbm_4GiB"] * 1e-9)
        fetched = None if traffic is None else traffic / 128.0 / sec
        # The two rooflines of the path, each against what this device was measured to
        # deliver in the same run: the walk's 16-byte accesses against independent random
        # 16-byte reads from a table the size of the corpus automaton, the gather's bytes
        # against a device copy; and the walk's accesses (measured line fetches where the
        # counters are current) against what the dependent chains could fetch if every
        # access were an HBM miss.
        r["frac_random_access"] = (walk_bytes_per_launch / 16.0 / sec) / m["random_16B_reads_per_s"]
        r["frac_streaming"] = (gather_bytes_per_launch / sec) / m["copy_bytes_per_s"]
        r["frac_latency_bound"] = ((walk_bytes_per_launch / 16.0 / sec) if fetched is None
                                   else fetched) / all_hbm
        out["latency_bound"] = {
            "chains_in_flight": chains,
            "line_loads_per_s_all_hbm": all_hbm,
            "line_loads_per_s_all_l2": chains / (m["dependent_line_load_ns"]["l2_1MiB"] * 1e-9),
            "measured_hbm_line_fetches_per_s": fetched,
            "algorithmic_accesses_per_s": walk_bytes_per_launch / 16.0 / sec,
        }
    if g["replay"]:
        out["single_launch_replay"] = g["replay"]
    if g["tree"]:
        out["tree_draft"] = g["tree"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_leg(w, cc)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
