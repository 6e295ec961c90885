#!/usr/bin/env python3
"""Benchmark of the MI355X LightLDA hot path: tokens/s of whole iterations
(alias build + cycle-MH sweep + count rebuild) on a synthetic Zipf corpus,
the roofline figures of the sweep's dominant kernel, and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c1|c4|c5] [--mh-steps M]

Prints ONE JSON line.  One GPU only: --gpus N with N > 1 exits with a message.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def algorithmic_bytes_per_token(mh_steps: int) -> float:
    """Bytes the method touches per token per sweep, counted operand by operand
    (no reuse assumed): token stream 16 B (doc id, position, z in, z out), document
    header 8 B, state at the snapshot topic 16 B (n_kw, n_k, n_kd probe), each word
    step 24 B (alias bin 8, n_kw 4, n_k 4, n_kd probe 8), each doc step 20 B
    (z of a random token 4, n_kw 4, n_k 4, n_kd probe 8): 40 + 22 m for m steps."""
    return 40.0 + 22.0 * mh_steps


def chain_shape(mh_steps: int):
    """(word steps, doc steps) of a cycle chain that starts with a word step."""
    return (mh_steps + 1) // 2, mh_steps // 2


def doc_pass_bytes_per_token(mh_steps: int) -> float:
    """The doc pass's share of the figure above: token stream 16 B, document header 8 B,
    n_k and the n_kd probe at the snapshot topic 12 B, per word step n_k + n_kd probe
    12 B, per doc step z of a random token + n_k + n_kd probe 16 B (64 B for 2 steps).
    The rest -- every n_kw and the alias bins, 4 + 12 per word step + 4 per doc step --
    is the word pass's share."""
    nw, nd = chain_shape(mh_steps)
    return 36.0 + 12.0 * nw + 16.0 * nd


# HBM-side bytes per launch of the doc pass kernel and of the word pass's gather kernel, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command (profiles/all_kernels_<workload>_mh2.txt:
# counter KiB x calibration factor x 1024, fetched + written); keyed by (workload, mh_steps,
# dense_alias_min_count as passed to the library).  None where not measured.
MEASURED_TRAFFIC_BYTES = {
    ("c3", 2, 10000): {"doc_pass_tiles_kernel": 48.70e9},
    ("c2", 2, 1000): {"doc_pass_tiles_kernel": 6.59e9},
    ("c4", 2, None): {"doc_pass_tiles_kernel": 75.05e9, "word_pass_gather_kernel": 50.33e9},
    ("c5", 2, None): {"doc_pass_tiles_kernel": 92.44e9, "word_pass_gather_kernel": 147.41e9},
}


def cpu_baseline(cfg, doff, words, mh_steps, sample_docs, dense_alias_min_count=0, lazy_rows=False):
    """The oracle as it stands on the first `sample_docs` documents (same V, K).  lazy_rows: the
    oracle counts a word's n_kw row when it first needs it (workloads whose V x K table does
    not fit in host memory)."""
    import oracle
    D = min(sample_docs, len(doff) - 1)
    sdoff = np.ascontiguousarray(doff[: D + 1])
    swords = np.ascontiguousarray(words[: int(sdoff[-1])])
    o = oracle.Oracle(sdoff, swords, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                      dense_alias_min_count=dense_alias_min_count, lazy_alias=True,
                      lazy_rows=lazy_rows)
    t0 = time.perf_counter()
    o.build_alias()
    o.sweep(mh_steps)
    o.rebuild_counts()
    dt = time.perf_counter() - t0
    n = o.N
    o.close()
    return {
        "value": n / dt, "unit": "tokens/s", "cores": 1, "host_cores": os.cpu_count(),
        "kind": "oracle",
        "sample": "first %d documents (%d tokens) of the same corpus, same V and K; one full "
                  "iteration (alias tables of the words that occur, sweep, recount) on 1 of the "
                  "host's %d cores, %.1f s" % (D, n, os.cpu_count(), dt),
    }


CPU_SAMPLE_DOCS = {"c1": 1000, "c2": 60000, "c3": 600000, "c4": 10000, "c5": 1000}


def store_options(workload, cfg, words, dense_alias_min_count):
    """lda_options of a workload and a description of its n_kw store.  c4: dense rows for the
    head words; c5: no dense row; every word without a dense row draws from the mixture.
    c1-c3: dense rows, and the mixture below `dense_alias_min_count` tokens (-1: K; 0: a dense
    table for every word)."""
    if workload in ("c4", "c5"):
        dense_rows = cfg.dense_rows if workload == "c4" else -1
        cnt = np.bincount(words, minlength=cfg.V)
        tail = cnt[max(dense_rows, 0):]
        # dense K-bin tables only for words with at least K tokens (rows that can be dense)
        opts = dict(dense_rows=dense_rows, dense_alias_min_count=max(int(tail.max()) + 1, cfg.K))
        return opts, "hybrid n_kw (%s dense rows), mixture proposal below count %d" % (
            max(dense_rows, 0), opts["dense_alias_min_count"])
    if dense_alias_min_count != 0:
        min_count = cfg.K if dense_alias_min_count < 0 else dense_alias_min_count
        return dict(dense_rows=0, dense_alias_min_count=min_count), \
            "dense n_kw, mixture proposal below count %d" % min_count
    return {}, "dense n_kw"


def run_leg(workload, mh_steps, steps, warmup, dense_alias_min_count, corpora, stream_block_tokens=0):
    """One more leg of the metric, timed like the headline: mean over `steps` iterations.
    stream_block_tokens > 0: the corpus streamed from pinned host memory in blocks."""
    import torch
    from paper_1412_1576_amd import corpus, lda
    cfg = corpus.CONFIGS[workload]
    if workload not in corpora:
        corpora[workload] = corpus.make_corpus(cfg)
    doff, words = corpora[workload]
    N = int(doff[-1])
    opts, store = store_options(workload, cfg, words, dense_alias_min_count)
    stream = torch.cuda.Stream()
    g = lda.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                stream=stream.cuda_stream, stream_block_tokens=stream_block_tokens, **opts)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for it in range(warmup + steps):
        e = ev[it - warmup] if it >= warmup else None
        if e:
            e[0].record(stream)
        g.build_alias()
        if e:
            e[1].record(stream)
        g.sweep(mh_steps)
        if e:
            e[2].record(stream)
        g.rebuild_counts()
        if e:
            e[3].record(stream)
    g.sync()
    torch.cuda.synchronize()
    assert int(g.get_nk().sum()) == N, "count invariant violated"
    g.close()
    mean = lambda a, b: sum(e[a].elapsed_time(e[b]) for e in ev) / steps
    step_ms, sweep_ms = mean(0, 3), mean(1, 2)
    if stream_block_tokens:
        store += "; streamed from pinned host memory in blocks of %d tokens" % stream_block_tokens
    return {
        "workload": "%s: N=%d tokens, V=%d, K=%d, mh_steps=%d, %s" % (cfg.name, N, cfg.V, cfg.K,
                                                                      mh_steps, store),
        "steps": steps, "warmup": warmup,
        "ms_per_step": step_ms, "tokens_per_s": N / (step_ms * 1e-3),
        "alias_ms": mean(0, 1), "sweep_ms": sweep_ms, "rebuild_ms": mean(2, 3),
        "sweep_tokens_per_s": N / (sweep_ms * 1e-3),
        "sweep_achieved_GBs": algorithmic_bytes_per_token(mh_steps) * N / (sweep_ms * 1e-3) / 1e9,
        "sweep_frac_of_hbm_peak": algorithmic_bytes_per_token(mh_steps) * N / (sweep_ms * 1e-3) / 1e9
                                  / HBM_PEAK_GBS,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--mh-steps", type=int, default=2)
    ap.add_argument("--docs", type=int, default=0, help="use only the first DOCS documents' worth "
                    "of the workload (debugging; the result is then not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-legs", action="store_true", help="skip the other legs of the "
                    "metric (c2, c4, c3 at 4 steps, c3 with a dense table for every word) that a "
                    "default run times after the headline workload")
    ap.add_argument("--cpu-sample-docs", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true", help="also launch a plain "
                    "elementwise kernel that reads 1 GiB and writes 1 GiB (scale for HBM counters)")
    ap.add_argument("--chunk-tokens", type=int, default=0)
    ap.add_argument("--block-threads", type=int, default=0)
    ap.add_argument("--tile-tokens", type=int, default=0)
    ap.add_argument("--record-bucket-tokens", type=int, default=0, help="order of the records the "
                    "sweep's passes exchange (lda_options.record_bucket_tokens); 0: default")
    ap.add_argument("--stream-block-tokens", type=int, default=0, help="stream the corpus from "
                    "pinned host memory in blocks of this many tokens (lda_options)")
    ap.add_argument("--dense-alias-min-count", type=int, default=-1, help="c1-c3: words with "
                    "fewer tokens draw from the sparsified mixture word-proposal (Sec. 4.2) "
                    "instead of a dense K-bin table; -1 (default) = K; 0 = dense tables for "
                    "every word")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU sharding is a "
              "design note, not code", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1412_1576_amd import corpus, lda
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    cfg = corpus.CONFIGS[args.workload]
    if args.docs:
        cfg = corpus.scaled(cfg, D=args.docs)
    t0 = time.perf_counter()
    doff, words = corpus.make_corpus(cfg)
    t_gen = time.perf_counter() - t0
    N = int(doff[-1])

    hybrid, store = store_options(args.workload, cfg, words, args.dense_alias_min_count)

    stream = torch.cuda.Stream()
    t0 = time.perf_counter()
    g = lda.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                stream=stream.cuda_stream, sweep_chunk_tokens=args.chunk_tokens,
                sweep_block_threads=args.block_threads, rebuild_tile_tokens=args.tile_tokens,
                time_sweep_passes=1, record_bucket_tokens=args.record_bucket_tokens,
                stream_block_tokens=args.stream_block_tokens, **hybrid)
    g.sync()
    t_init = time.perf_counter() - t0

    pass_ms = []  # (word pass, doc pass kernel) of every timed sweep, from the library's events

    def iteration(evs=None):
        if evs:
            evs[0].record(stream)
        g.build_alias()
        if evs:
            evs[1].record(stream)
        g.sweep(args.mh_steps)
        if evs:
            evs[2].record(stream)
        g.rebuild_counts()
        if evs:
            evs[3].record(stream)
            try:
                pass_ms.append(g.sweep_pass_ms())
            except lda.LdaError:   # this chain shape runs as one fused kernel
                pass

    for _ in range(args.warmup):
        iteration()
    g.sync()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)   # one kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        # the same kernel timed: what a plain streaming copy reaches on this device
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(10):
            torch.add(src, 1.0, out=dst)
        c1.record()
        torch.cuda.synchronize()
        copy_gbs = 10 * 2.0 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
        del src, dst

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    w0 = time.perf_counter()
    start.record(stream)
    for s in range(args.steps):
        iteration(evs[s])
    stop.record(stream)
    g.sync()
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    total_ms = start.elapsed_time(stop)
    alias_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    sweep_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    rebuild_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    loglik = g.loglik()[0]
    nk = g.get_nk()
    assert int(nk.sum()) == N, "count invariant violated"

    ms_per_step = total_ms / args.steps
    abytes = algorithmic_bytes_per_token(args.mh_steps)
    dom_ms = sweep_ms
    if len(pass_ms) == args.steps:
        word_ms = sum(p[0] for p in pass_ms) / args.steps
        doc_ms = sum(p[1] for p in pass_ms) / args.steps
        dominant, dbytes, dom_ms = "doc_pass_tiles_kernel", doc_pass_bytes_per_token(args.mh_steps), doc_ms
        if args.workload in ("c4", "c5") and word_ms > doc_ms:
            # every token of these stores goes through the one gather kernel of the word pass
            dominant, dbytes, dom_ms = "word_pass_gather_kernel", abytes - dbytes, word_ms
    else:
        word_ms, doc_ms = None, sweep_ms
        dominant, dbytes = "sweep_tiles_kernel", abytes
    achieved = dbytes * N / (dom_ms * 1e-3) / 1e9
    out = {
        "metric": "sampled tokens/sec (alias build + %d-step MH sweep + count rebuild)" % args.mh_steps,
        "value": N / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32 counts, fp64 acceptance",
        "data": "synthetic",
        "config": {
            "workload": "%s: D=%d docs, N=%d tokens, V=%d Zipf(%.2f), K=%d, alpha=%g, beta=%g, "
                        "mh_steps=%d, %s" % (cfg.name, cfg.D, N, cfg.V, cfg.s, cfg.K,
                                             cfg.alpha, cfg.beta, args.mh_steps, store),
            "sweep_tokens_per_s": N / (sweep_ms * 1e-3),
            "alias_ms": alias_ms, "sweep_ms": sweep_ms, "rebuild_ms": rebuild_ms,
            "word_pass_ms": word_ms, "doc_pass_kernel_ms": doc_ms,
            "sweep_algorithmic_bytes_per_token": abytes,
            "sweep_achieved_GBs": abytes * N / (sweep_ms * 1e-3) / 1e9,
            "wall_s_timed_region": wall, "corpus_gen_s": t_gen, "init_s": t_init,
            "loglik_after": loglik,
        },
        "roofline": {
            "bound": "hbm", "kernel": dominant,
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "algorithmic_bytes_per_token": dbytes,
            "traffic": MEASURED_TRAFFIC_BYTES.get(
                (cfg.name if not (args.docs or args.stream_block_tokens) else None, args.mh_steps,
                 None if args.workload in ("c4", "c5") else hybrid.get("dense_alias_min_count", 0)),
                {}).get(dominant),
        },
    }
    # the measured HBM-side bytes of the same kernel at this run's kernel time, next to the
    # model figure: what really crossed the memory interface per second
    if out["roofline"]["traffic"] and dom_ms:
        out["roofline"]["traffic_GBs"] = out["roofline"]["traffic"] / (dom_ms * 1e-3) / 1e9
    g.close()
    if args.calibrate_copy:
        out["config"]["streaming_copy_GBs"] = copy_gbs
    if not args.no_other_legs and not args.docs:
        # the other K of the metric and the other forms of the headline workload, timed in the
        # same run: (workload, mh_steps, dense_alias_min_count)
        corpora = {args.workload: (doff, words)}
        legs = [("c2", 2, -1), ("c3", 4, -1), ("c3", 2, 0), ("c4", 2, -1)]
        out["config"]["other_legs"] = [
            run_leg(w, m, max(3, min(args.steps, 10)), 1, dm, corpora)
            for (w, m, dm) in legs if (w, m, dm) != (args.workload, args.mh_steps, args.dense_alias_min_count)]
        # streamed data blocks: the K = 10^6 slice resident and in five blocks of 10^8 tokens from
        # pinned host memory (13 B per token to the device, 4 B back, every sweep)
        res = run_leg("c5", 2, 3, 1, -1, corpora)
        stm = run_leg("c5", 2, 3, 1, -1, corpora, stream_block_tokens=100_000_000)
        n5 = int(corpora["c5"][0][-1])
        # what the host link alone allows: a pinned 1 GiB buffer copied to the device
        pin = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
        dev = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dev.copy_(pin, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(4):
            dev.copy_(pin, non_blocking=True)
        torch.cuda.synchronize()
        h2d_gbs = 4 * (1 << 30) / (time.perf_counter() - t0) / 1e9
        del pin, dev
        load_ms = 13.0 * n5 / h2d_gbs / 1e6
        out["config"]["streamed_blocks"] = {
            "resident": res, "streamed": stm,
            "streamed_over_resident_sweep_time": stm["sweep_ms"] / res["sweep_ms"],
            "streamed_over_resident_iteration_time": stm["ms_per_step"] / res["ms_per_step"],
            "host_link_GBs_during_streamed_sweep": 17.0 * n5 / (stm["sweep_ms"] * 1e-3) / 1e9,
            "host_to_device_GBs_plain_copy": h2d_gbs,
            "load_alone_ms": load_ms,   # 13 B per token at the plain copy's rate
            "overlap_efficiency": load_ms / stm["sweep_ms"],  # 1: the sweep hides behind the loads
        }
        corpora.clear()
    if not args.no_cpu_baseline:
        sample = args.cpu_sample_docs or CPU_SAMPLE_DOCS[args.workload]
        out["cpu_baseline"] = cpu_baseline(cfg, doff, words, args.mh_steps, sample,
                                           hybrid.get("dense_alias_min_count", 0),
                                           lazy_rows=args.workload in ("c4", "c5"))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
