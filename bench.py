#!/usr/bin/env python3
"""Benchmark of the whole hot path (E-step + M-step) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A "step" is one full iteration of Alg. 1 over the synthetic corpus.  The corpus (seeded, generated on
the host, resident in HBM before the timed region) has the shape of the NYTimes-like workload:
D=300K, V=100K, T=100M.  The headline value is tokens/s at K=10,000 (the sparse regime the metric is
quoted on); the same corpus fitted with K=1,000 is reported in "also", and the PubMed-shaped workload
(D=8.2M, V=141K, T=738M, K=5,000) in "also_c4", each with the roofline of its own sampling kernel.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(st, K, z_bytes):
    """HBM bytes the sampling kernel must move for the iterations counted in ``st`` (the model is the list below).

    per token : 4 (document id) + 4 (token index) + 8 (row descriptor) + 2 * z_bytes (the assignment, written in
                canonical order and again in word-major order for CountByVZ)
    per run of consecutive tokens of one (word, document) pair : 4*K_d (the packed row of A, fetched once)
    per (word, chunk) with tokens : the tree level above the bottom and the block bases, 4*n3pad + 8*n3, the
                row total, 4, and the Bhat row: 4*Kpad for a dense row, or 8 (descriptor) + 8 per non-zero of
                the sparse row of a light word
    per iteration : the base vector the light words share, 4*Kpad
    Bhat gathers and the dense branch are served from LDS and count as zero.
    """
    kpad = (K + 63) // 64 * 64
    n3 = kpad // 64
    n3pad = (n3 + 63) // 64 * 64
    it = st["iterations"]
    tok = st["sum_tokens"] * (4 + 4 + 8 + 2 * z_bytes) + 4 * st["sum_row_fetch"]
    tree = 4 * n3pad + 8 * n3 + 4
    dense_rows = st["words_present"] - st["light_words_present"]
    stage = it * (dense_rows * (4 * kpad + tree) + st["light_words_present"] * (8 + tree))
    stage += 8 * st["sum_light_entries"] + (it * 4 * kpad if st["light_words_present"] else 0)
    return tok + stage


def source_digest():
    """Digest of the HIP sources the library is built from: the tag that ties a stored counter figure to the
    kernels it was measured on."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_1610_02496_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(workload, steps, warmup):
    """Bytes beyond L2 per pass of the sampling kernel as `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` counted them
    on this same command (the summary under profiles/ states the command, the calibration and the digest of the
    kernel sources it ran).  The counters cannot be read from inside the process, so the figure is a stored one:
    it is returned only for the command line and the kernel sources it was measured with, otherwise None."""
    path = os.path.join(ROOT, "profiles", "estep_kernel_%s_hbm_traffic.md" % workload)
    try:
        kv = dict(line.split("=", 1) for line in open(path) if "=" in line and line.split("=")[0].strip().isidentifier())
    except OSError:
        return None
    kv = {k.strip(): v.strip() for k, v in kv.items()}
    if kv.get("bench_args") != "--steps %d --warmup %d" % (steps, warmup) or kv.get("source_digest") != source_digest():
        return None
    try:
        return float(kv["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def run_holdout(g, corpus, docs, n_foldin):
    """Holdout log-likelihood by document completion on the model just trained.  The scored documents are a
    prefix of the training corpus standing in for held-out ones (the synthetic corpus has no separate held-out
    part): the figure of interest is the cost of the call, which includes the layout build and upload of the
    documents, ``n_foldin`` fold-in iterations and the scoring pass."""
    docs = min(docs, corpus.spec.D)
    doc_ptr = np.ascontiguousarray(corpus.doc_ptr[: docs + 1])
    T = int(doc_ptr[-1])
    word_ids = np.ascontiguousarray(corpus.word_ids[:T])
    pos = np.arange(T) - np.repeat(doc_ptr[:-1], np.diff(doc_ptr))
    observed = (pos % 2 == 0).astype(np.uint8)
    t0 = time.perf_counter()
    ll, scored, _ = g.holdout_loglik(doc_ptr, word_ids, observed, n_foldin, 12345)
    dt = time.perf_counter() - t0
    n_obs = int(observed.sum())
    return {"documents": docs, "observed_tokens": n_obs, "scored_tokens": scored, "n_foldin": n_foldin,
            "seconds": dt, "foldin_tokens_per_s": n_obs * n_foldin / dt, "loglik_per_scored_token": ll,
            "note": "documents are a prefix of the training corpus (stand-in for held-out documents); even positions "
                    "observed, odd positions scored; seconds include layout build, upload, fold-in and scoring"}


def run_gpu(corpus, K, steps, warmup, opts, holdout_docs=0):
    import torch
    import paper_1610_02496_amd as pk
    s = corpus.spec
    alpha, beta = 50.0 / K, s.beta
    t0 = time.time()
    g = pk.Saber(corpus.doc_ptr, corpus.word_ids, s.V, K, alpha, beta, s.seed, profile=1, **opts)
    log("[bench] K=%d init %.1fs (layout build + upload + first M-step)" % (K, time.time() - t0))
    g.iterate(warmup)
    g.reset_stats()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.iterate(steps)            # synchronous: returns after the stream has drained
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = g.get_stats()
    ll = g.loglik()
    T = corpus.T
    z_bytes = 2 if K <= 65536 else 4
    launches = max(1, st["sample_launches"])
    bytes_total = algorithmic_bytes(st, K, z_bytes)
    ms_sample = st["ms_sample"]
    achieved = bytes_total / (ms_sample * 1e-3) / 1e9 if ms_sample > 0 else 0.0
    res = {
        "K": K, "tokens_per_s": T * steps / dt, "ms_per_step": dt * 1e3 / steps,
        "sample_tokens_per_s": T * steps / (ms_sample * 1e-3) if ms_sample > 0 else None,
        "ms_sample": ms_sample / steps, "ms_count_dz": st["ms_count_dz"] / steps, "ms_ck": st["ms_ck"] / steps,
        "ms_phi": st["ms_phi"] / steps,
        "mean_Kd_per_token": st["sum_row_entries"] / max(1, st["sum_tokens"]),
        "row_entries_fetched_per_token": st["sum_row_fetch"] / max(1, st["sum_tokens"]),
        "dense_fraction": st["sum_tokens_dense"] / max(1, st["sum_tokens"]),
        "bytes_per_token_model": bytes_total / max(1, st["sum_tokens"]),
        "nnz_cd": st["nnz_cd"], "loglik": ll, "iterations_run": warmup + steps,
        "roofline": {"bound": "hbm", "kernel": "estep_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_launch": bytes_total / launches, "ms_per_launch": ms_sample / launches,
                     "achieved_is": "algorithmic (model) bytes of a pass / its duration between HIP events on the library's "
                                    "stream; most of them are rows of A that the 256 MB Infinity Cache serves, so this is a "
                                    "fraction of the HBM peak figure, not a count of HBM transactions"},
    }
    if holdout_docs:
        res["holdout"] = run_holdout(g, corpus, holdout_docs, 10)
    g.close()
    return res


def run_streaming(corpus, K, steps, warmup, workers, chunks):
    """Host streaming (Sec. 3.1.2): the same iterations with the token lists in pinned host memory, `workers`
    device buffers and `chunks` document chunks; 4 bytes per token and iteration cross the host link."""
    import torch
    import paper_1610_02496_amd as pk
    s = corpus.spec
    g = pk.Saber(corpus.doc_ptr, corpus.word_ids, s.V, K, 50.0 / K, s.beta, s.seed, stream_workers=workers,
                 **({"n_chunks": chunks} if chunks else {}))
    g.iterate(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.iterate(steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    res = {"workers": workers, "chunks": chunks, "tokens_per_s": corpus.T * steps / dt, "ms_per_step": dt * 1e3 / steps,
           "host_link_bytes_per_token": 4, "host_link_gbs": 4.0 * corpus.T * steps / dt / 1e9, "loglik": g.loglik()}
    g.close()
    return res


def cpu_model_name():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def run_cpu_baseline(corpus, K, docs):
    """The oracle, as it stands, on a document prefix of the same corpus: one full iteration (E-step + M-step), first
    on one thread (the canonical oracle: `value`), then on all the cores this process may use (`value_all_cores`; the
    oracle's E-step is an OpenMP loop over tokens that read frozen counts and draw from a counter-based generator,
    its M-step is serial).  The multi-threaded assignments must equal the single-threaded ones before either figure
    is reported."""
    import oracle
    s = corpus.spec
    docs = min(docs, s.D)
    doc_ptr = np.ascontiguousarray(corpus.doc_ptr[: docs + 1])
    T = int(doc_ptr[-1])
    word_ids = np.ascontiguousarray(corpus.word_ids[:T])
    nproc = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = nproc
    cores = max(1, min(usable, int(os.environ.get("OMP_NUM_THREADS", usable))))
    seconds, z = {}, {}
    for threads in (1, cores):
        m = oracle.Model(doc_ptr, word_ids, s.V, K, 50.0 / K, s.beta, s.seed)
        t0 = time.perf_counter()
        m.iterate(1, nthreads=threads)
        seconds[threads] = time.perf_counter() - t0
        z[threads] = m.z.copy()
        m.close()
    assert np.array_equal(z[1], z[cores]), "the oracle's assignments depend on its thread count"
    return {"value": T / seconds[1], "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "value_all_cores": T / seconds[cores], "cores_all": cores, "nproc": nproc, "cpu_model": cpu_model_name(),
            "threads_bit_identical": True,
            "sample": "first %d documents (%d tokens) of the same corpus, K=%d, V=%d, iteration 1 (E-step + M-step): %.1fs on "
                      "1 thread, %.1fs on %d threads" % (docs, T, K, s.V, seconds[1], seconds[cores], cores)}


def run_c4(steps, warmup, copy_gbs):
    """The PubMed-shaped workload (D=8.2M, V=141K, T=738M, fitted K=5,000) under the same clock: short documents, a
    third of the tokens on the dense branch; library defaults (six document chunks)."""
    import corpusgen
    os.environ.setdefault("LDA_CORPUS_PROGRESS", "2000000")
    spec = corpusgen.SPECS["C4"]
    t0 = time.time()
    corpus = corpusgen.generate(spec, with_topics=False)
    log("[bench] corpus %s: D=%d V=%d T=%d generated in %.1fs" % (spec.name, spec.D, spec.V, corpus.T, time.time() - t0))
    res = run_gpu(corpus, spec.K, steps, warmup, {})
    res["workload"] = ("C4: seeded LDA corpus D=%d V=%d T=%d (PubMed-shaped), fitted K=%d, alpha=50/K, beta=0.01, iterations "
                       "%d..%d from the Philox initial assignment" % (spec.D, spec.V, corpus.T, spec.K, warmup + 1, warmup + steps))
    if copy_gbs:
        res["roofline"]["frac_of_copy_kernel"] = res["roofline"]["achieved"] / copy_gbs
    res["roofline"]["traffic"] = profiled_traffic("C4", steps, warmup)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"],
                    help="C3 (default) is the benchmark line; C4 (738 M tokens) and C5 (7.1 G tokens: 6 minutes of corpus "
                         "generation, 30 GB of host memory for the token list) are the large workloads")
    ap.add_argument("--docs", type=int, default=0, help="use only a document prefix (experiments; 0 = full corpus)")
    ap.add_argument("--no-also", action="store_true", help="skip the secondary K")
    ap.add_argument("--no-c4", action="store_true", help="skip the PubMed-shaped workload (about 80 s: 738 M tokens to generate)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-docs", type=int, default=24000)
    ap.add_argument("--block-threads", type=int, default=0)
    ap.add_argument("--tile-tokens", type=int, default=0)
    ap.add_argument("--chunks", type=int, default=0)
    ap.add_argument("--stage-min", type=int, default=0)
    ap.add_argument("--light-block", type=int, default=0)
    ap.add_argument("--probe-bytes", type=int, default=1 << 30, help="size of the copy-bandwidth probe (0 = skip)")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=INT",
                    help="any other field of saber_options, for experiments (e.g. --opt dz_lds_entries=2048)")
    ap.add_argument("--streaming", default="3:2", metavar="WORKERS:CHUNKS",
                    help="also time the iterations with host streaming in this configuration ('' = skip)")
    ap.add_argument("--topic-conc", type=float, default=0.0,
                    help="override the mean per-word Dirichlet concentration of the planted topics (the workloads use "
                         "0.01; smaller values give topics that differ more); the workload name then says so")
    ap.add_argument("--holdout-docs", type=int, default=30000,
                    help="documents scored by the holdout log-likelihood after the timed region (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path would shard by document, "
            "but no multi-GPU code is part of it)" % args.gpus)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU available; the HIP path has no CPU fallback")
        sys.exit(3)

    import corpusgen
    spec = corpusgen.SPECS[args.workload]
    if args.workload in ("C4", "C5"):
        os.environ.setdefault("LDA_CORPUS_PROGRESS", "2000000")   # the generator reports on stderr while it works
        if args.streaming == "3:2":
            args.streaming = "3:0"                                 # chunks as the library cuts them
    if args.docs:
        spec = corpusgen.scaled(spec, args.docs)
    if args.topic_conc > 0:
        import dataclasses
        spec = dataclasses.replace(spec, topic_conc=args.topic_conc, name="%s(topic concentration %g)" % (spec.name, args.topic_conc))
    t0 = time.time()
    corpus = corpusgen.generate(spec, with_topics=False)
    log("[bench] corpus %s: D=%d V=%d T=%d generated in %.1fs" % (spec.name, spec.D, spec.V, corpus.T, time.time() - t0))
    T_main = corpus.T
    opts = {}
    if args.block_threads: opts["block_threads"] = args.block_threads
    if args.tile_tokens: opts["tile_tokens"] = args.tile_tokens
    if args.chunks: opts["n_chunks"] = args.chunks
    if args.stage_min: opts["stage_min_tokens"] = args.stage_min
    if args.light_block: opts["light_block_threads"] = args.light_block
    for kv in args.opt:
        name, val = kv.split("=")
        opts[name] = int(val)

    copy_gbs = None
    if args.probe_bytes:
        import paper_1610_02496_amd as pk
        copy_gbs = pk.bandwidth_probe(args.probe_bytes, 10)
        log("[bench] plain copy kernel: %.0f GB/s (read+write)" % copy_gbs)
    main_res = run_gpu(corpus, spec.K, args.steps, args.warmup, opts, args.holdout_docs)
    main_res["roofline"]["copy_kernel_gbs"] = copy_gbs
    if copy_gbs:
        main_res["roofline"]["frac_of_copy_kernel"] = main_res["roofline"]["achieved"] / copy_gbs
    if not opts and not args.docs and not args.topic_conc:
        main_res["roofline"]["traffic"] = profiled_traffic(args.workload, args.steps, args.warmup)
        if main_res["roofline"]["traffic"] is None:
            main_res["roofline"]["traffic_note"] = ("no counter figure stored for this command line and these kernel sources "
                                                    "(digest %s)" % source_digest())
    log("[bench] K=%d: %s" % (spec.K, json.dumps(main_res)))
    also = None
    if args.workload == "C3" and not args.no_also:
        also = run_gpu(corpus, 1000, args.steps, args.warmup, opts)
        log("[bench] K=1000: %s" % json.dumps(also))
    streaming = None
    if args.streaming and not opts:
        w, nch = (int(x) for x in args.streaming.split(":"))
        streaming = run_streaming(corpus, spec.K, args.steps, args.warmup, w, nch)
        streaming["vs_resident"] = streaming["tokens_per_s"] / main_res["tokens_per_s"]
        log("[bench] host streaming: %s" % json.dumps(streaming))
    cpu = None
    if not args.no_cpu_baseline:
        cpu = run_cpu_baseline(corpus, spec.K, args.cpu_docs)
        log("[bench] cpu baseline: %s" % json.dumps(cpu))
    also_c4 = None
    if args.workload == "C3" and not args.no_c4 and not opts and not args.docs and not args.topic_conc:
        corpus = None                                # 0.4 GB; the next corpus takes 3 GB
        also_c4 = run_c4(args.steps, args.warmup, copy_gbs)
        log("[bench] C4: %s" % json.dumps(also_c4))

    out = {
        "metric": "Gibbs tokens sampled/sec/iteration (whole ESCA iteration: E-step + M-step) at K=%d" % spec.K,
        "value": main_res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: seeded LDA corpus D=%d V=%d T=%d (%s-shaped), fitted K=%d, alpha=50/K, beta=0.01, "
                               "iterations %d..%d from the Philox initial assignment"
                               % (spec.name, spec.D, spec.V, T_main,
                                  {"C4": "PubMed", "C5": "ClueWeb12-subset"}.get(args.workload, "NYTimes"), spec.K,
                                  args.warmup + 1, args.warmup + args.steps)},
        "roofline": main_res["roofline"], "cpu_baseline": cpu,
        "detail": {k: v for k, v in main_res.items() if k not in ("roofline", "holdout")},
    }
    if "holdout" in main_res:
        out["holdout"] = main_res["holdout"]
    if streaming is not None:
        out["streaming"] = streaming
    if also is not None:
        out["also"] = also
    if also_c4 is not None:
        out["also_c4"] = also_c4
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
