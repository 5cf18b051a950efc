#!/usr/bin/env python3
"""Benchmark of the SGNS training hot path on one MI355X.

A step is one pass of the whole hot path (subsampling, width and negative draws, row gathers,
window arithmetic, scatter, loss) over one synthetic corpus resident in HBM: the 'Mid' workload,
vocabulary 71,000 Zipf(1.05) with 16 planted clusters, 17M tokens in 1,000-token sentences, d=128,
W=5, N=5, subsampling t=1e-4, min-count 5.  Step e is epoch e of a (warmup+steps)-epoch schedule.

Prints one JSON line: words/sec (corpus tokens, pre-subsampling), the HBM roofline of the window
kernel from its algorithmic bytes ((2N+4) rows of 4d bytes per kept word) and live HIP-event
timing, and the CPU oracle timed on a prefix of the same corpus (on one core, and with its sentences
striped over all the host's cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
WORKLOADS = {
    # name: (generator kwargs, dim, window, negatives, subsample_t, table_size)
    "mid": (dict(vocab=71000, s=1.05, n_sent=17000, sent_len=1000, seed=1), 128, 5, 5, 1e-4, 1 << 24),
    # prefixes of the two big configurations (same vocabulary / row sizes, fewer sentences), for --workload only
    "large": (dict(vocab=550000, s=1.1, n_sent=44000, sent_len=1000, seed=1), 300, 5, 10, 1e-5, 1 << 24),
    "graph": (dict(n_nodes=1000000, m=5, walks_per_node=1, walk_len=80, seed=1), 128, 10, 5, 0.0, 1 << 24),
    "small": (dict(vocab=8000, s=1.05, n_sent=600, sent_len=1000, seed=1, band_start=400), 128, 5, 5, 1e-4, 1 << 20),
}


def time_epochs(tokens, sent_off, counts, *, dim, window, negatives, subsample_t, table_size, steps, warmup,
                update_mode=0, storage=0, window_mode=0):
    """ms per epoch (HIP events on the launch stream) and the figures derived from it for one resident corpus."""
    import numpy as np
    import torch
    from paper_2312_07743_amd import binding as B
    from paper_2312_07743_amd.trainer import Trainer
    n_tokens = int(tokens.numel()) if isinstance(tokens, torch.Tensor) else len(tokens)
    tr = Trainer(vocab=len(counts), dim=dim, window=window, negatives=negatives, counts=counts, tokens_per_epoch=n_tokens,
                 seed=2024, table_size=table_size, subsample_t=subsample_t, total_epochs=warmup + steps,
                 update_mode=update_mode, storage=storage, window_mode=window_mode)
    tr.set_corpus(tokens, sent_off)
    for e in range(warmup):
        tr.train_epoch(e)
    torch.cuda.synchronize()
    tr.counters(reset=True)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for e in range(warmup, warmup + steps):
        tr.train_epoch(e)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    kept, _ = tr.counters()
    loss, pairs = tr.loss()
    plan = B.w2v_debug_get_plan(tr.ctx)
    tr.close()
    algo = (2 * negatives + 4) * (2 if storage else 4) * dim * (kept / steps)
    return {"ms_per_epoch": ms, "words_per_s": n_tokens / (ms * 1e-3), "kept_fraction": kept / (steps * n_tokens),
            "algorithmic_GBs": algo / (ms * 1e-3) / 1e9, "frac_of_8TBs": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "mean_loss": loss / max(pairs, 1), "update_mode": "summed" if plan["update"] == 1 else "overwrite",
            "wavefronts": plan["wavefronts"], "epochs_timed": steps, "table_storage": "bf16" if storage else "f32"}


def other_workloads(mid):
    """The other configurations, a few epochs each on corpora generated in device memory (prefixes of the two 800M-token
    ones: bytes and work per word do not depend on the corpus length).  Same algorithmic bytes per kept word as the
    headline, (2N+4) rows of 4d bytes, also for the summed mode, which moves more rows than that."""
    import torch
    from paper_2312_07743_amd import synth_device
    out = []
    for d in (64, 256, 300, 512):
        r = time_epochs(mid.tokens, mid.sent_off, mid.counts, dim=d, window=5, negatives=5, subsample_t=1e-4,
                        table_size=1 << 24, steps=3, warmup=2)
        out.append(dict(workload=f"mid corpus, d={d}, W=5, N=5, t=1e-4", **r))
    for d in (128, 256):          # extension: tables stored as bfloat16 (half the algorithmic bytes per kept word)
        r = time_epochs(mid.tokens, mid.sent_off, mid.counts, dim=d, window=5, negatives=5, subsample_t=1e-4,
                        table_size=1 << 24, steps=3, warmup=2, storage=1)
        out.append(dict(workload=f"mid corpus, d={d}, W=5, N=5, t=1e-4, bfloat16 tables", **r))
    tok, counts = synth_device.zipf_tokens(550000, 1.1, 44_000_000, seed=1)
    off = torch.arange(44_001, dtype=torch.int64, device="cuda") * 1000
    for storage in (0, 1):
        r = time_epochs(tok, off, counts, dim=300, window=5, negatives=10, subsample_t=1e-5, table_size=1 << 24, steps=3,
                        warmup=1, storage=storage)
        out.append(dict(workload="large prefix: vocab 550,000 Zipf(1.1), 44M tokens in 1,000-token sentences, d=300, W=5, "
                                 "N=10, t=1e-5" + (", bfloat16 tables" if storage else ""), **r))
    del tok
    tok, counts = synth_device.barabasi_albert_walk_tokens(1_000_000, 5, 1, 80, seed=1)
    off = torch.arange(1_000_001, dtype=torch.int64, device="cuda") * 80
    for mode, fixed, name in ((0, 0, "library default"), (1, 0, "update_mode 1"),
                              (1, 1, "update_mode 1, fixed window width ceil(W/2) (the paper's variant)")):
        r = time_epochs(tok, off, counts, dim=128, window=10, negatives=5, subsample_t=0.0, table_size=1 << 24, steps=3,
                        warmup=1, update_mode=mode, window_mode=fixed)
        out.append(dict(workload=f"graph prefix: Barabasi-Albert 1M nodes (m=5), 80M tokens in walks of 80, d=128, W=10, N=5, "
                                 f"no subsampling, {name}", **r))
    del tok
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mid", choices=sorted(WORKLOADS))
    ap.add_argument("--dim", type=int, default=None, help="override d (dimension sweep)")
    ap.add_argument("--in-flight", type=int, default=0, help="sentences_in_flight (0 = fill the GPU)")
    ap.add_argument("--fixed-width", action="store_true",
                    help="window_mode 1: every window has width ceil(W/2) (the paper's own variant, Section 3.2)")
    ap.add_argument("--from-host", action="store_true",
                    help="feed the corpus from pinned host memory through w2v_train_epoch_host (PCIe-inclusive rate)")
    ap.add_argument("--staging-mb", type=int, default=128)
    ap.add_argument("--negative-block", type=int, default=0,
                    help="reuse of negatives over the windows centred in one stretch of this many tokens (an extension "
                         "the paper names as future work; 0 = the paper's fresh negatives per window)")
    ap.add_argument("--full-size", action="store_true",
                    help="large / graph at their whole size (800M tokens; the corpus alone takes minutes to generate) "
                         "instead of the prefix")
    ap.add_argument("--coherent-tables", action="store_true",
                    help="keep syn0 / syn1neg in uncached device memory (wavefronts on different XCDs see each other's "
                         "updates at once; for walk corpora)")
    ap.add_argument("--update-mode", type=int, default=0, choices=(0, 1, 2),
                    help="cfg.update_mode: 0 the library's choice from the word counts, 1 overwrite, 2 summed lock-free updates")
    ap.add_argument("--storage", type=int, default=0, choices=(0, 1),
                    help="cfg.storage: 0 float tables (the paper's precision), 1 bfloat16 tables with stochastic rounding")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other configurations (d sweep, large and graph prefixes) that the "
                         "default run of the mid workload adds as `other_workloads`")
    ap.add_argument("--naive", action="store_true",
                    help="time the no-reuse comparator kernel instead of the window kernel (traffic comparison only)")
    ap.add_argument("--cpu-sentences", type=int, default=5000)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy three times (scale for the rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (a second GPU is never used); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    if args.copy_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": a.numel() * 4, "copy_bytes_written": a.numel() * 4, "copies": 3}))
        return
    from paper_2312_07743_amd import synth
    from paper_2312_07743_amd.trainer import Trainer

    gen_kw, dim, window, negatives, t_sub, table_size = WORKLOADS[args.workload]
    gen_kw = dict(gen_kw)
    if args.dim:
        dim = args.dim
    if args.full_size:
        if args.workload == "large":
            gen_kw["n_sent"] = 800000
        elif args.workload == "graph":
            gen_kw["walks_per_node"] = 10
        gen_kw["progress"] = lambda text: print(text, file=sys.stderr, flush=True)
    if args.workload == "graph":
        corpus = synth.barabasi_albert_walks(**gen_kw)
        what = f"Barabasi-Albert graph ({gen_kw['n_nodes']} nodes, m={gen_kw['m']}), uniform walks of {gen_kw['walk_len']}"
    else:
        corpus = synth.planted_corpus(**gen_kw)
        what = f"Zipf({gen_kw['s']}) + 16 planted clusters"
    E = args.warmup + args.steps
    tr = Trainer(vocab=corpus.vocab, dim=dim, window=window, negatives=negatives, counts=corpus.counts,
                 tokens_per_epoch=corpus.n_tokens, seed=2024, table_size=table_size, subsample_t=t_sub,
                 total_epochs=E, sentences_in_flight=args.in_flight, window_mode=1 if args.fixed_width else 0, negative_block=args.negative_block,
                 coherent_tables=args.coherent_tables, update_mode=args.update_mode, storage=args.storage)
    tr.set_corpus(corpus.tokens, corpus.sent_off)
    if args.from_host:
        t_pin = torch.as_tensor(corpus.tokens).pin_memory()
        o_pin = torch.as_tensor(corpus.sent_off.view(np.int64)).pin_memory()

        def run_epoch(e):
            tr.train_epoch_from_host(t_pin, o_pin, epoch=e, staging_bytes=args.staging_mb << 20)
    else:
        def run_epoch(e):
            tr.train_epoch(e, naive=args.naive)
    for e in range(args.warmup):
        run_epoch(e)
    torch.cuda.synchronize()
    tr.loss(reset=True)

    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    host_s = 0.0                                 # time the calls themselves take on the host (they only queue work)
    for k in range(args.steps):
        starts[k].record()                       # torch's current stream is the one the library launches on
        h0 = time.perf_counter()
        run_epoch(args.warmup + k)
        host_s += time.perf_counter() - h0
        stops[k].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = [a.elapsed_time(b) for a, b in zip(starts, stops)]
    kept, _ = tr.counters()
    loss_sum, pairs = tr.loss()

    words = corpus.n_tokens * args.steps
    row_bytes = (2 if args.storage else 4) * dim
    rows_per_kept = 2 * negatives + 4
    if args.negative_block > 1:
        # the negatives' rows move once per stretch that has a kept token (first timed epoch taken as typical)
        keep, _, _ = tr.draws(epoch=args.warmup)
        sent = np.repeat(np.arange(corpus.n_sent), np.diff(corpus.sent_off.astype(np.int64)))
        stretch = (np.arange(corpus.n_tokens) - corpus.sent_off.astype(np.int64)[sent]) // args.negative_block
        key = (sent.astype(np.int64) << 32) | stretch
        rows_per_kept = 4 + 2 * negatives * len(np.unique(key[keep != 0])) / max(int(keep.sum()), 1)
    algo_bytes_per_launch = rows_per_kept * row_bytes * (kept / args.steps)
    avg_kernel_s = float(np.mean(kernel_ms)) / 1e3
    achieved = algo_bytes_per_launch / avg_kernel_s / 1e9
    traffic = traffic_source = None
    # measured L2<->memory bytes per launch: NOT measured in this run, read from the committed rocprofv3 counter
    # summary of this workload (two --pmc runs of this same command, see the file)
    tpath = os.path.join(ROOT, "profiles", f"window_kernel_all_workloads_counters.txt")
    if os.path.exists(tpath) and not (args.naive or args.fixed_width or args.from_host or args.negative_block > 1
                                      or args.coherent_tables or args.storage or args.update_mode):
        for line in open(tpath):
            if line.startswith("hbm_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
                traffic_source = f"profiles/{os.path.basename(tpath)} (rocprofv3 --pmc runs of this command, not this run)"

    # what a plain streaming copy reaches on this machine (1 GiB read + 1 GiB written per pass), for scale
    a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    b.copy_(a)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        b.copy_(a)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * a.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del a, b

    props = torch.cuda.get_device_properties(0)
    out = {
        "metric": "trained words/sec on 1 MI355X; achieved HBM GB/s vs peak",
        "value": words / wall, "unit": "words/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not args.storage else "f32 arithmetic, bf16 table storage", "data": "synthetic",
        "config": {"workload": f"{args.workload}: vocab {corpus.vocab} {what}, "
                               f"{corpus.n_tokens} tokens in {corpus.n_sent} sentences, d={dim}, W={window}, "
                               f"N={negatives}, subsample t={t_sub}, lr 0.025 linear decay"
                               + (", fixed width ceil(W/2)" if args.fixed_width else "")
                               + (f", negatives shared by stretches of {args.negative_block} tokens "
                                  f"({rows_per_kept:.2f} rows per kept word)" if args.negative_block > 1 else "")
                               + (", tables in uncached device memory" if args.coherent_tables else "")
                               + (f", corpus fed from pinned host memory in batches of {args.staging_mb // 2} MiB"
                                  if args.from_host else ""),
                   "kept_words_per_s": kept / wall, "kept_fraction": kept / words,
                   "mean_loss": loss_sum / max(pairs, 1), "sentences_in_flight": args.in_flight,
                   "host_ms_per_step_inside_the_calls": host_s / args.steps * 1e3,
                   "device": f"{props.name}, {props.multi_processor_count} CUs, "
                             f"{props.total_memory / 2**30:.0f} GiB"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "naive_kernel" if args.naive else "train_kernel", "avg_launch_ms": avg_kernel_s * 1e3,
                     "algorithmic_bytes_per_launch": algo_bytes_per_launch,
                     "streaming_copy_GBs_same_box": copy_gbs},
    }

    plain = not (args.naive or args.fixed_width or args.from_host or args.negative_block > 1 or args.coherent_tables
                 or args.dim or args.in_flight or args.update_mode or args.storage)
    if args.workload == "mid" and plain and not args.no_other_workloads:
        tr.close()
        out["other_workloads"] = other_workloads(corpus)

    if not args.no_cpu_baseline:
        from oracle import Oracle                     # the CPU oracle, timed as it stands (never tuned)
        orc = Oracle("float")
        ns = min(args.cpu_sentences, corpus.n_sent)
        syn0, syn1 = orc.init_weights(2024, corpus.vocab, dim)
        c0 = time.perf_counter()
        orc.train_epoch(syn0, syn1, corpus.counts, corpus.tokens, corpus.sent_off, window=window, negatives=negatives,
                        seed=2024, epoch=0, total_epochs=E, table_size=table_size, subsample_t=t_sub, s_end=ns,
                        window_mode=1 if args.fixed_width else 0, negative_block=args.negative_block, storage=args.storage)
        cdt = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": int(corpus.sent_off[ns]) / cdt, "unit": "words/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"first {ns} sentences ({int(corpus.sent_off[ns])} tokens) of the same corpus, "
                                         f"one epoch, {cdt:.1f} s"}
        # The same oracle with its sentences striped over the host's cores, each thread updating the shared
        # tables without locks (sentences are the independent units: paper Sections 2.2 and 2.3).
        threads = max(1, min(16, os.cpu_count() or 1))
        if threads > 1:
            from concurrent.futures import ThreadPoolExecutor
            na = min(ns * threads, corpus.n_sent)
            syn0, syn1 = orc.init_weights(2024, corpus.vocab, dim)

            def stripe(t):
                return orc.train_epoch(syn0, syn1, corpus.counts, corpus.tokens, corpus.sent_off, window=window,
                                       negatives=negatives, seed=2024, epoch=0, total_epochs=E, table_size=table_size,
                                       subsample_t=t_sub, s_begin=t, s_end=na, s_stride=threads,
                                       window_mode=1 if args.fixed_width else 0, negative_block=args.negative_block)
            c0 = time.perf_counter()
            with ThreadPoolExecutor(threads) as pool:
                parts = list(pool.map(stripe, range(threads)))
            adt = time.perf_counter() - c0
            out["cpu_baseline_all_cores"] = {
                "value": int(corpus.sent_off[na]) / adt, "unit": "words/s", "cores": threads,
                "kind": "oracle, sentences striped over threads that share the tables lock-free",
                "mean_loss": sum(r["loss_sum"] for r in parts) / max(sum(r["pairs"] for r in parts), 1),
                "sample": f"first {na} sentences ({int(corpus.sent_off[na])} tokens) of the same corpus, "
                          f"one epoch, {adt:.1f} s"}
    tr.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
