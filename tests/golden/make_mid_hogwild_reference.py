"""Writes the stored references of the lock-free (Hogwild) parity tests: the serial CPU oracle's per-epoch mean
loss, pair count and quality figures, one run per training seed (the seed keys the initial weights and every random
draw).  Calls only oracle/ and the input generator.

    python tests/golden/make_mid_hogwild_reference.py
        mid_hogwild_reference.json: the 'Mid' workload (vocabulary 71,000 Zipf(1.05) with 16 planted clusters, 17M
        tokens, d=128, W=5, N=5, t=1e-4), two epochs, three seeds; about five minutes per seed
    python tests/golden/make_mid_hogwild_reference.py --negative-block 16     (one seed, writes
        mid_hogwild_reference_nb16.json: the same with negatives shared by stretches of 16 tokens)
    python tests/golden/make_mid_hogwild_reference.py --fixed-width           (one seed, writes
        mid_hogwild_reference_fixed_width.json: every window has width ceil(W/2))
    python tests/golden/make_mid_hogwild_reference.py --large-shape           (one seed, writes
        large_shape_hogwild_reference.json: the hyper-parameters of the 'Large' workload, d=300, N=10, t=1e-5, on
        6,000 sentences of its Zipf(1.1) text with planted clusters, four epochs; about twenty minutes)
    python tests/golden/make_mid_hogwild_reference.py --graph-shape           (two seeds, writes
        graph_hogwild_reference.json: the hyper-parameters of the 'Graph' workload, d=128, W=10, N=5, no subsampling,
        on 10 uniform walks of 80 steps from every node of a 100,000-node Barabasi-Albert graph (m=5): 80M tokens,
        as many visits per node and epoch as the whole workload has, two epochs; about an hour per seed)
    python tests/golden/make_mid_hogwild_reference.py --bf16                  (one seed, writes
        mid_hogwild_reference_bf16.json: the 'Mid' workload with the tables stored as bfloat16, stochastic rounding)
    --jobs J runs up to J seeds at a time in processes of their own.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ProcessPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
sys.path.insert(0, os.path.dirname(HERE))

from oracle import Oracle                                   # noqa: E402
from paper_2312_07743_amd import synth                      # noqa: E402
from util import cluster_margin, edge_recovery, planted_score   # noqa: E402

MID = dict(params=dict(dim=128, window=5, negatives=5, table_size=1 << 24, subsample_t=1e-4, epochs=2),
           corpus=dict(vocab=71000, s=1.05, n_sent=17000, sent_len=1000, seed=1), seeds=(5, 6, 7))


def setting(args):
    """(file name, oracle parameters, corpus generator arguments, training seeds) of the chosen reference"""
    if args.negative_block > 1:
        return (f"mid_hogwild_reference_nb{args.negative_block}.json",
                dict(MID["params"], negative_block=args.negative_block), MID["corpus"], MID["seeds"][:1])
    if args.bf16:
        return "mid_hogwild_reference_bf16.json", dict(MID["params"], storage=1), MID["corpus"], MID["seeds"][:1]
    if args.fixed_width:
        return ("mid_hogwild_reference_fixed_width.json", dict(MID["params"], window_mode=1), MID["corpus"],
                MID["seeds"][:1])
    if args.large_shape:
        return ("large_shape_hogwild_reference.json",
                dict(dim=300, window=5, negatives=10, table_size=1 << 24, subsample_t=1e-5, epochs=4),
                dict(vocab=550000, s=1.1, n_sent=6000, sent_len=1000, seed=1), MID["seeds"][:1])
    if args.graph_shape:
        return ("graph_hogwild_reference.json",
                dict(dim=128, window=10, negatives=5, table_size=1 << 24, subsample_t=0.0, epochs=2),
                dict(n_nodes=100000, m=5, walks_per_node=10, walk_len=80, seed=1), MID["seeds"][:2])
    return "mid_hogwild_reference.json", MID["params"], MID["corpus"], MID["seeds"]


def make_corpus(corpus):
    return synth.barabasi_albert_walks(**corpus) if "n_nodes" in corpus else synth.planted_corpus(**corpus)


def one_run(job):
    params, corpus, seed = job
    orc = Oracle("float")
    c = make_corpus(corpus)
    syn0, syn1 = orc.init_weights(seed, c.vocab, params["dim"], storage=params.get("storage", 0))
    run = {"seed": seed, "epochs": []}
    for e in range(params["epochs"]):
        t = time.time()
        r = orc.train_epoch(syn0, syn1, c.counts, c.tokens, c.sent_off, window=params["window"],
                            negatives=params["negatives"], seed=seed, epoch=e, total_epochs=params["epochs"],
                            table_size=params["table_size"], subsample_t=params["subsample_t"],
                            negative_block=params.get("negative_block", 0), window_mode=params.get("window_mode", 0),
                            storage=params.get("storage", 0))
        rec = {"mean_loss": r["loss_sum"] / r["pairs"], "pairs": r["pairs"]}
        if c.labels is not None:
            rec["planted_score"] = planted_score(syn0, c.labels)
            rec["cluster_margin"] = cluster_margin(syn0, c.labels)
        else:
            rec["edge_score"], rec["edge_margin"] = edge_recovery(syn0, c.tokens, c.sent_off)
        run["epochs"].append(rec)
        print(seed, e, rec, f"{time.time() - t:.0f}s", flush=True)
    return run


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--negative-block", type=int, default=0)
    ap.add_argument("--fixed-width", action="store_true")
    ap.add_argument("--large-shape", action="store_true")
    ap.add_argument("--graph-shape", action="store_true")
    ap.add_argument("--bf16", action="store_true")
    ap.add_argument("--jobs", type=int, default=1)
    args = ap.parse_args()
    name, params, corpus, seeds = setting(args)
    c = make_corpus(corpus)
    path = os.path.join(HERE, name)
    out = {"params": params, "corpus": corpus, "vocab": c.vocab, "tokens": c.n_tokens, "runs": []}
    want = "planted_score" if c.labels is not None else "edge_score"
    del c
    if os.path.exists(path):                       # resume: keep the seeds that are already complete
        old = json.load(open(path))
        if old.get("params") == params and old.get("corpus") == corpus:
            out["runs"] = [r for r in old.get("runs", [])
                           if len(r["epochs"]) == params["epochs"] and all(
                               want in e and ("cluster_margin" in e or want == "edge_score") for e in r["epochs"])]
    todo = [(params, corpus, seed) for seed in seeds if not any(r["seed"] == seed for r in out["runs"])]
    with ProcessPoolExecutor(max(1, args.jobs)) as pool:
        for run in pool.map(one_run, todo):
            out["runs"].append(run)
            out["runs"].sort(key=lambda r: r["seed"])
            with open(path, "w") as f:
                json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
