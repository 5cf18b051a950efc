"""Writes tests/golden/mid_hogwild_reference.json: the serial CPU oracle's per-epoch mean loss, pair
count and planted-cluster recovery on the 'Mid' workload (vocabulary 71,000 Zipf(1.05) with 16 planted
clusters, 17M tokens, d=128, W=5, N=5, t=1e-4), two epochs, for three training seeds (the seed keys the initial weights and every random
draw).  Calls only oracle/ and the input generator; takes about ten minutes on one core.

    python tests/golden/make_mid_hogwild_reference.py
    python tests/golden/make_mid_hogwild_reference.py --negative-block 16     (one seed, writes
        mid_hogwild_reference_nb16.json: the same with negatives shared by stretches of 16 tokens)
    python tests/golden/make_mid_hogwild_reference.py --fixed-width           (one seed, writes
        mid_hogwild_reference_fixed_width.json: every window has width ceil(W/2))
    python tests/golden/make_mid_hogwild_reference.py --large-shape           (one seed, writes
        large_shape_hogwild_reference.json: the hyper-parameters of the 'Large' workload, d=300, N=10, t=1e-5, on
        6,000 sentences of its Zipf(1.1) text with planted clusters, four epochs; about twenty minutes)
"""
import argparse
import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
sys.path.insert(0, os.path.dirname(HERE))

from oracle import Oracle                                   # noqa: E402
from paper_2312_07743_amd import synth                      # noqa: E402
from util import planted_score                              # noqa: E402

PARAMS = dict(dim=128, window=5, negatives=5, table_size=1 << 24, subsample_t=1e-4, epochs=2)
SEEDS = (5, 6, 7)
CORPUS = dict(vocab=71000, s=1.05, n_sent=17000, sent_len=1000, seed=1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--negative-block", type=int, default=0)
    ap.add_argument("--fixed-width", action="store_true")
    ap.add_argument("--large-shape", action="store_true")
    args = ap.parse_args()
    global PARAMS, SEEDS, CORPUS
    name = "mid_hogwild_reference.json"
    if args.negative_block > 1:
        PARAMS = dict(PARAMS, negative_block=args.negative_block)
        SEEDS = SEEDS[:1]
        name = f"mid_hogwild_reference_nb{args.negative_block}.json"
    elif args.fixed_width:
        PARAMS = dict(PARAMS, window_mode=1)
        SEEDS = SEEDS[:1]
        name = "mid_hogwild_reference_fixed_width.json"
    elif args.large_shape:
        PARAMS = dict(dim=300, window=5, negatives=10, table_size=1 << 24, subsample_t=1e-5, epochs=4)
        CORPUS = dict(vocab=550000, s=1.1, n_sent=6000, sent_len=1000, seed=1)
        SEEDS = SEEDS[:1]
        name = "large_shape_hogwild_reference.json"
    orc = Oracle("float")
    c = synth.planted_corpus(**CORPUS)
    path = os.path.join(HERE, name)
    out = {"params": PARAMS, "corpus": CORPUS, "vocab": c.vocab, "tokens": c.n_tokens, "runs": []}
    if os.path.exists(path):                       # resume: keep the seeds that are already complete
        old = json.load(open(path))
        if old.get("params") == PARAMS and old.get("corpus") == CORPUS:
            out["runs"] = [r for r in old.get("runs", []) if len(r["epochs"]) == PARAMS["epochs"]]
    for seed in SEEDS:
        if any(r["seed"] == seed for r in out["runs"]):
            continue
        syn0, syn1 = orc.init_weights(seed, c.vocab, PARAMS["dim"])
        run = {"seed": seed, "epochs": []}
        for e in range(PARAMS["epochs"]):
            t = time.time()
            r = orc.train_epoch(syn0, syn1, c.counts, c.tokens, c.sent_off, window=PARAMS["window"],
                                negatives=PARAMS["negatives"], seed=seed, epoch=e,
                                total_epochs=PARAMS["epochs"], table_size=PARAMS["table_size"],
                                subsample_t=PARAMS["subsample_t"], negative_block=PARAMS.get("negative_block", 0),
                                window_mode=PARAMS.get("window_mode", 0))
            run["epochs"].append({"mean_loss": r["loss_sum"] / r["pairs"], "pairs": r["pairs"],
                                  "planted_score": planted_score(syn0, c.labels)})
            print(seed, e, run["epochs"][-1], f"{time.time() - t:.0f}s", flush=True)
        out["runs"].append(run)
        with open(path, "w") as f:
            json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
