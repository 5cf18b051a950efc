"""Helpers shared by the GPU parity tests."""
import numpy as np


def run_oracle(orc, corpus, *, dim, window, negatives, seed, epochs=1, table_size=1 << 16, subsample_t=0.0,
               window_mode=0, lr0=0.025, syn0=None, syn1neg=None, first_token_global_pos=0, tokens_per_epoch=None,
               total_epochs=None, start_epoch=0, update_mode=0, negative_block=0, storage=0):
    if syn0 is None:
        syn0, syn1neg = orc.init_weights(seed, corpus.vocab, dim, storage=storage)
    else:
        syn0, syn1neg = syn0.copy(), syn1neg.copy()
    total_epochs = total_epochs or epochs
    loss = pairs = 0
    for e in range(start_epoch, start_epoch + epochs):
        r = orc.train_epoch(syn0, syn1neg, corpus.counts, corpus.tokens, corpus.sent_off, window=window,
                            negatives=negatives, seed=seed, epoch=e, total_epochs=total_epochs, table_size=table_size,
                            subsample_t=subsample_t, window_mode=window_mode, lr0=lr0, update_mode=update_mode,
                            first_token_global_pos=first_token_global_pos, tokens_per_epoch=tokens_per_epoch,
                            negative_block=negative_block, storage=storage)
        loss += r["loss_sum"]
        pairs += r["pairs"]
    return syn0, syn1neg, loss, pairs


def run_gpu(corpus, *, dim, window, negatives, seed, epochs=1, table_size=1 << 16, subsample_t=0.0, window_mode=0,
            lr0=0.025, sentences_in_flight=0, syn0=None, syn1neg=None, first_token_global_pos=0,
            tokens_per_epoch=None, total_epochs=None, start_epoch=0, naive=False, unit_shift=None, negative_block=0,
            unit_tail=None, storage=0):
    from paper_2312_07743_amd import binding
    from paper_2312_07743_amd.trainer import Trainer
    tr = Trainer(vocab=corpus.vocab, dim=dim, window=window, negatives=negatives, counts=corpus.counts,
                 tokens_per_epoch=tokens_per_epoch or corpus.n_tokens, seed=seed, table_size=table_size,
                 subsample_t=subsample_t, total_epochs=total_epochs or epochs, sentences_in_flight=sentences_in_flight,
                 window_mode=window_mode, lr0=lr0, syn0=syn0, syn1neg=syn1neg, negative_block=negative_block,
                 storage=storage)
    tr.set_corpus(corpus.tokens, corpus.sent_off)
    if unit_shift is not None:
        binding.w2v_debug_set_units(tr.ctx, unit_shift)
    if unit_tail is not None:                      # (fine_shift, first sentence cut that finely)
        binding.w2v_debug_set_unit_tail(tr.ctx, *unit_tail)
    for e in range(start_epoch, start_epoch + epochs):
        tr.train_epoch(e, first_token_global_pos, naive=naive)
    loss, pairs = tr.loss()
    out = tr.embeddings(0), tr.embeddings(1), loss, pairs
    tr.close()
    return out


def scaled_error(got, ref):
    """|delta_ij| / max(|ref_ij|, rms(ref_row_i)): relative per element, with the row's own scale as the floor so that
    elements that happen to be near zero do not make the measure meaningless."""
    ref = ref.astype(np.float64)
    got = got.astype(np.float64)
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    return np.abs(got - ref) / np.maximum(np.maximum(np.abs(ref), rms), 1e-300)


def assert_rows_close(got, ref, tol=1e-4, what=""):
    """The gate of the strict-order parity tests on scaled_error(got, ref).

    One Tiny epoch is 100,000 dependent fp32 updates: the fp32 oracle itself sits 0.95e-4 (same measure) from its
    own fp64 build (tests/test_oracle_pins.py measures it), so two correct fp32 evaluations that merely sum in a
    different order can be up to about 2e-4 apart on a few elements.  The gate is therefore: every element within
    2*tol, and all but at most one element in 10,000 within tol."""
    scaled = scaled_error(got, ref)
    worst = float(scaled.max())
    over = int((scaled > tol).sum())
    assert worst <= 2 * tol, f"{what}: worst scaled error {worst:.3e} (limit {2 * tol})"
    assert over <= 1e-4 * scaled.size, f"{what}: {over} of {scaled.size} elements beyond {tol}, worst {worst:.3e}"
    return worst


def assert_no_further_from_fp64_than_fp32_oracle(got, ref32, ref64, factor=1.5, what=""):
    """The HIP result (fp32 arithmetic) may sit no further from the fp64 oracle than `factor` times the distance of
    the fp32 oracle from it: both are fp32 evaluations of the same epoch that round in different orders."""
    floor = float(scaled_error(ref32, ref64).max())
    mine = float(scaled_error(got, ref64).max())
    assert mine <= factor * floor, f"{what}: {mine:.3e} from the fp64 oracle, the fp32 oracle {floor:.3e}"
    return mine, floor


def planted_score(emb, labels, topk=10):
    """Mean, over the planted words, of the share of their topk cosine neighbours in their own cluster."""
    idx = np.flatnonzero(labels >= 0)
    e = emb / np.maximum(np.linalg.norm(emb, axis=1, keepdims=True), 1e-30)
    sims = e[idx] @ e.T
    sims[np.arange(len(idx)), idx] = -np.inf
    nn = np.argpartition(-sims, topk, axis=1)[:, :topk]
    return float((labels[nn] == labels[idx][:, None]).mean())


def cluster_margin(emb, labels):
    """Mean cosine between planted words of one cluster minus the mean cosine between planted words of different
    clusters: a quality axis that keeps moving after the top-10 score has reached 1."""
    idx = np.flatnonzero(labels >= 0)
    e = emb[idx].astype(np.float64)
    e /= np.maximum(np.linalg.norm(e, axis=1, keepdims=True), 1e-30)
    sims = e @ e.T
    same = labels[idx][:, None] == labels[idx][None, :]
    off_diag = ~np.eye(len(idx), dtype=bool)
    return float(sims[same & off_diag].mean() - sims[~same].mean())


def _walk_edges(tokens, sent_off, vocab):
    """Sorted unique keys a*vocab+b of the ordered pairs (a, b) of words that follow one another inside a sentence
    (both directions): for a walk corpus, the edges of the graph that the walks used."""
    tok = np.asarray(tokens, np.int64)
    ends = np.asarray(sent_off, np.int64)[1:-1] - 1          # last token of every sentence but the final one
    ok = np.ones(len(tok) - 1, bool)
    ok[ends[(ends >= 0) & (ends < len(ok))]] = False
    a, b = tok[:-1][ok], tok[1:][ok]
    return np.unique(np.concatenate([a * vocab + b, b * vocab + a]))


def edge_recovery(emb, tokens, sent_off, n_sample=2000, topk=10, seed=0):
    """Walk corpora: (share of the topk cosine neighbours of a sampled node that are joined to it by an edge the
    walks used, mean cosine over those edges minus mean cosine over random node pairs).  The edges are the structure
    planted in such a corpus; the first figure plays the part of the planted-cluster score, the second is a
    continuous margin."""
    vocab = emb.shape[0]
    edges = _walk_edges(tokens, sent_off, vocab)
    rng = np.random.default_rng(seed)
    e = emb.astype(np.float32)
    e /= np.maximum(np.linalg.norm(e, axis=1, keepdims=True), 1e-30)
    seen = np.unique(edges // vocab)
    sample = rng.choice(seen, size=min(n_sample, len(seen)), replace=False)
    hits = 0
    for a in range(0, len(sample), 250):
        part = sample[a:a + 250]
        sims = e[part] @ e.T
        sims[np.arange(len(part)), part] = -np.inf
        nn = np.argpartition(-sims, topk, axis=1)[:, :topk]
        keys = part[:, None].astype(np.int64) * vocab + nn
        pos = np.searchsorted(edges, keys)
        hits += int((edges[np.minimum(pos, len(edges) - 1)] == keys).sum())
    pick = edges[rng.integers(0, len(edges), size=200000)]
    on_edges = float((e[pick // vocab] * e[pick % vocab]).sum(axis=1).mean())
    ra, rb = rng.choice(seen, size=200000), rng.choice(seen, size=200000)
    at_random = float((e[ra] * e[rb]).sum(axis=1).mean())
    return hits / (len(sample) * topk), on_edges - at_random


def bf16_agreement(got, ref):
    """(share of identical elements, mean difference in bfloat16 steps, share of elements more than two steps apart)
    of two float32 arrays of bfloat16 values.  A step is 2^-7 of max(|ref element|, rms of its row): elements near zero
    are measured on their row's scale."""
    steps = scaled_error(got, ref) / 2.0 ** -7
    return float((got == ref).mean()), float(steps.mean()), float((steps > 2.001).mean())
