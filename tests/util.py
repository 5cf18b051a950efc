"""Helpers shared by the GPU parity tests."""
import numpy as np


def run_oracle(orc, corpus, *, dim, window, negatives, seed, epochs=1, table_size=1 << 16, subsample_t=0.0,
               window_mode=0, lr0=0.025, syn0=None, syn1neg=None, first_token_global_pos=0, tokens_per_epoch=None,
               total_epochs=None, start_epoch=0, update_mode=0, negative_block=0):
    if syn0 is None:
        syn0, syn1neg = orc.init_weights(seed, corpus.vocab, dim)
    else:
        syn0, syn1neg = syn0.copy(), syn1neg.copy()
    total_epochs = total_epochs or epochs
    loss = pairs = 0
    for e in range(start_epoch, start_epoch + epochs):
        r = orc.train_epoch(syn0, syn1neg, corpus.counts, corpus.tokens, corpus.sent_off, window=window,
                            negatives=negatives, seed=seed, epoch=e, total_epochs=total_epochs, table_size=table_size,
                            subsample_t=subsample_t, window_mode=window_mode, lr0=lr0, update_mode=update_mode,
                            first_token_global_pos=first_token_global_pos, tokens_per_epoch=tokens_per_epoch,
                            negative_block=negative_block)
        loss += r["loss_sum"]
        pairs += r["pairs"]
    return syn0, syn1neg, loss, pairs


def run_gpu(corpus, *, dim, window, negatives, seed, epochs=1, table_size=1 << 16, subsample_t=0.0, window_mode=0,
            lr0=0.025, sentences_in_flight=0, syn0=None, syn1neg=None, first_token_global_pos=0,
            tokens_per_epoch=None, total_epochs=None, start_epoch=0, naive=False, unit_shift=None, negative_block=0,
            unit_tail=None):
    from paper_2312_07743_amd import binding
    from paper_2312_07743_amd.trainer import Trainer
    tr = Trainer(vocab=corpus.vocab, dim=dim, window=window, negatives=negatives, counts=corpus.counts,
                 tokens_per_epoch=tokens_per_epoch or corpus.n_tokens, seed=seed, table_size=table_size,
                 subsample_t=subsample_t, total_epochs=total_epochs or epochs, sentences_in_flight=sentences_in_flight,
                 window_mode=window_mode, lr0=lr0, syn0=syn0, syn1neg=syn1neg, negative_block=negative_block)
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


def assert_rows_close(got, ref, tol=1e-4, what=""):
    """|delta_ij| <= tol * max(|ref_ij|, rms(ref_row_i)): relative per element, with the row's own scale
    as the floor so that elements that happen to be near zero do not make the test meaningless.

    One Tiny epoch is 100,000 dependent fp32 updates: the fp32 oracle itself sits 0.95e-4 (same measure)
    from its own fp64 build, so two correct fp32 evaluations that merely sum in a different order can be
    up to about 2e-4 apart on a few elements.  The gate is therefore: every element within 2*tol, and all
    but at most one element in 10,000 within tol."""
    ref = ref.astype(np.float64)
    got = got.astype(np.float64)
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    scaled = np.abs(got - ref) / np.maximum(np.maximum(np.abs(ref), rms), 1e-300)
    worst = float(scaled.max())
    over = int((scaled > tol).sum())
    assert worst <= 2 * tol, f"{what}: worst scaled error {worst:.3e} (limit {2 * tol})"
    assert over <= 1e-4 * scaled.size, f"{what}: {over} of {scaled.size} elements beyond {tol}, worst {worst:.3e}"
    return worst


def planted_score(emb, labels, topk=10):
    """Mean, over the planted words, of the share of their topk cosine neighbours in their own cluster."""
    idx = np.flatnonzero(labels >= 0)
    e = emb / np.maximum(np.linalg.norm(emb, axis=1, keepdims=True), 1e-30)
    sims = e[idx] @ e.T
    sims[np.arange(len(idx)), idx] = -np.inf
    nn = np.argpartition(-sims, topk, axis=1)[:, :topk]
    return float((labels[nn] == labels[idx][:, None]).mean())
