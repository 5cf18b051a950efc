"""Pins of the oracle's epoch loop: which windows and contexts a sentence yields (closed
forms at syn1neg = 0), invariants, a negative control on window order, and convergence to
the brute-force co-occurrence statistics of an 8-word toy corpus."""
import math

import numpy as np
import pytest

from paper_2312_07743_amd import synth


def _sigmoid(x):
    return 1.0 / (1.0 + math.exp(-x))


def _one_sentence(words):
    return np.array(words, np.int32), np.array([0, len(words)], np.uint64)


def test_three_distinct_words_closed_form(orc64):
    # W=1 (width always 1), N=0, syn1neg=0: every dot product is 0, g = alpha/2, syn0 never moves.
    V, d = 5, 3
    rng = np.random.default_rng(0)
    syn0 = rng.normal(size=(V, d))
    s0 = syn0.copy()
    syn1 = np.zeros((V, d))
    tok, off = _one_sentence([1, 3, 4])
    r = orc64.train_epoch(syn0, syn1, np.ones(V, np.uint64), tok, off, window=1, negatives=0,
                          seed=1, lr0=0.5, lr_min_frac=1.0)
    a = 0.5
    want = np.zeros((V, d))
    want[1] = 0.5 * a * s0[3]                 # centre 1: context {3}
    want[3] = 0.5 * a * (s0[1] + s0[4])       # centre 3: context {1,4}
    want[4] = 0.5 * a * s0[3]                 # centre 4: context {3} (window cut at the sentence end)
    assert np.array_equal(syn0, s0)
    assert np.allclose(syn1, want, rtol=0, atol=1e-16)
    assert r["pairs"] == 4 and r["loss_sum"] == pytest.approx(4 * math.log(2))


def test_repeated_word_sentence_follows_window_order(orc64):
    # sentence a b a, W=1, N=0.  The third window sees the output row the first one wrote.
    d, a = 2, 0.4
    Ia, Ib = np.array([1.0, 2.0]), np.array([0.5, -1.0])
    syn0 = np.stack([Ia, Ib]).copy()
    syn1 = np.zeros((2, d))
    tok, off = _one_sentence([0, 1, 0])
    orc64.train_epoch(syn0, syn1, np.ones(2, np.uint64), tok, off, window=1, negatives=0,
                      seed=1, lr0=a, lr_min_frac=1.0)
    Oa = 0.5 * a * Ib                          # window 1: centre a, context b
    Ob = 0.5 * a * (Ia + Ia)                   # window 2: centre b, contexts a, a (output row b was 0)
    x = float(Ib @ Oa)                         # window 3: centre a, context b
    g = a * (1 - _sigmoid(x))
    want_b = Ib + g * Oa
    want_Oa = Oa + g * Ib
    assert np.allclose(syn0[0], Ia, atol=1e-16)          # a only ever met zero output rows
    assert np.allclose(syn0[1], want_b, atol=1e-15)
    assert np.allclose(syn1[0], want_Oa, atol=1e-15) and np.allclose(syn1[1], Ob, atol=1e-15)


def test_windows_do_not_cross_sentences_and_dropped_tokens_close_the_gap(orc64):
    V, d = 6, 2
    syn0 = np.arange(V * d, dtype=np.float64).reshape(V, d) + 1
    s0 = syn0.copy()
    syn1 = np.zeros((V, d))
    # two sentences; token -1 and token 99 are invalid ids and behave like subsampled words
    tok = np.array([0, -1, 1, 99, 2, 3, 4], np.int32)
    off = np.array([0, 5, 7], np.uint64)
    r = orc64.train_epoch(syn0, syn1, np.ones(V, np.uint64), tok, off, window=1, negatives=0,
                          seed=3, lr0=1.0, lr_min_frac=1.0, dump=True)
    assert list(r["keep"]) == [1, 0, 1, 0, 1, 1, 1]
    want = np.zeros((V, d))
    want[0] = 0.5 * s0[1]
    want[1] = 0.5 * (s0[0] + s0[2])            # 0 and 2 are neighbours of 1 once the invalid ids are gone
    want[2] = 0.5 * s0[1]
    want[3] = 0.5 * s0[4]                      # second sentence: 3 and 4 only see each other
    want[4] = 0.5 * s0[3]
    assert np.allclose(syn1, want, atol=1e-16)
    assert r["pairs"] == 6


def test_dumps_agree_with_the_scalar_functions_and_single_word_sentences_do_nothing(orc32):
    c = synth.zipf_corpus(50, 1.0, 6, 40, seed=4)
    tok = np.concatenate([c.tokens, [7]]).astype(np.int32)       # a last sentence of one word
    off = np.concatenate([c.sent_off, [len(tok)]]).astype(np.uint64)
    counts = np.bincount(tok, minlength=50).astype(np.uint64)
    syn0, syn1 = orc32.init_weights(3, 50, 8)
    N, W, tsz, seed, ep, first = 4, 3, 4096, 21, 2, 1000
    r = orc32.train_epoch(syn0, syn1, counts, tok, off, window=W, negatives=N, seed=seed, epoch=ep,
                          total_epochs=3, first_token_global_pos=first, table_size=tsz,
                          subsample_t=5e-2, dump=True)
    thr = orc32.thresholds(counts, 5e-2)
    end = orc32.table_ends(counts, tsz)
    assert 0 < r["keep"].sum() < len(tok)
    for t in range(len(tok)):
        k = orc32.keep(thr, int(tok[t]), seed, ep, first + t)
        assert r["keep"][t] == k
        if k:
            assert r["width"][t] == orc32.width(W, 0, seed, ep, first + t)
            assert list(r["neg"][t]) == [orc32.negative(end, tsz, seed, ep, first + t, j) for j in range(N)]
        else:
            assert r["width"][t] == 0 and np.all(r["neg"][t] == -1)


def test_rows_of_unseen_words_stay_bit_identical(orc32):
    V, d = 200, 16
    c = synth.zipf_corpus(100, 1.0, 5, 200, seed=8)               # ids 100..199 never occur
    counts = np.concatenate([c.counts, np.zeros(100, np.uint64)])
    syn0, syn1 = orc32.init_weights(1, V, d)
    syn1[:] = np.random.default_rng(1).normal(scale=0.1, size=(V, d)).astype(np.float32)
    a0, a1 = syn0.copy(), syn1.copy()
    orc32.train_epoch(syn0, syn1, counts, c.tokens, c.sent_off, window=5, negatives=5, seed=2, table_size=1 << 16)
    assert np.array_equal(syn0[100:], a0[100:]) and np.array_equal(syn1[100:], a1[100:])
    seen = np.flatnonzero(c.counts > 0)
    assert not np.array_equal(syn0[seen], a0[seen])


def test_first_window_loss_is_six_ln2_per_pair_on_fresh_weights(orc32):
    # syn1neg = 0 at the start: each pairing costs ln 2, so a window costs |C| * (1 + unmasked negatives) * ln 2
    c = synth.zipf_corpus(1000, 1.0, 1, 2, seed=3)                # one sentence of two words -> two windows
    syn0, syn1 = orc32.init_weights(5, 1000, 128)
    big = synth.zipf_corpus(1000, 1.0, 100, 1000, seed=3)
    r = orc32.train_epoch(syn0, syn1, big.counts, c.tokens, c.sent_off, window=5, negatives=5, seed=9,
                          lr0=1e-9, dump=True)
    masked = sum(int(n == c.tokens[t]) for t in range(2) for n in r["neg"][t])
    assert r["pairs"] == 2
    assert r["loss_sum"] == pytest.approx((12 - masked) * math.log(2), rel=1e-6)


def test_swapping_two_windows_changes_the_result(orc32):
    # negative control for strict window order: the same multiset of windows in another order is another result
    V, d = 30, 8
    rng = np.random.default_rng(2)
    syn0 = rng.normal(scale=0.3, size=(V, d)).astype(np.float32)
    syn1 = rng.normal(scale=0.3, size=(V, d)).astype(np.float32)
    w1 = ([1, 2, 3], [4, 5, 6])
    w2 = ([2, 3, 7], [3, 5, 8])
    a0, a1, b0, b1 = syn0.copy(), syn1.copy(), syn0.copy(), syn1.copy()
    orc32.window_step(a0, a1, *w1, 0.2); orc32.window_step(a0, a1, *w2, 0.2)
    orc32.window_step(b0, b1, *w2, 0.2); orc32.window_step(b0, b1, *w1, 0.2)
    assert np.max(np.abs(a0 - b0)) > 1e-5


def test_mean_loss_decreases_over_epochs(orc32):
    c = synth.zipf_corpus(300, 1.0, 20, 500, seed=11)
    syn0, syn1 = orc32.init_weights(4, 300, 32)
    E = 4
    means = []
    for e in range(E):
        r = orc32.train_epoch(syn0, syn1, c.counts, c.tokens, c.sent_off, window=5, negatives=5, seed=6,
                              epoch=e, total_epochs=E, table_size=1 << 16)
        means.append(r["loss_sum"] / r["pairs"])
    assert means[0] < 6 * math.log(2) + 1e-3
    assert all(b < a for a, b in zip(means, means[1:])), means


def _toy_markov_corpus(n_tokens, seed):
    """8 words in two groups of four; the next word stays in the group with probability 0.9."""
    rng = np.random.default_rng(seed)
    tok = np.empty(n_tokens, np.int32)
    tok[0] = 0
    stay = rng.random(n_tokens) < 0.9
    pick = rng.integers(0, 4, size=n_tokens)
    for i in range(1, n_tokens):
        g = tok[i - 1] // 4
        if not stay[i]:
            g = 1 - g
        tok[i] = 4 * g + pick[i]
    return tok


def test_toy_vocab8_converges_to_brute_force_cooccurrence_statistics(orc64):
    """At a stationary point of SGNS with negatives equal to the centre dropped,
       exp(<syn0[a], syn1neg[w]>) * N * P_n(w) = P(w|a) / (1 - P(w|a)),
    where P(w|a) is the share of centre word w among the windows that contain a as a context
    word.  P(w|a) is counted by brute force from the corpus (fixed-width windows), i.e. it is
    what an exhaustive full-softmax skip-gram model of the same corpus converges to."""
    V, d, N, W = 8, 8, 4, 4                                    # fixed-width mode: b = ceil(W/2) = 2
    sent_len, n_sent = 200, 40
    tok = _toy_markov_corpus(sent_len * n_sent, 5)
    off = (np.arange(n_sent + 1) * sent_len).astype(np.uint64)
    counts = np.bincount(tok, minlength=V).astype(np.uint64)
    co = np.zeros((V, V))                                      # co[a, w]: a is a context word of centre w
    for s in range(n_sent):
        sent = tok[s * sent_len:(s + 1) * sent_len]
        for i, w in enumerate(sent):
            for j in range(max(0, i - 2), min(sent_len, i + 3)):
                if j != i:
                    co[sent[j], w] += 1
    p_cond = co / co.sum(axis=1, keepdims=True)
    p_n = counts.astype(np.float64) ** 0.75
    p_n /= p_n.sum()
    syn0, syn1 = orc64.init_weights(1, V, d)
    syn0 *= 20
    E = 60
    for e in range(E):
        orc64.train_epoch(syn0, syn1, counts, tok, off, window=W, negatives=N, seed=13, epoch=e,
                          total_epochs=E, table_size=1 << 16, lr0=0.05, window_mode=1)
    x = syn0 @ syn1.T
    r = np.exp(x) * N * p_n[None, :]
    got = r / (1 + r)
    assert np.max(np.abs(got - p_cond)) < 0.02, np.round(got - p_cond, 3)
    # and the same-group structure is what nearest neighbours recover
    sim = (syn0 / np.linalg.norm(syn0, axis=1, keepdims=True))
    cs = sim @ sim.T
    np.fill_diagonal(cs, -2)
    assert all((np.argmax(cs[a]) // 4) == a // 4 for a in range(V))


def test_both_readings_of_the_update_order_reach_the_same_quality(orc32):
    # the paper's claim that the order in which a window's pairings are applied does not matter for quality
    c = synth.planted_corpus(vocab=2000, n_sent=60, sent_len=500, seed=3, n_clusters=4, cluster_size=10,
                             band_start=100, burst_p=0.05, min_count=1)
    res = []
    for mode in (0, 1):
        syn0, syn1 = orc32.init_weights(2, c.vocab, 32)
        for e in range(3):
            r = orc32.train_epoch(syn0, syn1, c.counts, c.tokens, c.sent_off, window=5, negatives=5, seed=4,
                                  epoch=e, total_epochs=3, table_size=1 << 18, update_mode=mode)
        res.append(r["loss_sum"] / r["pairs"])
    assert abs(res[0] - res[1]) / res[0] < 0.02, res


def test_negative_block_shares_the_stretch_start_draws(orc32):
    """Negative reuse over several windows (Section 7 names it as future work): with a block of B tokens every
    window centred in the same stretch of B consecutive tokens of a sentence uses the draws of the stretch's
    first position.  Checked against the scalar draw function at positions computed here, not by the oracle."""
    rng = np.random.default_rng(5)
    lens = [37, 1, 0, 64, 9]
    tok = rng.integers(0, 60, size=sum(lens)).astype(np.int32)
    off = np.cumsum([0] + lens).astype(np.uint64)
    counts = np.bincount(tok, minlength=60).astype(np.uint64)
    V, d, N, tsz, seed, first = 60, 4, 3, 4099, 21, 1000
    end = orc32.table_ends(counts, tsz)
    base = None
    for B in (0, 1, 4, 16):
        syn0, syn1 = orc32.init_weights(3, V, d)
        r = orc32.train_epoch(syn0, syn1, counts, tok, off, window=2, negatives=N, seed=seed, epoch=1, total_epochs=2,
                              first_token_global_pos=first, tokens_per_epoch=5000, table_size=tsz, subsample_t=5e-3,
                              dump=True, negative_block=B)
        if B <= 1:
            if base is None:
                base = (syn0.copy(), syn1.copy(), r["neg"].copy())
            else:                                   # a block of one token is the paper's method, bit for bit
                assert np.array_equal(syn0, base[0]) and np.array_equal(syn1, base[1]) and np.array_equal(r["neg"], base[2])
        assert 0 < r["keep"].sum() < len(tok)
        for s in range(len(lens)):
            for t in range(int(off[s]), int(off[s + 1])):
                if not r["keep"][t]:
                    assert np.all(r["neg"][t] == -1)
                    continue
                o = t - int(off[s])
                start = t if B <= 1 else int(off[s]) + (o // B) * B
                want = [orc32.negative(end, tsz, seed, 1, first + start, k) for k in range(N)]
                assert list(r["neg"][t]) == want
        # keep decisions and widths do not depend on the block
        assert r["width"].max() <= 2


def test_negative_block_hand_case(orc64):
    # Two windows share one negative set: with syn1neg = 0 every dot product of the first window is 0, so the
    # negatives' rows move by -alpha/2 * (sum of its context rows); the second window then sees those rows.
    V, d = 6, 2
    rng = np.random.default_rng(2)
    syn0 = rng.normal(size=(V, d))
    s0 = syn0.copy()
    counts = np.array([0, 0, 0, 0, 5, 7], np.uint64)          # negatives can only be words 4 or 5
    tok, off = _one_sentence([0, 1])
    end = orc64.table_ends(counts, 64)
    syn1 = np.zeros((V, d))
    r = orc64.train_epoch(syn0, syn1, counts, tok, off, window=1, negatives=1, seed=9, lr0=0.5, lr_min_frac=1.0,
                          table_size=64, negative_block=2, dump=True)
    n = orc64.negative(end, 64, 9, 0, 0, 0)                    # the draw of position 0 serves both windows
    assert list(r["neg"][:, 0]) == [n, n]
    a = 0.5
    # window 0: centre 0, context {1}; window 1: centre 1, context {0}
    o_n = -0.5 * a * s0[1]                                     # negative row after window 0
    o_t0 = 0.5 * a * s0[1]
    x = float(s0[0] @ o_n)                                     # window 1 pairs context 0 with the moved negative row
    g = a * (0.0 - _sigmoid(x))
    assert np.allclose(syn1[n], o_n + g * s0[0], rtol=0, atol=1e-15)
    assert np.allclose(syn1[0], o_t0, rtol=0, atol=1e-15)
    assert np.allclose(syn0[0], s0[0] + g * o_n, rtol=0, atol=1e-15)      # context of window 1 moves by g * (old negative row)
