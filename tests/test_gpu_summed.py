"""GPU checks of (1) the window kernel's own integer decisions, written out by the training launch itself,
(2) summed lock-free updates: in strict order (nobody else writes) adding the change to what memory holds must
reproduce the oracle like the overwriting mode does, (3) work plans made on the device from the sizes of the call."""
import numpy as np
import pytest
import torch

from paper_2312_07743_amd import binding as B
from paper_2312_07743_amd import synth
from util import assert_rows_close, run_oracle

pytestmark = pytest.mark.gpu


def _trainer(c, *, dim, window, negatives, seed, **kw):
    from paper_2312_07743_amd.trainer import Trainer
    kw.setdefault("tokens_per_epoch", c.n_tokens)
    kw.setdefault("table_size", 1 << 16)
    return Trainer(vocab=c.vocab, dim=dim, window=window, negatives=negatives, counts=c.counts, seed=seed, **kw)


@pytest.mark.parametrize("case", ["tiny_strict", "tiny_lock_free", "subsampled_far_position", "shared_negatives",
                                  "ten_negatives_units", "three_negatives_wide", "graph_summed"])
def test_training_launch_writes_out_the_oracles_decisions(orc32, case):
    """keep / width / negatives as the window kernel's sampling stage computes them while it trains (not the separate
    draw-dump kernel), against the oracle's dump of the same epoch: bit-exact, in strict order and lock-free, with
    sentences cut into units, with invalid ids, far first positions, shared negatives and every negative path."""
    kw = dict(dim=128, window=5, negatives=5, seed=99, table_size=1 << 20, subsample_t=0.0, total_epochs=1)
    ep, first, in_flight, units, nb, update = 0, 0, 1, None, 0, 0
    if case.startswith("tiny"):
        c = synth.zipf_corpus(1000, 1.0, 100, 1000, seed=7)
        in_flight = 1 if case == "tiny_strict" else 0
    elif case == "subsampled_far_position":
        c = synth.planted_corpus(vocab=5000, n_sent=40, sent_len=700, seed=2, band_start=300, min_count=2)
        kw.update(subsample_t=1e-3, total_epochs=3, negatives=5)
        ep, first, in_flight = 2, 123456789012, 0
    elif case == "shared_negatives":
        c = synth.zipf_corpus(400, 1.1, 30, 500, seed=5)
        kw.update(subsample_t=2e-2)
        nb, in_flight = 4, 0
    elif case == "ten_negatives_units":
        c = synth.zipf_corpus(2000, 1.1, 12, 900, seed=6)
        kw.update(dim=300, negatives=10, subsample_t=1e-2)
        in_flight, units = 3, 2
    elif case == "three_negatives_wide":
        c = synth.zipf_corpus(333, 1.2, 17, 301, seed=9)
        kw.update(dim=64, window=10, negatives=3, table_size=100003, subsample_t=1e-2)
        in_flight = 0
    else:
        c = synth.barabasi_albert_walks(n_nodes=4000, m=5, walks_per_node=2, walk_len=80, seed=4)
        kw.update(window=10)
        in_flight, update = 0, 2
    tok = c.tokens.copy()
    tok[5], tok[11] = -3, c.vocab + 4                         # invalid ids get no window
    T = len(tok) + first
    tr = _trainer(c, tokens_per_epoch=T, sentences_in_flight=in_flight, negative_block=nb, update_mode=update, **kw)
    tr.set_corpus(tok, c.sent_off)
    if units is not None:
        B.w2v_debug_set_units(tr.ctx, units)
    keep, width, neg = tr.train_draws(epoch=ep, first_token_global_pos=first)
    kept, invalid = tr.counters()
    loss, pairs = tr.loss()
    tr.close()
    syn0, syn1 = orc32.init_weights(1, c.vocab, 4)
    r = orc32.train_epoch(syn0, syn1, c.counts, tok, c.sent_off, window=kw["window"], negatives=kw["negatives"],
                          seed=kw["seed"], epoch=ep, total_epochs=kw["total_epochs"], tokens_per_epoch=T,
                          first_token_global_pos=first, table_size=kw["table_size"], subsample_t=kw["subsample_t"],
                          negative_block=nb, dump=True)
    assert np.array_equal(keep, r["keep"]) and keep[5] == 0 and keep[11] == 0
    assert np.array_equal(width, r["width"])
    assert np.array_equal(neg, r["neg"])
    assert kept == int(keep.sum()) and invalid == 2 and pairs == r["pairs"]


@pytest.mark.parametrize("shape", ["graph", "text_d64", "text_d256_n10", "text_d100_fixed_width"])
def test_summed_updates_in_strict_order_match_the_oracle(orc32, shape):
    """With one wavefront nobody else writes, so (what memory holds) + (copy - starting value) is the copy: the
    summed mode, forced on in strict order, must reproduce the oracle within the strict-order tolerance."""
    if shape == "graph":
        c = synth.barabasi_albert_walks(n_nodes=3000, m=5, walks_per_node=1, walk_len=80, seed=4)
        kw = dict(dim=128, window=10, negatives=5, seed=23, table_size=1 << 18)
    elif shape == "text_d64":
        c = synth.zipf_corpus(400, 1.0, 9, 333, seed=3)
        kw = dict(dim=64, window=5, negatives=5, seed=8, table_size=50021, subsample_t=3e-2)
    elif shape == "text_d256_n10":
        c = synth.zipf_corpus(800, 1.1, 8, 500, seed=13)
        kw = dict(dim=256, window=7, negatives=10, seed=5, table_size=1 << 16, subsample_t=1e-2)
    else:
        c = synth.zipf_corpus(300, 1.0, 7, 300, seed=12)
        kw = dict(dim=100, window=9, negatives=6, seed=5, table_size=50021, window_mode=1)
    tr = _trainer(c, sentences_in_flight=1, update_mode=2, **kw)
    tr.set_corpus(c.tokens, c.sent_off)
    B.w2v_debug_set_update(tr.ctx, 1)
    tr.train_epoch(0)
    assert B.w2v_debug_get_plan(tr.ctx)["update"] == 1
    loss, pairs = tr.loss()
    g0, g1 = tr.embeddings(0), tr.embeddings(1)
    tr.close()
    r0, r1, rl, rp = run_oracle(orc32, c, **kw)
    assert pairs == rp and abs(loss - rl) <= 2e-5 * abs(rl)
    assert_rows_close(g0, r0, 1e-4, "syn0")
    assert_rows_close(g1, r1, 1e-4, "syn1neg")


def test_summed_updates_with_units_and_the_flush_at_sentence_ends(orc32):
    """Sentences of every length around the ring size, cut into units, summed mode forced on in strict order: the
    rows that leave at a unit's end go back four at a time."""
    rng = np.random.default_rng(4)
    lens = [1000, 0, 1, 2, 7, 21, 22, 23, 63, 64, 65, 129, 700, 5, 999]
    tok = rng.zipf(1.3, size=sum(lens)).astype(np.int64)
    tok = np.where(tok > 300, rng.integers(0, 300, size=tok.size), tok - 1).astype(np.int32)
    off = np.cumsum([0] + lens).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok, minlength=300).astype(np.uint64))
    for unit_shift, t in ((0, 0.0), (2, 3e-2), (6, 3e-2)):
        kw = dict(dim=128, window=10, negatives=5, seed=9, subsample_t=t, table_size=50021)
        tr = _trainer(c, sentences_in_flight=1, update_mode=2, **kw)
        tr.set_corpus(c.tokens, c.sent_off)
        B.w2v_debug_set_update(tr.ctx, 1)
        B.w2v_debug_set_units(tr.ctx, unit_shift)
        tr.train_epoch(0)
        loss, pairs = tr.loss()
        g0, g1 = tr.embeddings(0), tr.embeddings(1)
        tr.close()
        r0, r1, rl, rp = run_oracle(orc32, c, **kw)
        assert pairs == rp and abs(loss - rl) <= 2e-5 * abs(rl)
        assert_rows_close(g0, r0, 1e-4, "syn0")
        assert_rows_close(g1, r1, 1e-4, "syn1neg")


def test_part_of_an_epoch_is_planned_by_its_own_size():
    """An epoch fed in several lock-free calls: every call's units are cut from the sizes of that call (the token count
    is read on the device), not from the epoch's, so 17 sentences of 1,000 tokens out of a 17M-token epoch become
    units of at least 125 tokens."""
    c = synth.planted_corpus(vocab=20000, s=1.05, n_sent=340, sent_len=1000, seed=3, band_start=500, min_count=1)
    T_epoch = 17_000_000
    kw = dict(dim=128, window=5, negatives=5, seed=5, table_size=1 << 20, subsample_t=1e-3, tokens_per_epoch=T_epoch,
              sentences_in_flight=0)
    off = c.sent_off.astype(np.int64)
    whole = _trainer(c, **kw)
    whole.set_corpus(c.tokens, c.sent_off)
    whole.train_epoch(0)
    plan = B.w2v_debug_get_plan(whole.ctx)
    assert plan["wavefronts"] > 1000 and plan["unit_shift"] == 2 and plan["fine_shift"] == 3
    loss_whole, pairs_whole = whole.loss()
    whole.close()
    parts = _trainer(c, **kw)
    n_units = 0
    for s0 in range(0, c.n_sent, 17):
        s1 = min(c.n_sent, s0 + 17)
        parts.set_corpus(c.tokens[off[s0]:off[s1]], (off[s0:s1 + 1] - off[s0]).astype(np.uint64))
        parts.train_epoch(0, first_token_global_pos=int(off[s0]))
        plan = B.w2v_debug_get_plan(parts.ctx)
        assert plan["unit_shift"] == 2 and plan["fine_shift"] == 3, plan
        assert plan["units"] == ((s1 - s0) - max(1, (s1 - s0) // 8)) * 4 + max(1, (s1 - s0) // 8) * 8
        n_units += plan["units"]
    loss_parts, pairs_parts = parts.loss()
    parts.close()
    assert pairs_parts == pairs_whole                         # draws are keyed by global positions
    # Twenty launches of 76 units each run far fewer sentences side by side than one launch of all 340: they lose
    # fewer updates, so their loss lies between that of strict order and that of the single lock-free call.
    serial = _trainer(c, **dict(kw, sentences_in_flight=1))
    serial.set_corpus(c.tokens, c.sent_off)
    serial.train_epoch(0)
    loss_serial, pairs_serial = serial.loss()
    serial.close()
    assert pairs_serial == pairs_whole
    assert 0.99 * loss_serial <= loss_parts <= 1.01 * loss_whole, (loss_serial, loss_parts, loss_whole)
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------------------------------
# bfloat16 table storage (extension): strict order against the oracle run with the same storage
# ---------------------------------------------------------------------------------------------------------------
def _bf16_parity(orc32, orc64, c, **kw):
    """Both sides round with the same random bits, but the values they round differ in the last fp32 bits (other
    summation order), so now and then a rounding falls the other way: one bfloat16 step, which later roundings of that
    element then see, and the two evaluations drift apart with the length of the run.  The yardstick is the distance
    between two evaluations that are both correct, the fp32 and the fp64 build of the oracle on the same case: the HIP
    path's result carries its own fp32 rounding (another summation order, hardware exp / log / rcp) on top of the fp32
    oracle's, so it may be up to 2.5 times as far from the fp32 oracle as the fp64 build is: in the share of elements
    that differ, in the mean distance in bfloat16 steps, and in the share of elements beyond two steps (+ 0.1 %)."""
    from util import bf16_agreement, run_gpu
    g0, g1, gl, gp = run_gpu(c, sentences_in_flight=1, storage=1, **kw)
    r0, r1, rl, rp = run_oracle(orc32, c, storage=1, **kw)
    d0, d1, dl, dp = run_oracle(orc64, c, storage=1, **kw)
    assert gp == rp == dp and abs(gl - rl) <= 2 * abs(dl - rl) + 1e-4 * abs(rl), (gp, rp, gl, rl, dl)
    out = []
    for got, ref, dbl, name in ((g0, r0, d0, "syn0"), (g1, r1, d1, "syn1neg")):
        assert not np.any(got.view(np.uint32) & 0xFFFF)
        same, mean_steps, far = bf16_agreement(got, ref)
        fsame, fmean, ffar = bf16_agreement(dbl.astype(np.float32), ref)
        assert 1.0 - same <= 2.5 * (1.0 - fsame) + 1e-3 and mean_steps <= 2.5 * fmean + 1e-3 and far <= 2.5 * ffar + 1e-3, \
            (name, (same, mean_steps, far), (fsame, fmean, ffar))
        out.append(((same, mean_steps, far), (fsame, fmean, ffar)))
    return out


def test_bf16_initial_weights_are_the_nearest_bf16_of_the_float_ones(orc32):
    from paper_2312_07743_amd.trainer import Trainer
    V, d = 300, 100
    tr = Trainer(vocab=V, dim=d, window=5, negatives=5, counts=np.ones(V, np.uint64), tokens_per_epoch=10, seed=1234,
                 table_size=256, storage=1)
    ref0, ref1 = orc32.init_weights(1234, V, d, storage=1)
    assert np.array_equal(tr.embeddings(0), ref0) and np.array_equal(tr.embeddings(1), ref1)
    assert float(tr.syn0[:, d:].float().abs().sum()) == 0.0
    tr.close()


@pytest.mark.parametrize("shape", ["d128", "d64_w10", "d128_w10", "d256_n10", "d300_n10_subsampled", "d100_fixed_shared"])
def test_bf16_storage_in_strict_order_matches_the_oracle(orc32, orc64, shape):
    if shape == "d128":
        c = synth.zipf_corpus(500, 1.0, 8, 400, seed=3)
        kw = dict(dim=128, window=5, negatives=5, seed=11, table_size=1 << 16)
    elif shape == "d64_w10":
        c = synth.barabasi_albert_walks(n_nodes=40, m=5, walks_per_node=1, walk_len=80, seed=4)     # a short run: see above
        kw = dict(dim=64, window=10, negatives=5, seed=23, table_size=1 << 18)
    elif shape == "d128_w10":                      # 32 windows sampled at a time, their rounding draws kept in LDS
        c = synth.barabasi_albert_walks(n_nodes=60, m=5, walks_per_node=1, walk_len=80, seed=9)
        kw = dict(dim=128, window=10, negatives=5, seed=29, table_size=1 << 18)
    elif shape == "d256_n10":
        c = synth.zipf_corpus(800, 1.1, 6, 400, seed=13)
        kw = dict(dim=256, window=7, negatives=10, seed=5, table_size=1 << 16)
    elif shape == "d300_n10_subsampled":
        c = synth.zipf_corpus(3000, 1.1, 12, 600, seed=31)
        kw = dict(dim=300, window=5, negatives=10, seed=17, subsample_t=1e-3, table_size=1 << 20)
    else:
        c = synth.zipf_corpus(300, 1.0, 7, 300, seed=12)
        kw = dict(dim=100, window=9, negatives=6, seed=5, table_size=50021, window_mode=1, negative_block=4)
    print(shape, "(identical, mean steps, beyond two steps): HIP vs fp32 oracle, fp64 vs fp32 oracle:", _bf16_parity(orc32, orc64, c, **kw))
