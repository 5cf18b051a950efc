"""GPU parity: the HIP path against the CPU oracle on the same seeded inputs, through the C ABI.
Integer decisions bit-exact; embeddings after strict-order training within 1e-4 (scaled per row)."""
import numpy as np
import pytest
import torch

from paper_2312_07743_amd import binding as B
from paper_2312_07743_amd import synth
from util import assert_no_further_from_fp64_than_fp32_oracle, assert_rows_close, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def test_cross_lane_reduction_unit():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(60, 64)).astype(np.float32)
    d_in = torch.as_tensor(x).cuda()
    d_out = torch.zeros(64, dtype=torch.float32, device="cuda")
    B.w2v_debug_reduce(d_in, d_out, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy()[:60]
    assert np.allclose(got, x.astype(np.float64).sum(axis=1), rtol=0, atol=2e-5)


@pytest.mark.parametrize("V,d", [(300, 128), (77, 300), (50, 64)])
def test_initial_weights_bit_exact(orc32, V, d):
    from paper_2312_07743_amd.trainer import Trainer
    tr = Trainer(vocab=V, dim=d, window=2, negatives=2, counts=np.ones(V, np.uint64), tokens_per_epoch=10, seed=1234,
                 table_size=256)
    ref0, ref1 = orc32.init_weights(1234, V, d)
    assert np.array_equal(tr.embeddings(0), ref0) and np.array_equal(tr.embeddings(1), ref1)
    torch.cuda.synchronize()
    assert float(tr.syn0[:, d:].abs().sum()) == 0.0          # padding columns are zero
    tr.close()


@pytest.mark.parametrize("case", ["tiny", "subsampled", "odd_table"])
def test_integer_decisions_bit_exact(orc32, case):
    from paper_2312_07743_amd.trainer import Trainer
    if case == "tiny":
        c, kw = synth.zipf_corpus(1000, 1.0, 100, 1000, seed=7), dict(window=5, negatives=5, table_size=1 << 24, t=0.0, ep=0, first=0, E=1)
    elif case == "subsampled":
        c, kw = synth.planted_corpus(vocab=5000, n_sent=40, sent_len=700, seed=2, band_start=300, min_count=2), \
            dict(window=5, negatives=10, table_size=1 << 20, t=1e-3, ep=2, first=123456789012, E=3)
    else:
        c, kw = synth.zipf_corpus(333, 1.2, 17, 301, seed=9), dict(window=10, negatives=3, table_size=100003, t=1e-2, ep=1, first=5, E=2)
    tok = c.tokens.copy()
    tok[5] = -3
    tok[11] = c.vocab + 4                                     # invalid ids are dropped
    T = len(tok) + kw["first"]
    tr = Trainer(vocab=c.vocab, dim=64, window=kw["window"], negatives=kw["negatives"], counts=c.counts,
                 tokens_per_epoch=T, seed=99, table_size=kw["table_size"], subsample_t=kw["t"], total_epochs=kw["E"])
    tr.set_corpus(tok, c.sent_off)
    keep, width, neg = tr.draws(epoch=kw["ep"], first_token_global_pos=kw["first"])
    tr.close()
    syn0, syn1 = orc32.init_weights(1, c.vocab, 4)
    r = orc32.train_epoch(syn0, syn1, c.counts, tok, c.sent_off, window=kw["window"], negatives=kw["negatives"], seed=99,
                          epoch=kw["ep"], total_epochs=kw["E"], tokens_per_epoch=T, first_token_global_pos=kw["first"],
                          table_size=kw["table_size"], subsample_t=kw["t"], dump=True)
    assert np.array_equal(keep, r["keep"]) and keep[5] == 0 and keep[11] == 0
    assert np.array_equal(width, r["width"])
    assert np.array_equal(neg, r["neg"])
    if kw["t"] > 0:
        assert 0.2 < keep.mean() < 0.98


def _parity(orc32, corpus, tol=1e-4, unit_shift=None, **kw):
    g0, g1, gl, gp = run_gpu(corpus, sentences_in_flight=1, unit_shift=unit_shift, **kw)
    r0, r1, rl, rp = run_oracle(orc32, corpus, **kw)
    assert gp == rp, (gp, rp)
    assert abs(gl - rl) <= 2e-5 * abs(rl) + 1e-9, (gl, rl)
    w0 = assert_rows_close(g0, r0, tol, "syn0")
    w1 = assert_rows_close(g1, r1, tol, "syn1neg")
    return max(w0, w1)


def test_tiny_config_strict_order_matches_oracle(orc32, orc64):
    """configs[0]: vocab 1000 Zipf(1.0), 100 sentences x 1000 tokens, d=128, W=5, N=5, no subsampling.  Gated against
    the fp32 oracle (every element within 2e-4, all but 1 in 10,000 within 1e-4) and against the fp64 oracle: the HIP
    path may be no further from it than 1.5 times the fp32 oracle is (the distance tests/test_oracle_pins.py pins)."""
    c = synth.zipf_corpus(1000, 1.0, 100, 1000, seed=7)
    kw = dict(dim=128, window=5, negatives=5, seed=42, table_size=1 << 24)
    g0, g1, gl, gp = run_gpu(c, sentences_in_flight=1, **kw)
    r0, r1, rl, rp = run_oracle(orc32, c, **kw)
    d0, d1, dl, dp = run_oracle(orc64, c, **kw)
    assert gp == rp == dp
    assert abs(gl - rl) <= 2e-5 * abs(rl) and abs(gl - dl) <= 2e-5 * abs(dl)
    worst = max(assert_rows_close(g0, r0, 1e-4, "syn0"), assert_rows_close(g1, r1, 1e-4, "syn1neg"))
    far0 = assert_no_further_from_fp64_than_fp32_oracle(g0, r0, d0, 1.5, "syn0")
    far1 = assert_no_further_from_fp64_than_fp32_oracle(g1, r1, d1, 1.5, "syn1neg")
    print("tiny: worst scaled error against the fp32 oracle", worst, "; (HIP, fp32 oracle) from the fp64 oracle:", far0, far1)


@pytest.mark.parametrize("dim", [64, 100, 256, 300, 512])
def test_row_lengths_of_the_dimension_sweep(orc32, dim):
    c = synth.planted_corpus(vocab=3000, n_sent=12, sent_len=400, seed=5, band_start=200, n_clusters=4,
                             cluster_size=20, min_count=2)
    _parity(orc32, c, dim=dim, window=5, negatives=5, seed=3, subsample_t=1e-3)


@pytest.mark.parametrize("window,negatives,mode", [(1, 0, 0), (2, 1, 0), (5, 10, 0), (10, 5, 0), (16, 20, 0),
                                                   (5, 5, 1), (10, 5, 1), (3, 7, 0)])
def test_window_and_negative_ranges(orc32, window, negatives, mode):
    c = synth.zipf_corpus(400, 1.0, 9, 333, seed=window * 100 + negatives)
    _parity(orc32, c, dim=128, window=window, negatives=negatives, seed=8, window_mode=mode, table_size=50021)


def test_large_like_hyperparameters(orc32):
    """configs[3] in small: Zipf(1.1), d=300 (rows padded to 320 floats), W=5, N=10 (two batches of output rows
    per window), heavy subsampling."""
    c = synth.zipf_corpus(5000, 1.1, 60, 1000, seed=31)
    _parity(orc32, c, dim=300, window=5, negatives=10, seed=17, subsample_t=1e-5, table_size=1 << 20)
    _parity(orc32, c, dim=300, window=5, negatives=10, seed=17, subsample_t=1e-3, table_size=1 << 20)


def test_graph_like_hyperparameters(orc32):
    """configs[4] in small: uniform walks of 80 on a Barabasi-Albert graph (ids not sorted by frequency, walks
    revisit nodes), d=128, W=10, N=5, no subsampling."""
    c = synth.barabasi_albert_walks(n_nodes=3000, m=5, walks_per_node=1, walk_len=80, seed=4)
    _parity(orc32, c, dim=128, window=10, negatives=5, seed=23, table_size=1 << 18)
    _parity(orc32, c, dim=128, window=10, negatives=5, seed=23, table_size=1 << 18, window_mode=1)


def test_fixed_width_sizes_the_ring_by_the_fixed_width(orc32):
    # W=16 with rows of 512 floats is only possible because the widest window is ceil(16/2) = 8
    c = synth.zipf_corpus(300, 1.0, 5, 200, seed=12)
    _parity(orc32, c, dim=512, window=16, negatives=4, seed=5, window_mode=1, table_size=50021)


@pytest.mark.parametrize("unit_shift", [1, 2, 3, 6, 12])
def test_sentences_cut_into_units_of_work(orc32, unit_shift):
    """A sentence handed out as 2^k stretches (each with its lead-in and lead-out context) must train exactly
    the windows of the whole sentence: one wavefront taking the units in order reproduces the oracle."""
    rng = np.random.default_rng(4)
    lens = [1000, 0, 1, 2, 7, 63, 64, 65, 129, 700, 5, 999]          # stretches shorter than a window too
    tok = rng.zipf(1.3, size=sum(lens)).astype(np.int64)
    tok = np.where(tok > 300, rng.integers(0, 300, size=tok.size), tok - 1).astype(np.int32)
    tok[17] = -5                                                     # an invalid id is counted once, not per unit
    off = np.cumsum([0] + lens).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok[tok >= 0], minlength=300).astype(np.uint64))
    for t, window in ((0.0, 5), (3e-2, 5), (3e-2, 10), (0.3, 2)):
        _parity(orc32, c, dim=128, window=window, negatives=5, seed=9, subsample_t=t, table_size=50021,
                unit_shift=unit_shift)


@pytest.mark.parametrize("unit_shift,fine_shift,coarse", [(None, 3, 5), (1, 4, 9), (2, 0, 3), (0, 6, 0), (3, 5, 12),
                                                         (1, 2, 100)])
def test_queue_that_ends_in_smaller_units(orc32, unit_shift, fine_shift, coarse):
    """The sentences from index `coarse` on are cut into 2^fine_shift stretches, the ones before into 2^unit_shift
    (what lock-free launches do with their last sentences so that the wavefronts finish together): in strict
    order the result is still the oracle's."""
    rng = np.random.default_rng(14)
    lens = [300, 0, 1, 700, 2, 64, 65, 129, 0, 500, 5, 999]
    tok = rng.integers(0, 200, size=sum(lens)).astype(np.int32)
    tok[[3, 1500]] = 7777
    off = np.cumsum([0] + lens).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok[tok < 200], minlength=200).astype(np.uint64))
    for t, window, block in ((0.0, 5, 0), (3e-2, 10, 0), (3e-2, 5, 8)):
        g = run_gpu(c, sentences_in_flight=1, unit_shift=unit_shift, unit_tail=(fine_shift, coarse), dim=128,
                    window=window, negatives=5, seed=19, subsample_t=t, table_size=50021, negative_block=block)
        r = run_oracle(orc32, c, dim=128, window=window, negatives=5, seed=19, subsample_t=t, table_size=50021,
                       negative_block=block)
        assert g[3] == r[3] and abs(g[2] - r[2]) <= 2e-5 * abs(r[2])
        assert_rows_close(g[0], r[0], 1e-4, "syn0")
        assert_rows_close(g[1], r[1], 1e-4, "syn1neg")


def test_units_do_not_change_counters():
    from paper_2312_07743_amd.trainer import Trainer
    c = synth.planted_corpus(vocab=3000, n_sent=40, sent_len=777, seed=5, band_start=200, n_clusters=4,
                             cluster_size=20, min_count=2)
    tok = c.tokens.copy()
    tok[::501] = -1
    seen = []
    for shift in (0, 2, 5):
        tr = Trainer(vocab=c.vocab, dim=64, window=5, negatives=3, counts=c.counts, tokens_per_epoch=c.n_tokens, seed=3,
                     table_size=1 << 14, subsample_t=1e-3)
        tr.set_corpus(tok, c.sent_off)
        B.w2v_debug_set_units(tr.ctx, shift)
        tr.train_epoch(0)
        seen.append((tr.counters(), tr.loss()[1]))
        tr.close()
    assert seen[0] == seen[1] == seen[2] and seen[0][0][1] == len(tok[::501])


@pytest.mark.parametrize("block,window,negatives", [(2, 5, 5), (8, 5, 5), (64, 5, 5), (8, 5, 3), (8, 10, 5), (16, 5, 10),
                                                    (4, 16, 1)])
def test_negatives_shared_by_a_stretch_of_tokens(orc32, block, window, negatives):
    """cfg.negative_block: the windows centred in one stretch of tokens use one set of negatives, whose rows the
    kernel keeps in registers from window to window.  Frequent words make targets hit the shared negatives, short
    and empty sentences end stretches early; strict order must reproduce the oracle."""
    rng = np.random.default_rng(block)
    lens = [900, 0, 1, 130, 66, 2, 700, 17]
    tok = rng.zipf(1.25, size=sum(lens)).astype(np.int64)
    tok = np.where(tok > 400, rng.integers(0, 400, size=tok.size), tok - 1).astype(np.int32)
    off = np.cumsum([0] + lens).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok, minlength=400).astype(np.uint64))
    # (without subsampling the few shared rows take so many updates in a row that fp32 rounding alone moves them
    #  by 1e-4 to 4e-4 at the usual learning rate, fp32 against fp64 oracle; a smaller rate keeps that at 2e-5)
    for t, shift, lr0 in ((0.0, None, 0.005), (2e-2, None, 0.025), (2e-2, 2, 0.025)):
        _parity(orc32, c, dim=128, window=window, negatives=negatives, seed=13, subsample_t=t, table_size=50021,
                negative_block=block, unit_shift=shift, lr0=lr0)


def test_negative_block_draws_bit_exact(orc32):
    from paper_2312_07743_amd.trainer import Trainer
    c = synth.zipf_corpus(333, 1.2, 17, 301, seed=9)
    tr = Trainer(vocab=c.vocab, dim=64, window=5, negatives=4, counts=c.counts, tokens_per_epoch=c.n_tokens, seed=99,
                 table_size=100003, subsample_t=1e-2, total_epochs=2, negative_block=16)
    tr.set_corpus(c.tokens, c.sent_off)
    keep, width, neg = tr.draws(epoch=1)
    tr.close()
    syn0, syn1 = orc32.init_weights(1, c.vocab, 4)
    r = orc32.train_epoch(syn0, syn1, c.counts, c.tokens, c.sent_off, window=5, negatives=4, seed=99, epoch=1,
                          total_epochs=2, table_size=100003, subsample_t=1e-2, dump=True, negative_block=16)
    assert np.array_equal(keep, r["keep"]) and np.array_equal(width, r["width"]) and np.array_equal(neg, r["neg"])


@pytest.mark.parametrize("dim,window,negatives", [(320, 16, 20), (299, 16, 7), (512, 10, 20), (1, 3, 2), (7, 16, 12),
                                                  (260, 5, 11), (64, 16, 6), (321, 10, 5), (511, 7, 13), (450, 5, 20)])
def test_extreme_shapes(orc32, dim, window, negatives):
    # largest rings and row counts the limits allow, row lengths at the edges of the lane layouts
    c = synth.zipf_corpus(500, 1.0, 6, 250, seed=dim + window)
    _parity(orc32, c, dim=dim, window=window, negatives=negatives, seed=4, table_size=50021, subsample_t=5e-2)


def test_degenerate_vocabularies_and_schedules(orc32):
    # one word: every negative equals the target (all masked) and every context word is the target's own word
    tok = np.zeros(300, np.int32)
    c1 = synth.Corpus(tok, np.array([0, 100, 300], np.uint64), np.array([300], np.uint64))
    _parity(orc32, c1, dim=64, window=3, negatives=4, seed=1, table_size=17)
    # two words, one of them never sampled as a negative (count 0 owns no table slot)
    tok = np.array([0, 1] * 200, np.int32)
    c2 = synth.Corpus(tok, np.array([0, 400], np.uint64), np.array([400, 0], np.uint64))
    _parity(orc32, c2, dim=128, window=5, negatives=5, seed=2, table_size=64)
    # only invalid ids: nothing is trained, nothing is written
    c3 = synth.Corpus(np.full(500, -7, np.int32), np.array([0, 250, 500], np.uint64), np.array([1, 1, 1], np.uint64))
    _parity(orc32, c3, dim=128, window=5, negatives=5, seed=3, table_size=64)
    # the last epoch of a long schedule: the learning rate sits on its floor for the later sentences
    c4 = synth.zipf_corpus(300, 1.0, 8, 300, seed=6)
    _parity(orc32, c4, dim=128, window=5, negatives=5, seed=4, table_size=4099, epochs=1, start_epoch=9, total_epochs=10,
            lr0=0.05)


def test_degenerate_sentences(orc32):
    # empty sentences, one-word sentences, sentences of invalid ids only, a long sentence (> one FIFO refill)
    rng = np.random.default_rng(3)
    parts = [[], [5], [-1, -1, 999999], [3, 3, 3, 3], [], list(rng.integers(0, 50, size=2500)), [7, 8], []]
    tok = np.array([t for p in parts for t in p], np.int32)
    off = np.cumsum([0] + [len(p) for p in parts]).astype(np.uint64)
    counts = np.bincount(tok[(tok >= 0) & (tok < 50)], minlength=50).astype(np.uint64)
    c = synth.Corpus(tok, off, counts)
    _parity(orc32, c, dim=128, window=5, negatives=5, seed=5, table_size=4099)
    _parity(orc32, c, dim=128, window=5, negatives=5, seed=5, table_size=4099, subsample_t=2e-2)


def test_corpus_passed_as_one_long_sentence(orc32):
    """Ignoring sentence delimiters (the other half of the paper's own window variant, Section 3.2) means passing the
    corpus as one sentence: 12,000 tokens, far more than the kept-token FIFO or one sampling chunk holds, with random
    and with fixed window widths, subsampled, as one unit of work and cut into 8 and into 64 stretches (each stretch
    reads the W kept tokens on either side as context only, so the windows are those of the whole sentence)."""
    c0 = synth.zipf_corpus(800, 1.05, 12, 1000, seed=21)
    one = synth.Corpus(c0.tokens, np.array([0, c0.n_tokens], np.uint64), c0.counts)
    for window_mode in (0, 1):
        kw = dict(dim=128, window=5, negatives=5, seed=9, table_size=1 << 16, subsample_t=5e-3, window_mode=window_mode)
        _parity(orc32, one, unit_shift=0, **kw)
        _parity(orc32, one, unit_shift=3, **kw)
        _parity(orc32, one, unit_shift=6, **kw)
    # the same tokens with delimiters train other windows: the delimiters matter
    r_one = run_oracle(orc32, one, dim=128, window=5, negatives=5, seed=9, table_size=1 << 16, subsample_t=5e-3)
    r_cut = run_oracle(orc32, c0, dim=128, window=5, negatives=5, seed=9, table_size=1 << 16, subsample_t=5e-3)
    assert r_one[3] > r_cut[3]


@pytest.mark.parametrize("shape", [dict(dim=128, window=10, negatives=5), dict(dim=300, window=5, negatives=10),
                                   dict(dim=300, window=9, negatives=5), dict(dim=100, window=10, negatives=7)])
def test_shapes_that_sample_32_windows_at_a_time(orc32, shape):
    """Rows of five floats per lane, and rows of two floats per lane with windows up to 10, sample 32 instead of 64
    windows at a time into a kept-token FIFO of 128 entries (their ring leaves less LDS): one sentence of 6,000 tokens
    (the FIFO wraps about fifty times), subsampled, as one unit and cut into 16 stretches, and ragged short sentences
    around the chunk size."""
    c0 = synth.zipf_corpus(600, 1.05, 6, 1000, seed=33)
    one = synth.Corpus(c0.tokens, np.array([0, c0.n_tokens], np.uint64), c0.counts)
    kw = dict(seed=19, table_size=1 << 16, subsample_t=5e-3, **shape)
    _parity(orc32, one, unit_shift=0, **kw)
    _parity(orc32, one, unit_shift=4, **kw)
    rng = np.random.default_rng(5)
    lens = [31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 1, 0, 2, 160, 400]
    tok = rng.integers(0, 200, size=sum(lens)).astype(np.int32)
    off = np.cumsum([0] + lens).astype(np.uint64)
    ragged = synth.Corpus(tok, off, np.bincount(tok, minlength=200).astype(np.uint64))
    _parity(orc32, ragged, seed=23, table_size=4099, **shape)


def test_repeated_context_words(orc32):
    # walks that step back and stay: most windows hold a word at several context positions (one ring row,
    # counted with its multiplicity); a run of one word fills more than 15 slots of a wide window
    rng = np.random.default_rng(8)

    def walk(n, V):
        out = [int(rng.integers(0, V))]
        for _ in range(n - 1):
            r = rng.random()
            if r < 0.35 and len(out) >= 2:
                out.append(out[-2])
            elif r < 0.45:
                out.append(out[-1])
            else:
                out.append(int(rng.integers(0, V)))
        return out

    parts = [walk(120, 200) for _ in range(6)] + [[7] * 40, [1, 2] * 25]
    tok = np.array([t for p in parts for t in p], np.int32)
    off = np.cumsum([0] + [len(p) for p in parts]).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok, minlength=200).astype(np.uint64))
    for window, negatives in ((10, 5), (16, 3), (5, 10)):
        _parity(orc32, c, dim=128, window=window, negatives=negatives, seed=2, table_size=4099)


def test_second_epoch_and_split_feeding(orc32):
    # epoch index and first_token_global_pos enter the random keys and the learning rate
    c = synth.zipf_corpus(200, 1.0, 6, 300, seed=1)
    kw = dict(dim=128, window=5, negatives=5, seed=77, table_size=1 << 14)
    _parity(orc32, c, epochs=2, **kw)
    _parity(orc32, c, epochs=1, start_epoch=1, total_epochs=3, first_token_global_pos=40000,
            tokens_per_epoch=100000, **kw)


def test_disjoint_vocabulary_slices_run_concurrently_without_conflicts(orc32):
    # every sentence owns its words and N = 0: no two wavefronts touch the same row, so full
    # concurrency must reproduce the serial oracle (whole sentences as units of work: stretches of one
    # sentence share its words)
    c = synth.disjoint_slice_corpus(vocab=6400, n_sent=640, sent_len=150, seed=4)
    kw = dict(dim=128, window=5, negatives=0, seed=6, table_size=1 << 14)
    g0, g1, gl, gp = run_gpu(c, sentences_in_flight=0, unit_shift=0, **kw)
    r0, r1, rl, rp = run_oracle(orc32, c, **kw)
    assert gp == rp and abs(gl - rl) <= 2e-5 * rl
    assert_rows_close(g0, r0, 1e-4, "syn0")
    assert_rows_close(g1, r1, 1e-4, "syn1neg")


def test_untouched_rows_and_padding_stay_bit_identical(orc32):
    from paper_2312_07743_amd.trainer import Trainer
    c = synth.zipf_corpus(100, 1.0, 8, 250, seed=2)
    V, d = 160, 100                                            # ids 100..159 never occur and own no table slot
    counts = np.concatenate([c.counts, np.zeros(60, np.uint64)])
    rng = np.random.default_rng(0)
    s0 = rng.normal(scale=0.1, size=(V, d)).astype(np.float32)
    s1 = rng.normal(scale=0.1, size=(V, d)).astype(np.float32)
    tr = Trainer(vocab=V, dim=d, window=5, negatives=5, counts=counts, tokens_per_epoch=c.n_tokens, seed=3,
                 table_size=1 << 12, syn0=s0, syn1neg=s1)
    tr.syn0[:, d:] = 7.0                                       # whatever sits in the padding must survive
    tr.syn1neg[:, d:] = -7.0
    tr.set_corpus(c.tokens, c.sent_off)
    tr.train_epoch(0)
    a0, a1 = tr.embeddings(0), tr.embeddings(1)
    assert np.array_equal(a0[100:], s0[100:]) and np.array_equal(a1[100:], s1[100:])
    assert not np.array_equal(a0[:100], s0[:100])
    assert bool((tr.syn0[:, d:] == 7.0).all()) and bool((tr.syn1neg[:, d:] == -7.0).all())
    tr.close()


def test_no_reuse_comparator_kernel_matches_the_classic_pair_order(orc32):
    # the traffic comparator executes the original word2vec loop order; checked so that its byte counts
    # belong to a correct trainer
    c = synth.zipf_corpus(300, 1.0, 6, 400, seed=12)
    kw = dict(dim=128, window=5, negatives=5, seed=9, table_size=1 << 14, subsample_t=1e-2)
    g0, g1, gl, gp = run_gpu(c, sentences_in_flight=1, naive=True, **kw)
    r0, r1, rl, rp = run_oracle(orc32, c, update_mode=2, **kw)
    assert gp == rp and abs(gl - rl) <= 2e-5 * rl
    assert_rows_close(g0, r0, 1e-4, "syn0")
    assert_rows_close(g1, r1, 1e-4, "syn1neg")
    c = synth.zipf_corpus(200, 1.0, 4, 300, seed=13)
    kw = dict(dim=300, window=3, negatives=7, seed=9, table_size=1 << 14)
    g0, g1, gl, gp = run_gpu(c, sentences_in_flight=1, naive=True, **kw)
    r0, r1, rl, rp = run_oracle(orc32, c, update_mode=2, **kw)
    assert gp == rp
    assert_rows_close(g0, r0, 1e-4, "syn0")
    assert_rows_close(g1, r1, 1e-4, "syn1neg")
