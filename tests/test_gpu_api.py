"""GPU tests of the C ABI's call sequence and error reporting (the argument checks that need a context)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2312_07743_amd import binding as B
from paper_2312_07743_amd import synth

pytestmark = pytest.mark.gpu


def _raw_context(vocab=50, dim=64, table_size=1 << 10):
    ld = B.w2v_query_ld(dim)
    syn0 = torch.zeros((vocab, ld), dtype=torch.float32, device="cuda")
    syn1 = torch.zeros((vocab, ld), dtype=torch.float32, device="cuda")
    nbytes = B.w2v_query_workspace(vocab, table_size)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    cfg = B.make_config(vocab=vocab, dim=dim, window=3, negatives=2, tokens_per_epoch=100, seed=1, syn0=syn0,
                        syn1neg=syn1, ld=ld, workspace=ws, workspace_bytes=nbytes, total_epochs=2,
                        stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return B.w2v_create(cfg, 1), (syn0, syn1, ws)


def test_call_order_and_argument_errors():
    ctx, keep = _raw_context()
    L = B.lib()
    tok = torch.zeros(100, dtype=torch.int32, device="cuda")
    off = torch.tensor([0, 100], dtype=torch.int64, device="cuda")
    # training before the table exists
    assert L.w2v_train_epoch(ctx, tok.data_ptr(), off.data_ptr(), 1, 0, 0) == B.W2V_ESTATE
    assert "w2v_build_unigram_table" in B.w2v_last_error(ctx)
    counts = np.ones(50, np.uint64)
    # a table larger than the workspace was sized for; all-zero counts; null counts
    assert L.w2v_build_unigram_table(ctx, counts.ctypes.data, 1 << 20) == B.W2V_ENOMEM
    assert L.w2v_build_unigram_table(ctx, np.zeros(50, np.uint64).ctypes.data, 1 << 10) == B.W2V_EINVAL
    assert L.w2v_build_unigram_table(ctx, None, 1 << 10) == B.W2V_EINVAL
    assert L.w2v_build_unigram_table(ctx, counts.ctypes.data, 0) == B.W2V_EINVAL
    B.w2v_build_unigram_table(ctx, counts, 1 << 10)
    assert L.w2v_train_epoch(ctx, tok.data_ptr(), off.data_ptr(), 1, 0, 2) == B.W2V_EINVAL      # epoch >= total_epochs
    assert L.w2v_train_epoch(ctx, tok.data_ptr(), off.data_ptr(), 1, 101, 0) == B.W2V_EINVAL    # position beyond the epoch
    assert L.w2v_train_epoch(ctx, None, off.data_ptr(), 1, 0, 0) == B.W2V_EINVAL
    assert L.w2v_train_epoch(ctx, None, None, 0, 0, 0) == B.W2V_OK                              # nothing to do
    assert L.w2v_debug_draws(ctx, tok.data_ptr(), off.data_ptr(), 1, 0, 0, None, None, None) == B.W2V_EINVAL
    assert L.w2v_get_embeddings(ctx, 2, tok.data_ptr(), 10**9, 1) == B.W2V_EINVAL
    assert L.w2v_get_embeddings(ctx, 0, tok.data_ptr(), 10, 1) == B.W2V_EINVAL                  # destination too small
    assert L.w2v_get_embeddings(ctx, 0, None, 10**9, 1) == B.W2V_EINVAL
    B.w2v_train_epoch(ctx, tok, off, 1, 0, 0)
    B.w2v_destroy(ctx)
    del keep


def test_embeddings_to_device_loss_reset_and_counters():
    from paper_2312_07743_amd.trainer import Trainer
    c = synth.zipf_corpus(120, 1.0, 5, 200, seed=3)
    tok = c.tokens.copy()
    tok[3] = -7
    tr = Trainer(vocab=c.vocab, dim=100, window=4, negatives=3, counts=c.counts, tokens_per_epoch=c.n_tokens, seed=8,
                 table_size=1 << 12, total_epochs=2)
    tr.set_corpus(tok, c.sent_off)
    tr.train_epoch(0)
    kept, invalid = tr.counters()
    assert invalid == 1 and kept == c.n_tokens - 1
    loss, pairs = tr.loss(reset=True)
    assert pairs > 0 and loss > 0
    assert tr.loss() == (0.0, 0) and tr.counters() == (0, 0)
    host = tr.embeddings(0)
    dev = torch.empty((c.vocab, 100), dtype=torch.float32, device="cuda")
    B.w2v_get_embeddings(tr.ctx, 0, dev, dev.numel(), True)
    assert np.array_equal(dev.cpu().numpy(), host)
    assert np.array_equal(tr.syn0[:, :100].cpu().numpy(), host)
    tr.train_epoch(1)
    assert tr.loss()[1] > 0
    tr.close()


def test_two_contexts_on_their_own_streams_do_not_disturb_each_other():
    """Two trainers with different shapes, each on a stream of its own, epochs issued alternately: each must end
    exactly where it ends when it runs alone (strict order makes a run deterministic)."""
    from paper_2312_07743_amd.trainer import Trainer
    ca = synth.zipf_corpus(300, 1.0, 6, 400, seed=1)
    cb = synth.zipf_corpus(500, 1.1, 5, 300, seed=2)

    def make(c, dim, window, negatives, stream):
        with torch.cuda.stream(stream):
            tr = Trainer(vocab=c.vocab, dim=dim, window=window, negatives=negatives, counts=c.counts,
                         tokens_per_epoch=c.n_tokens, seed=9, table_size=1 << 14, subsample_t=1e-2, total_epochs=2,
                         sentences_in_flight=1)
            tr.set_corpus(c.tokens, c.sent_off)
        return tr

    def run_alone(c, dim, window, negatives):
        tr = make(c, dim, window, negatives, torch.cuda.current_stream())
        for e in range(2):
            tr.train_epoch(e)
        out = tr.embeddings(0), tr.embeddings(1), tr.loss()
        tr.close()
        return out

    want_a, want_b = run_alone(ca, 128, 5, 5), run_alone(cb, 300, 3, 8)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ta, tb = make(ca, 128, 5, 5, sa), make(cb, 300, 3, 8, sb)
    for e in range(2):
        ta.train_epoch(e)
        tb.train_epoch(e)
    got_a = ta.embeddings(0), ta.embeddings(1), ta.loss()
    got_b = tb.embeddings(0), tb.embeddings(1), tb.loss()
    ta.close()
    tb.close()
    for got, want in ((got_a, want_a), (got_b, want_b)):
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]) and got[2] == want[2]
    torch.cuda.synchronize()


def test_tables_in_uncached_memory_train_the_same(orc32):
    """Trainer(coherent_tables=True) keeps syn0 / syn1neg in uncached device memory (for lock-free runs whose
    wavefronts must see each other's rows across XCDs): in strict order the result is the oracle's, and equal bit
    for bit to training on ordinary device memory."""
    from paper_2312_07743_amd.trainer import Trainer
    from util import assert_rows_close, run_oracle
    c = synth.zipf_corpus(500, 1.0, 6, 400, seed=21)
    kw = dict(dim=100, window=5, negatives=5, seed=13, table_size=1 << 14, subsample_t=1e-2)
    got = []
    for coherent in (False, True):
        tr = Trainer(vocab=c.vocab, counts=c.counts, tokens_per_epoch=c.n_tokens, sentences_in_flight=1,
                     coherent_tables=coherent, **kw)
        tr.set_corpus(c.tokens, c.sent_off)
        tr.train_epoch(0)
        got.append((tr.embeddings(0), tr.embeddings(1), tr.loss()))
        assert bool(torch.isfinite(tr.syn0).all()) and float(tr.syn0[:, kw["dim"]:].abs().max()) == 0.0
        tr.close()
    assert np.array_equal(got[0][0], got[1][0]) and np.array_equal(got[0][1], got[1][1]) and got[0][2] == got[1][2]
    r0, r1, rl, rp = run_oracle(orc32, c, **kw)
    assert got[1][2][1] == rp
    assert_rows_close(got[1][0], r0, 1e-4, "syn0")
    assert_rows_close(got[1][1], r1, 1e-4, "syn1neg")


def test_automatic_choice_of_the_update_mode():
    """cfg.update_mode = 0: text (a few thousand frequent rows carry most tokens) is trained with overwriting
    updates, walks over a graph with far more nodes than an L2 holds rows with summed ones; strict order and
    update_mode = 1 always overwrite, update_mode = 2 sums on text too."""
    from paper_2312_07743_amd.trainer import Trainer
    text = synth.zipf_corpus(71000, 1.05, 50, 1000, seed=2)
    walks = synth.barabasi_albert_walks(n_nodes=200000, m=5, walks_per_node=1, walk_len=20, seed=2)
    for c, mode, in_flight, want in ((text, 0, 0, 0), (walks, 0, 0, 1), (walks, 0, 1, 0), (walks, 1, 0, 0),
                                     (text, 2, 0, 1), (walks, 0, 100, 1)):
        tr = Trainer(vocab=c.vocab, dim=128, window=5, negatives=5, counts=c.counts, tokens_per_epoch=c.n_tokens, seed=1,
                     table_size=1 << 16, update_mode=mode, sentences_in_flight=in_flight)
        tr.set_corpus(c.tokens, c.sent_off)
        tr.train_epoch(0)
        plan = B.w2v_debug_get_plan(tr.ctx)
        assert plan["update"] == want, (mode, in_flight, plan)
        assert plan["wavefronts"] == (in_flight if in_flight else plan["wavefronts"]) and plan["wavefronts"] >= 1
        assert bool(torch.isfinite(tr.syn0).all())
        tr.close()
