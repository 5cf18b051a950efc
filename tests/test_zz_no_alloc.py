"""w2v_train_epoch_static, the entry point for callers that cannot allocate (its scratch memory is an array inside
the library), against w2v_train_epoch through the C ABI: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2312_07743_amd import binding as B
from paper_2312_07743_amd import synth

pytestmark = pytest.mark.gpu


def _trainer(c, T, **kw):
    from paper_2312_07743_amd.trainer import Trainer
    return Trainer(vocab=c.vocab, counts=c.counts, tokens_per_epoch=T, seed=17, table_size=1 << 16, total_epochs=2, **kw)


def _static_epoch(tr, epoch, first=0):
    out_loss = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    out_pairs = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    B.w2v_train_epoch_static(tr.ctx, tr.tokens, tr.sent_off, tr.n_sent, first, epoch, out_loss, out_pairs)
    torch.cuda.synchronize()
    return float(out_loss.item()), int(out_pairs.item())


@pytest.mark.parametrize("shape", [dict(dim=128, window=5, negatives=5), dict(dim=300, window=4, negatives=10),
                                   dict(dim=128, window=5, negatives=5, storage=1)])
def test_strict_order_equals_the_allocating_entry_point_bit_for_bit(shape):
    big = synth.zipf_corpus(600, 1.05, 9, 500, seed=3)
    small = synth.Corpus(big.tokens[:700].copy(), np.array([0, 300, 300, 700], np.uint64), big.counts)
    T = big.n_tokens
    a = _trainer(big, T, sentences_in_flight=1, subsample_t=1e-2, **shape)
    b = _trainer(big, T, sentences_in_flight=1, subsample_t=1e-2, **shape)
    for epoch, c in ((0, big), (1, small)):                      # the second call has the smaller input
        a.set_corpus(c.tokens, c.sent_off)
        b.set_corpus(c.tokens, c.sent_off)
        a.loss(reset=True)
        a.train_epoch(epoch)
        want_loss, want_pairs = a.loss()
        got_loss, got_pairs = _static_epoch(b, epoch)
        assert got_pairs == want_pairs and want_pairs > 0
        assert got_loss == want_loss                             # same kernels, same order: the same double
        assert np.array_equal(a.embeddings(0), b.embeddings(0)) and np.array_equal(a.embeddings(1), b.embeddings(1))
        assert b.loss() == (0.0, 0) and b.counters() == (0, 0)   # the context's own accumulators are not touched
    a.close()
    b.close()


def test_lock_free_calls_with_summed_updates_and_the_limit_of_the_scratch_array():
    c = synth.barabasi_albert_walks(n_nodes=20000, m=5, walks_per_node=2, walk_len=80, seed=2)
    small = synth.Corpus(c.tokens[:80 * 3000].copy(), c.sent_off[:3001].copy(), c.counts)
    kw = dict(dim=128, window=10, negatives=5, update_mode=2)
    a, b = _trainer(c, c.n_tokens, **kw), _trainer(c, c.n_tokens, **kw)
    per_wave = 22 * 128 * 4
    room = ((32 << 20) - 256) // per_wave
    for epoch, part in ((0, c), (1, small)):
        a.set_corpus(part.tokens, part.sent_off)
        b.set_corpus(part.tokens, part.sent_off)
        a.loss(reset=True)
        a.train_epoch(epoch)
        want_loss, want_pairs = a.loss()
        got_loss, got_pairs = _static_epoch(b, epoch)
        plan = B.w2v_debug_get_plan(b.ctx)
        assert plan["update"] == 1 and 1 < plan["wavefronts"] <= room
        assert got_pairs == want_pairs                           # draws do not depend on the schedule
        assert abs(got_loss - want_loss) <= 0.01 * want_loss     # lock-free runs agree statistically
        assert bool(torch.isfinite(b.syn0).all()) and bool(torch.isfinite(b.syn1neg).all())
    a.close()
    b.close()
    # more wavefronts than the array has snapshot room for: refused, nothing launched
    d = _trainer(c, c.n_tokens, sentences_in_flight=room + 1, **kw)
    d.set_corpus(small.tokens, small.sent_off)
    with pytest.raises(B.W2VError) as err:
        _static_epoch(d, 0)
    assert err.value.code == B.W2V_EINVAL and "scratch" in str(err.value)
    d.set_corpus(small.tokens, small.sent_off)
    d.close()
    e = _trainer(c, c.n_tokens, sentences_in_flight=room, **kw)
    e.set_corpus(small.tokens, small.sent_off)
    loss, pairs = _static_epoch(e, 0)
    assert pairs > 0 and np.isfinite(loss)
    e.close()
