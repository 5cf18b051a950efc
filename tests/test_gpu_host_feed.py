"""GPU tests of host-fed training (w2v_train_epoch_host): batches copied into a device staging buffer while
the previous batch trains must give what training on a resident copy of the corpus gives."""
import numpy as np
import pytest
import torch

from paper_2312_07743_amd import binding as B
from paper_2312_07743_amd import synth
from paper_2312_07743_amd.trainer import Trainer
from util import assert_rows_close, run_oracle

pytestmark = pytest.mark.gpu


def _trainer(c, **kw):
    args = dict(vocab=c.vocab, dim=128, window=5, negatives=5, counts=c.counts, tokens_per_epoch=c.n_tokens, seed=11,
                table_size=1 << 16, subsample_t=1e-3, total_epochs=2)
    args.update(kw)
    return Trainer(**args)


@pytest.mark.parametrize("pinned", [False, True])
def test_strict_order_equals_resident_training_bit_for_bit(orc32, pinned):
    # ragged sentences (some empty), staging so small that a batch holds two or three sentences
    rng = np.random.default_rng(1)
    lens = [0, 700, 1, 350, 0, 0, 1000, 12, 999, 640, 3, 800, 0]
    tok = rng.integers(0, 400, size=sum(lens)).astype(np.int32)
    off = np.cumsum([0] + lens).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok, minlength=400).astype(np.uint64))
    res = _trainer(c, sentences_in_flight=1)
    res.set_corpus(c.tokens, c.sent_off)
    host = _trainer(c, sentences_in_flight=1)
    if pinned:
        t_host = torch.as_tensor(c.tokens).pin_memory()
        o_host = torch.as_tensor(c.sent_off.view(np.int64)).pin_memory()
    else:
        t_host, o_host = c.tokens, c.sent_off
    for e in range(2):
        res.train_epoch(e)
        B.w2v_train_epoch_host(host.ctx, t_host, o_host, len(lens), 0, e, host_staging(host, 2 * 8192), 2 * 8192)
    torch.cuda.synchronize()
    (l0, p0), (l1, p1) = res.loss(), host.loss()
    assert p0 == p1 and abs(l0 - l1) <= 1e-9 * abs(l0)      # per-launch partial sums are added in another order
    assert res.counters() == host.counters()
    for which in (0, 1):
        assert np.array_equal(res.embeddings(which), host.embeddings(which))
    # and the resident run is the oracle's (one epoch of the same corpus)
    r0, r1, rl, rp = run_oracle(orc32, c, dim=128, window=5, negatives=5, seed=11, table_size=1 << 16,
                                subsample_t=1e-3, epochs=2)
    assert rp == host.loss()[1]
    assert_rows_close(host.embeddings(0), r0, 1e-4, "syn0")
    res.close()
    host.close()


@pytest.mark.parametrize("variant", ["bf16", "summed"])
def test_strict_order_equals_resident_training_for_the_other_kernels(variant):
    """The host-fed path launches whatever kernel the context uses: tables stored as bfloat16, and summed updates
    (forced on in strict order through the test surface): bit-equal to training on a resident copy."""
    rng = np.random.default_rng(2)
    lens = [300, 0, 900, 1, 640, 77, 1000, 2, 512]
    tok = rng.integers(0, 300, size=sum(lens)).astype(np.int32)
    off = np.cumsum([0] + lens).astype(np.uint64)
    c = synth.Corpus(tok, off, np.bincount(tok, minlength=300).astype(np.uint64))
    kw = dict(sentences_in_flight=1, storage=1) if variant == "bf16" else dict(sentences_in_flight=1, update_mode=2)
    res, host = _trainer(c, **kw), _trainer(c, **kw)
    if variant == "summed":
        B.w2v_debug_set_update(res.ctx, 1)
        B.w2v_debug_set_update(host.ctx, 1)
    res.set_corpus(c.tokens, c.sent_off)
    for e in range(2):
        res.train_epoch(e)
        B.w2v_train_epoch_host(host.ctx, c.tokens, c.sent_off, len(lens), 0, e, host_staging(host, 2 * 8192), 2 * 8192)
    torch.cuda.synchronize()
    if variant == "summed":
        assert B.w2v_debug_get_plan(host.ctx)["update"] == 1
    (l0, p0), (l1, p1) = res.loss(), host.loss()
    assert p0 == p1 and abs(l0 - l1) <= 1e-9 * abs(l0) and res.counters() == host.counters()
    for which in (0, 1):
        assert np.array_equal(res.embeddings(which), host.embeddings(which))
    res.close()
    host.close()


def host_staging(tr, nbytes):
    if getattr(tr, "staging", None) is None or tr.staging.numel() != nbytes:
        tr.staging = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    return tr.staging


def test_lock_free_host_feed_counts_and_loss_match_resident_run():
    # 64 wavefronts either way.  Lock-free results depend on the schedule (which rows are stale when), and the two
    # runs cut the work differently, so the first-epoch mean losses only have to agree within 3 %; the counts
    # are schedule-independent and must be equal.
    c = synth.planted_corpus(vocab=20000, n_sent=3000, sent_len=1000, seed=3, band_start=500)
    res = _trainer(c, subsample_t=1e-4, total_epochs=1, sentences_in_flight=64)
    res.set_corpus(c.tokens, c.sent_off)
    res.train_epoch(0)
    host = _trainer(c, subsample_t=1e-4, total_epochs=1, sentences_in_flight=64)
    host.train_epoch_from_host(c.tokens, c.sent_off, epoch=0, staging_bytes=1 << 20)    # about 23 batches
    torch.cuda.synchronize()
    (l0, p0), (l1, p1) = res.loss(), host.loss()
    assert p0 == p1 and res.counters() == host.counters()
    assert abs(l0 / p0 - l1 / p1) < 0.03 * l0 / p0, (l0 / p0, l1 / p1)
    res.close()
    host.close()


def test_argument_errors():
    c = synth.zipf_corpus(100, 1.0, 3, 500, seed=1)
    tr = _trainer(c)
    L = B.lib()
    stg = torch.empty(4096, dtype=torch.uint8, device="cuda")
    args = (c.tokens.ctypes.data, c.sent_off.ctypes.data, 3, 0, 0)
    assert L.w2v_train_epoch_host(tr.ctx, *args, None, 4096) == B.W2V_EINVAL
    assert L.w2v_train_epoch_host(tr.ctx, *args, stg.data_ptr() + 8, 4096) == B.W2V_EINVAL
    assert L.w2v_train_epoch_host(tr.ctx, *args, stg.data_ptr(), 2048) == B.W2V_EINVAL       # 500 tokens need 2016 B per half
    assert "does not fit" in B.w2v_last_error(tr.ctx)
    assert L.w2v_train_epoch_host(tr.ctx, None, c.sent_off.ctypes.data, 3, 0, 0, stg.data_ptr(), 4096) == B.W2V_EINVAL
    bad = c.sent_off.copy()
    bad[1], bad[2] = bad[2], bad[1]
    assert L.w2v_train_epoch_host(tr.ctx, c.tokens.ctypes.data, bad.ctypes.data, 3, 0, 0, stg.data_ptr(), 4096) == B.W2V_EINVAL
    assert L.w2v_train_epoch_host(tr.ctx, c.tokens.ctypes.data, c.sent_off.ctypes.data, 0, 0, 0, stg.data_ptr(), 4096) == B.W2V_OK
    assert L.w2v_train_epoch_host(tr.ctx, *args[:4], 7, stg.data_ptr(), 4096) == B.W2V_EINVAL   # epoch >= total_epochs
    torch.cuda.synchronize()
    assert tr.loss()[1] == 0
    tr.close()
