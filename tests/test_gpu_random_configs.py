"""Strict-order parity on randomly drawn valid configurations: row lengths on and off the lane layouts, windows
and negative counts over their whole ranges, ragged and empty sentences, invalid ids, every way of cutting
sentences into work units, shared negatives, late positions in long schedules.  The draws are seeded, so the
cases are the same on every run."""
import numpy as np
import pytest

from paper_2312_07743_amd import synth
from util import run_gpu, run_oracle, assert_rows_close

pytestmark = pytest.mark.gpu

DIMS = [2, 3, 5, 17, 31, 32, 33, 63, 64, 65, 96, 100, 127, 128, 129, 130, 192, 200, 255, 256, 257, 260, 288, 300, 316,
        320, 321, 384, 400, 448, 450, 500, 511, 512]


def _draw_case(rng):
    dim = int(rng.choice(DIMS))
    lane_floats = 64 if dim <= 64 else 128 if dim <= 128 else 256 if dim <= 256 else 320 if dim <= 320 else 512
    mode = int(rng.choice([0, 0, 1]))
    window = int(rng.integers(1, (16 if mode else min(16, 5120 // lane_floats)) + 1))
    negatives = int(rng.choice([0, 1, 2, 3, 4, 5, 5, 5, 6, 7, 8, 10, 11, 12, 13, 15, 20]))
    V = int(rng.choice([10, 50, 300, 2000]))
    lens = rng.choice([0, 1, 2, 3, 7, 30, 64, 65, 100, 129, 300, 700], size=int(rng.integers(1, 12)))
    T = int(lens.sum())
    if rng.random() < 0.7:
        p = 1.0 / np.arange(1, V + 1)
        tok = rng.choice(V, size=T, p=p / p.sum()).astype(np.int32)
    else:
        tok = rng.integers(0, V, size=T).astype(np.int32)
    bad = rng.random(T) < (0.02 if rng.random() < 0.4 else 0.0)
    tok[bad] = rng.choice([-1, V, V + 5, 2**31 - 1, -2**31], size=int(bad.sum()))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    counts = np.bincount(tok[(tok >= 0) & (tok < V)], minlength=V).astype(np.uint64)
    if rng.random() < 0.3:
        counts = counts + rng.integers(0, 3, size=V).astype(np.uint64)      # counts need not be the corpus's own
    if counts.sum() == 0:
        counts[0] = 1
    unit_shift = rng.choice([-1, -1, 0, 1, 2, 3, 5])
    first = int(rng.choice([0, 0, 12345, 2**33 + 7]))
    total = int(rng.choice([1, 3]))
    kw = dict(dim=dim, window=window, negatives=negatives, seed=int(rng.integers(1 << 40)),
              table_size=max(V, int(rng.choice([17, 4099, 50021, 1 << 16]))),
              subsample_t=float(rng.choice([0.0, 0.0, 1e-1, 1e-2, 1e-3])), window_mode=mode,
              negative_block=int(rng.choice([0, 0, 0, 2, 4, 8, 16, 64])), first_token_global_pos=first,
              tokens_per_epoch=first + T + 1000, total_epochs=total, start_epoch=int(rng.integers(0, total)),
              epochs=1, lr0=0.01)
    return synth.Corpus(tok, off, counts), (None if unit_shift < 0 else int(unit_shift)), kw


@pytest.mark.parametrize("block", range(6))
def test_randomly_drawn_configurations_match_the_oracle(orc32, block):
    master = np.random.default_rng(1000 + block)
    for case in range(20):
        corpus, unit_shift, kw = _draw_case(np.random.default_rng(master.integers(1 << 62)))
        what = f"block {block} case {case}: V={corpus.vocab} sentences={np.diff(corpus.sent_off.astype(np.int64)).tolist()} " \
               f"unit_shift={unit_shift} {kw}"
        print(what, flush=True)
        g0, g1, gl, gp = run_gpu(corpus, sentences_in_flight=1, unit_shift=unit_shift, **kw)
        r0, r1, rl, rp = run_oracle(orc32, corpus, **kw)
        assert gp == rp, what
        assert abs(gl - rl) <= 2e-5 * abs(rl) + 1e-9, what
        assert_rows_close(g0, r0, 1e-4, "syn0, " + what)
        assert_rows_close(g1, r1, 1e-4, "syn1neg, " + what)
