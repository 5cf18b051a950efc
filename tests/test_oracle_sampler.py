"""Pins of the oracle's negative-sampling table, subsampling thresholds and learning rate:
closed forms, special cases and brute force."""
import math

import numpy as np
import pytest


def _zipf_counts(V, s, total):
    w = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    return np.maximum(1, np.round(w / w.sum() * total)).astype(np.uint64)


def test_table_shares_follow_count_to_the_three_quarters(orc32):
    counts = _zipf_counts(5000, 1.05, 2_000_000)
    tsz = 1 << 24
    end = orc32.table_ends(counts, tsz)
    assert end[-1] == tsz and np.all(np.diff(end.astype(np.int64)) >= 0)
    slots = np.diff(np.concatenate([[0], end.astype(np.int64)]))
    share = counts.astype(np.float64) ** 0.75
    share /= share.sum()
    assert slots.sum() == tsz
    assert np.max(np.abs(slots / tsz - share)) <= 1.0 / tsz + 1e-12


def test_equal_counts_give_a_uniform_table(orc32):
    V, tsz = 1000, 1 << 20
    end = orc32.table_ends(np.full(V, 7, np.uint64), tsz)
    want = np.floor((np.arange(1, V + 1) * tsz) / V)
    assert np.max(np.abs(end.astype(np.float64) - want)) <= 1
    # a perfect-power case that is exact in binary: V = 2^k words, tsz = 2^m
    end = orc32.table_ends(np.full(256, 16, np.uint64), 1 << 16)
    assert np.array_equal(end, (np.arange(1, 257) * 256).astype(np.uint64))


def test_zero_count_words_own_no_slot_and_lookup_matches_materialised_table(orc32):
    counts = np.array([50, 0, 7, 0, 0, 1, 900, 3], np.uint64)
    tsz = 4096
    end = orc32.table_ends(counts, tsz)
    slots = np.diff(np.concatenate([[0], end.astype(np.int64)]))
    assert slots[1] == 0 and slots[3] == 0 and slots[4] == 0
    table = np.repeat(np.arange(len(counts)), slots)           # brute-force materialisation
    assert len(table) == tsz
    got = np.array([orc32.word_of_slot(end, s) for s in range(tsz)])
    assert np.array_equal(got, table)


def test_all_zero_counts_rejected(orc32):
    with pytest.raises(ValueError):
        orc32.table_ends(np.zeros(4, np.uint64), 64)


def test_sampled_negatives_follow_the_distribution(orc32):
    counts = np.array([1000, 500, 250, 125, 60, 30, 15, 8], np.uint64)
    tsz = 1 << 16
    end = orc32.table_ends(counts, tsz)
    n = 120_000
    ids = np.array([orc32.negative(end, tsz, 1234, 0, p, p % 5) for p in range(n)])
    p_n = counts.astype(np.float64) ** 0.75
    p_n /= p_n.sum()
    cnt = np.bincount(ids, minlength=8)
    chi2 = ((cnt - n * p_n) ** 2 / (n * p_n)).sum()
    assert chi2 < 35.0, cnt                                     # dof 7: P(>35) ~ 1e-5


def test_negative_uses_draw_2_plus_k_and_multiply_high(orc32):
    counts = np.array([3, 1, 4, 1, 5, 9, 2, 6], np.uint64)
    tsz = 1000                                                  # not a power of two on purpose
    end = orc32.table_ends(counts, tsz)
    for p in (0, 17, 10**12):
        for k in range(4):
            u = orc32.draw(77, 3, p, 2 + k) >> 32
            slot = (u * tsz) >> 32
            assert orc32.negative(end, tsz, 77, 3, p, k) == orc32.word_of_slot(end, slot)


def test_thresholds_closed_form_cases(orc32):
    # total = 1e6; t = 1e-4  ->  f = 4t = 4e-4 (count 400) keeps with probability exactly 1/2
    counts = np.array([400, 100, 50, 1600, 0, 997850], np.uint64)
    assert counts.sum() == 1_000_000
    thr = orc32.thresholds(counts, 1e-4)
    assert abs(int(thr[0]) - (1 << 31)) <= 4                    # sqrt(1/4) up to the rounding of t/f
    assert thr[1] == 0xFFFFFFFF and thr[2] == 0xFFFFFFFF        # f <= t: always kept
    assert abs(int(thr[3]) - (1 << 30)) <= 4                    # f = 16 t -> 1/4
    assert thr[4] == 0xFFFFFFFF                                 # unseen word
    want = math.sqrt(1e-4 / (997850 / 1e6)) * 2**32
    assert abs(int(thr[5]) - want) <= 2
    assert np.all(orc32.thresholds(counts, 0.0) == 0xFFFFFFFF)  # t = 0 switches subsampling off


def test_keep_rate_matches_threshold(orc32):
    counts = np.array([400, 100, 1600, 997900], np.uint64)
    thr = orc32.thresholds(counts, 1e-4)
    n = 40_000
    for w, p in ((0, 0.5), (1, 1.0), (2, 0.25)):
        kept = sum(orc32.keep(thr, w, 5, 1, pos) for pos in range(n))
        assert abs(kept / n - p) < 4 * math.sqrt(max(p * (1 - p), 1e-9) / n) + 1e-12


def test_kept_fraction_of_the_mid_zipf_law(orc32):
    # 71,000 ranks, exponent 1.05, t = 1e-4: the expected kept fraction follows from the law itself
    V, s, t = 71000, 1.05, 1e-4
    f = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    f /= f.sum()
    want = float(np.sum(f * np.minimum(1.0, np.sqrt(t / f))))
    counts = np.maximum(1, np.round(f * 17_000_000)).astype(np.uint64)
    thr = orc32.thresholds(counts, t).astype(np.float64)
    pk = np.where(thr == 0xFFFFFFFF, 1.0, thr / 2.0**32)
    got = float(np.sum(counts / counts.sum() * pk))
    assert abs(got - want) < 2e-3
    assert 0.40 < got < 0.55


def test_learning_rate_schedule(orc32):
    T, E = 1000, 4
    assert orc32.lr(0.025, 1e-4, 0, E, T, 0) == np.float32(0.025)
    assert orc32.lr(0.025, 1e-4, 2, E, T, 0) == np.float32(0.0125)          # half way
    assert orc32.lr(0.025, 1e-4, 3, E, T, 1000) == np.float32(0.025 * 1e-4)  # floor at the very end
    assert orc32.lr(0.025, 1e-4, 1, E, T, 500) == np.float32(0.025 * (1 - 1500 / 4000))
    lrs = [orc32.lr(0.025, 1e-4, e, E, T, s) for e in range(E) for s in range(0, T, 100)]
    assert all(a > b for a, b in zip(lrs, lrs[1:]))


def test_initial_weights(orc32):
    V, d = 300, 128
    syn0, syn1 = orc32.init_weights(9, V, d)
    assert np.all(syn1 == 0)
    assert syn0.min() >= -0.5 / d and syn0.max() < 0.5 / d
    u = syn0.astype(np.float64) * d + 0.5                       # back to U[0,1)
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    assert abs(np.corrcoef(u[:, 0], u[:, 1])[0, 1]) < 0.2
    other, _ = orc32.init_weights(10, V, d)
    assert not np.array_equal(other, syn0)
    # each value is a multiple of 2^-24 / d, rounded once to float
    k = np.round((syn0.astype(np.float64) * d + 0.5) * 2**24)
    assert np.array_equal(((k / 2**24 - 0.5) / d).astype(np.float32), syn0)
