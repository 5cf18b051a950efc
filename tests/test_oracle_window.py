"""Pins of the oracle's one-window update: hand-computed cases, the closed form at
syn1neg = 0, central finite differences of the SGNS window loss, order independence,
and a brute-force expectation over all 8 words of a toy vocabulary."""
import itertools
import math

import numpy as np
import pytest

LN2 = math.log(2.0)


def _loss(syn0, syn1, ctx, out):
    """SGNS window log-loss written from its definition (float64):
    sum over context words c of  -log sigma(<I_c,O_target>) - sum_k [k not masked] log sigma(-<I_c,O_neg_k>)."""
    tot = 0.0
    for c in ctx:
        for k, o in enumerate(out):
            if k >= 1 and o == out[0]:
                continue
            x = float(np.dot(syn0[c].astype(np.float64), syn1[o].astype(np.float64)))
            tot += -math.log(1.0 / (1.0 + math.exp(-x))) if k == 0 else -math.log(1.0 / (1.0 + math.exp(x)))
    return tot


def test_hand_case_one_pair_x_zero(orc64):
    # d=2, I=(1,0), O_target=(0,1): x=0, sigma=1/2, g=alpha/2
    syn0 = np.array([[1.0, 0.0], [9.0, 9.0]])
    syn1 = np.array([[5.0, 5.0], [0.0, 1.0]])
    loss = orc64.window_step(syn0, syn1, ctx=[0], out=[1], alpha=0.5)
    assert np.allclose(syn0, [[1.0, 0.25], [9.0, 9.0]], rtol=0, atol=1e-15)
    assert np.allclose(syn1, [[5.0, 5.0], [0.25, 1.0]], rtol=0, atol=1e-15)
    assert loss == pytest.approx(LN2, abs=1e-15)


def test_hand_case_sigma_three_quarters(orc64):
    # x = ln 3 for both pairings: sigma = 3/4.  target: g = +alpha/4 ; negative: g = -3 alpha/4
    l3 = math.log(3.0)
    syn0 = np.array([[l3, 0.0]])
    syn1 = np.array([[1.0, 0.0], [1.0, 2.0]])
    a = 0.1
    loss = orc64.window_step(syn0, syn1, ctx=[0], out=[0, 1], alpha=a)
    # dI = a/4*(1,0) - 3a/4*(1,2) ; dO_0 = a/4*(l3,0) ; dO_1 = -3a/4*(l3,0)
    assert np.allclose(syn0, [[l3 + a / 4 - 3 * a / 4, -1.5 * a]], atol=1e-14)
    assert np.allclose(syn1, [[1 + a / 4 * l3, 0.0], [1 - 0.75 * a * l3, 2.0]], atol=1e-14)
    assert loss == pytest.approx(math.log(4 / 3) + math.log(4.0), abs=1e-13)


def test_closed_form_when_output_matrix_is_zero(orc64):
    rng = np.random.default_rng(0)
    V, d, a = 12, 6, 0.025
    syn0 = rng.normal(size=(V, d))
    syn1 = np.zeros((V, d))
    s0 = syn0.copy()
    ctx, out = [3, 4, 7, 3], [5, 1, 9, 1, 5, 2]      # duplicate context 3, duplicate negative 1, negative == target (masked)
    loss = orc64.window_step(syn0, syn1, ctx, out, a)
    S = s0[ctx].sum(axis=0)                          # duplicates counted twice
    want = np.zeros((V, d))
    want[5] = 0.5 * a * S
    want[1] = -0.5 * a * S * 2                       # drawn twice -> two deltas
    want[9] = -0.5 * a * S
    want[2] = -0.5 * a * S
    assert np.array_equal(syn0, s0)                  # every O is zero -> no input update at all
    assert np.allclose(syn1, want, rtol=0, atol=1e-16)
    assert loss == pytest.approx(len(ctx) * 5 * LN2, abs=1e-12)   # target + 4 unmasked negatives


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_update_is_minus_alpha_times_gradient_by_central_differences(orc64, seed):
    rng = np.random.default_rng(seed)
    V, d, a = 9, 5, 0.05
    syn0 = rng.normal(scale=0.7, size=(V, d))
    syn1 = rng.normal(scale=0.7, size=(V, d))
    ctx = [2, 6, 2, 8, 0]                            # word 2 twice
    out = [4, 1, 7, 1, 4, 3]                         # negative 1 twice; negative == target once
    a0, a1 = syn0.copy(), syn1.copy()
    lw = orc64.window_step(a0, a1, ctx, out, a)
    assert lw == pytest.approx(_loss(syn0, syn1, ctx, out), rel=1e-12)
    h = 1e-5
    for M, upd, which in ((syn0, a0, 0), (syn1, a1, 1)):
        grad = np.zeros_like(M)
        for i in range(V):
            for j in range(d):
                keep = M[i, j]
                M[i, j] = keep + h
                lp = _loss(syn0, syn1, ctx, out)
                M[i, j] = keep - h
                lm = _loss(syn0, syn1, ctx, out)
                M[i, j] = keep
                grad[i, j] = (lp - lm) / (2 * h)
        delta = upd - M
        assert np.allclose(delta, -a * grad, rtol=1e-6, atol=1e-9), which
    # rows outside the window are untouched, bit for bit
    for i in set(range(V)) - set(ctx):
        assert np.array_equal(a0[i], syn0[i])
    for i in set(range(V)) - set(out):
        assert np.array_equal(a1[i], syn1[i])


def test_pairing_order_is_free_and_negatives_commute(orc64, orc32):
    rng = np.random.default_rng(5)
    V, d = 10, 16
    syn0 = rng.normal(scale=0.5, size=(V, d))
    syn1 = rng.normal(scale=0.5, size=(V, d))
    ctx, out = [1, 2, 3, 4], [5, 6, 7, 8]
    ref0, ref1 = syn0.copy(), syn1.copy()
    orc64.window_step(ref0, ref1, ctx, out, 0.03)
    for pc in itertools.permutations(ctx):
        for negs in ([6, 7, 8], [8, 6, 7], [7, 8, 6]):
            b0, b1 = syn0.copy(), syn1.copy()
            orc64.window_step(b0, b1, list(pc), [5] + negs, 0.03)
            assert np.allclose(b0, ref0, rtol=0, atol=1e-14) and np.allclose(b1, ref1, rtol=0, atol=1e-14)
    # the float build agrees with the double build to float rounding
    f0, f1 = syn0.astype(np.float32), syn1.astype(np.float32)
    r0, r1 = f0.astype(np.float64), f1.astype(np.float64)
    orc32.window_step(f0, f1, ctx, out, 0.03)
    orc64.window_step(r0, r1, ctx, out, 0.03)
    assert np.allclose(f0, r0, rtol=0, atol=2e-7) and np.allclose(f1, r1, rtol=0, atol=2e-7)


def test_immediate_reading_differs_from_window_minibatch(orc64):
    rng = np.random.default_rng(6)
    syn0 = rng.normal(size=(6, 4))
    syn1 = rng.normal(size=(6, 4))
    a0, a1, b0, b1 = syn0.copy(), syn1.copy(), syn0.copy(), syn1.copy()
    orc64.window_step(a0, a1, [0, 1], [2, 3], 0.1)
    orc64.window_step(b0, b1, [0, 1], [2, 3], 0.1, immediate=True)
    assert not np.allclose(a0, b0, atol=1e-6)
    # with a single pairing the two readings are the same step
    a0, a1, b0, b1 = syn0.copy(), syn1.copy(), syn0.copy(), syn1.copy()
    orc64.window_step(a0, a1, [0], [2], 0.1)
    orc64.window_step(b0, b1, [0], [2], 0.1, immediate=True)
    assert np.allclose(a0, b0, atol=1e-15) and np.allclose(a1, b1, atol=1e-15)


def test_expected_sampled_gradient_equals_brute_force_over_all_words(orc64):
    """Average the input-row update over many sampled negative sets and compare with the
    expectation enumerated over the whole 8-word vocabulary: E[delta I] =
    alpha * [ (1 - sigma(x_t)) O_t  -  N * sum_{w != t} P_n(w) sigma(x_w) O_w ]."""
    rng = np.random.default_rng(7)
    V, d, N, a = 8, 4, 5, 0.1
    counts = np.array([400, 250, 120, 80, 60, 40, 30, 20], np.uint64)
    tsz = 1 << 16
    end = orc64.table_ends(counts, tsz)
    p_n = counts.astype(np.float64) ** 0.75
    p_n /= p_n.sum()
    syn0 = rng.normal(scale=0.8, size=(V, d))
    syn1 = rng.normal(scale=0.8, size=(V, d))
    c, t = 3, 1
    sig = 1.0 / (1.0 + np.exp(-(syn1 @ syn0[c])))
    want = (1 - sig[t]) * syn1[t]
    for w in range(V):
        if w != t:
            want = want - N * p_n[w] * sig[w] * syn1[w]
    want *= a
    n = 30_000
    acc = np.zeros(d)
    for p in range(n):
        negs = [orc64.negative(end, tsz, 2024, 0, p, k) for k in range(N)]
        b0, b1 = syn0.copy(), syn1.copy()
        orc64.window_step(b0, b1, [c], [t] + negs, a)
        acc += b0[c] - syn0[c]
    got = acc / n
    assert np.allclose(got, want, rtol=0, atol=4e-3 * a * 10), (got, want)
