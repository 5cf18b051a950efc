"""Pins of the oracle's counter-based random numbers and the integer draws built on them."""
import os

import numpy as np

G = 0x9E3779B97F4A7C15
M64 = (1 << 64) - 1
HERE = os.path.dirname(os.path.abspath(__file__))


def test_mixer_reproduces_published_splitmix64_stream(orc32):
    want = [int(l, 16) for l in open(os.path.join(HERE, "golden", "splitmix64_seed0.txt"))
            if l.strip() and not l.startswith("#")]
    got = [orc32.mix64((n * G) & M64) for n in range(1, len(want) + 1)]
    assert got == want
    assert orc32.mix64(0) == 0


def _mix_py(z):
    z &= M64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & M64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & M64
    z ^= z >> 31
    return z


def test_draw_composition_in_big_integers(orc32):
    # the keying (seed, epoch) -> key, position -> base, index -> draw, redone with Python ints
    # (no 64-bit wrap-around to get wrong), including positions beyond 2^32
    for seed, e, p, j in [(0, 0, 0, 0), (1, 0, 0, 0), (42, 0, 12345, 2), (42, 3, 16718844, 6),
                          (0xDEADBEEF, 1, (1 << 40) + 7, 11), (M64, 7, M64 >> 1, 21)]:
        key = _mix_py(seed + G * (e + 1))
        base = _mix_py(key ^ _mix_py(p))
        assert orc32.draw(seed, e, p, j) == _mix_py(base + G * (j + 1))


def test_draws_differ_across_every_key_component(orc32):
    ref = orc32.draw(5, 0, 100, 0)
    assert len({ref, orc32.draw(6, 0, 100, 0), orc32.draw(5, 1, 100, 0),
                orc32.draw(5, 0, 101, 0), orc32.draw(5, 0, 100, 1)}) == 5


def test_width_is_uniform_on_1_to_W(orc32):
    n = 200_000
    for W in (1, 5, 10):
        w = np.array([orc32.width(W, 0, 11, 0, p) for p in range(n // (5 if W == 1 else 1))])
        assert w.min() == 1 and w.max() == W
        cnt = np.bincount(w, minlength=W + 1)[1:]
        exp = len(w) / W
        chi2 = ((cnt - exp) ** 2 / exp).sum()
        assert chi2 < 40.0, (W, cnt)          # dof <= 9: P(chi2 > 40) ~ 1e-5


def test_fixed_width_mode_is_ceil_half(orc32):
    assert [orc32.width(W, 1, 3, 0, 9) for W in (1, 2, 5, 6, 10)] == [1, 1, 3, 3, 5]


def test_high_word_of_draw_is_uniform(orc32):
    u = np.array([orc32.draw(99, 2, p, 0) >> 32 for p in range(100_000)], dtype=np.float64) / 2.0**32
    cnt, _ = np.histogram(u, bins=20, range=(0, 1))
    chi2 = ((cnt - 5000.0) ** 2 / 5000.0).sum()
    assert chi2 < 60.0
    # lag-1 correlation between consecutive positions is noise
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.02
