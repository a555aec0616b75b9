"""Pins for the oracle's random-number path (CPU only)."""
import os
import numpy as np
from scipy import stats
from oracle import philox

HERE = os.path.dirname(__file__)


def test_known_answer_vectors():
    n = 0
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = philox.philox4x32_10(w[0], w[1], w[2], w[3], w[4], w[5])
        assert [int(o) for o in out] == w[6:10]
        n += 1
    assert n == 3


def test_word_layout_and_determinism():
    V = 11
    w = philox.random_words(seed=(7 << 32) | 5, stream=1, b=3, t=9, V=V)
    for v in range(V):
        blk = philox.philox4x32_10(v >> 2, 9, 3, 1, 5, 7)
        assert int(blk[v & 3]) == int(w[v])
    assert np.array_equal(w, philox.random_words((7 << 32) | 5, 1, 3, 9, V))
    # a different row, position, stream or seed gives a different block
    for other in [philox.random_words((7 << 32) | 5, 1, 4, 9, V), philox.random_words((7 << 32) | 5, 1, 3, 10, V),
                  philox.random_words((7 << 32) | 5, 0, 3, 9, V), philox.random_words((7 << 32) | 6, 1, 3, 9, V),
                  philox.random_words((8 << 32) | 5, 1, 3, 9, V)]:
        assert not np.array_equal(w, other)


def test_uniform_is_open_interval_and_exact_in_float32():
    words = np.array([0, 1, 0x1FF, 0x200, 0xFFFFFFFF, 0xFFFFFE00, 0x80000000], dtype=np.uint32)
    u = philox.uniforms(words)
    assert u.min() > 0.0 and u.max() < 1.0
    assert u[0] == 2.0 ** -24 and u[4] == 1.0 - 2.0 ** -24
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)   # exact in fp32
    assert np.all(np.isfinite(-np.log(-np.log(u))))
    # uniformity of the generated stream (KS test)
    big = philox.uniforms(philox.random_words(123, 0, 0, 0, 200000))
    assert stats.kstest(big, "uniform").pvalue > 1e-3


def test_gumbel_max_draws_from_softmax():
    rng = np.random.default_rng(5)
    logits = rng.normal(size=8) * 1.5
    for T in (1.0, 0.7):
        p = np.exp(logits / T - (logits / T).max())
        p /= p.sum()
        n = 40000
        cnt = np.zeros(8)
        for i in range(n):
            x, _ = philox.sample(logits, T, seed=99, stream=philox.STREAM_DRAFT, b=i % 97, t=i // 97)
            cnt[x] += 1
        chi2 = ((cnt - n * p) ** 2 / (n * p)).sum()
        assert chi2 < stats.chi2.ppf(0.9999, df=7), (chi2, cnt / n, p)


def test_greedy_and_tie_break():
    logits = np.array([0.1, 2.0, -1.0, 2.0, 0.5])
    x, _ = philox.sample(logits, 0.0, 1, 0, 0, 0)
    assert x == 1                               # lowest index among equal maxima
    x2, y = philox.sample(logits, 1.0, 1, 0, 0, 0)
    assert x2 == int(np.argmax(y)) and y.dtype == np.float32


def test_streams_are_uncorrelated():
    a = philox.gumbel(3, philox.STREAM_DRAFT, 2, 17, 50000)
    b = philox.gumbel(3, philox.STREAM_TARGET, 2, 17, 50000)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.02
    # Gumbel(0,1): mean = Euler gamma, variance = pi^2/6
    assert abs(a.mean() - 0.5772156649) < 0.02 and abs(a.var() - np.pi ** 2 / 6) < 0.05
