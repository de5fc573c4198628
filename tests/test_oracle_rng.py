"""Pins for the oracle's counter-based generator and Gumbel-max sampler (CPU only)."""
import numpy as np
from scipy import stats

from oracle import philox


def test_philox_known_answers():
    # Known-answer vectors distributed with the Random123 library (Salmon et al., SC'11)
    # for philox4x32 with 10 rounds; see tests/golden/philox4x32_10_kat.txt.
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    n = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(x, 16) for x in line.split()]
        ctr, key, exp = w[0:4], w[4:6], w[6:10]
        got = philox.philox4x32_10(np.array(ctr, dtype=np.uint32), key)
        assert [int(x) for x in got] == exp
        n += 1
    assert n == 3


def test_u01_open_interval_and_fp32_exact():
    bits = np.array([0, 1, 511, 512, 0xFFFFFFFF], dtype=np.uint32)
    u = philox.u01(bits)
    assert np.all(u > 0) and np.all(u < 1)
    assert np.all(u.astype(np.float32).astype(np.float64) == u)


def test_uniform_chi_square_and_stream_independence():
    u = philox.vocab_uniforms(seed=5, seq=0, step=3, row=1, purpose=0, vocab=200000)
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    assert stats.chisquare(hist).pvalue > 1e-3
    v = philox.vocab_uniforms(seed=5, seq=0, step=3, row=2, purpose=0, vocab=200000)
    assert abs(np.corrcoef(u, v)[0, 1]) < 0.01
    for other in (dict(seed=6), dict(seq=1), dict(step=4), dict(purpose=1)):
        kw = dict(seed=5, seq=0, step=3, row=1, purpose=0, vocab=64)
        kw.update(other)
        assert not np.array_equal(philox.vocab_uniforms(**kw), u[:64])


def test_gumbel_max_follows_softmax():
    from oracle.pacer_oracle import gumbel_argmax, softmax
    logits = np.array([0.3, -1.0, 2.0, 0.0, 1.1, -3.0])
    p = softmax(logits)
    n = 20000
    cnt = np.zeros(6)
    for s in range(n):
        u = philox.vocab_uniforms(seed=11, seq=0, step=s, row=0, purpose=2, vocab=6)
        cnt[gumbel_argmax(logits, u)] += 1
    assert stats.chisquare(cnt, p * n).pvalue > 1e-3
