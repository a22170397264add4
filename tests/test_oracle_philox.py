"""Pins for the oracle's counter-based dropout mask (CPU only)."""
import os

import numpy as np

from oracle import philox

HERE = os.path.dirname(os.path.abspath(__file__))


def _philox_int(ctr, key):
    """Independent big-int transcription of the Philox4x32-10 definition (SC'11, section 3.3/Table 2)."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) % 2**32, (k[1] + 0xBB67AE85) % 2**32]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 % 2**32, (p0 >> 32) ^ c[3] ^ k[1], p0 % 2**32]
    return c


def _kat():
    rows = []
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answer_vectors():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        got = philox.philox4x32_10(*[np.array([c]) for c in ctr], key[0], key[1])
        assert [int(g[0]) for g in got] == out
        assert _philox_int(ctr, key) == out


def test_vectorised_matches_bigint_on_random_counters():
    rng = np.random.default_rng(5)
    ctr = rng.integers(0, 2**32, size=(4, 64), dtype=np.uint64)
    key = [int(v) for v in rng.integers(0, 2**32, size=2, dtype=np.uint64)]
    got = philox.philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1])
    for i in range(64):
        assert [int(g[i]) for g in got] == _philox_int([int(c) for c in ctr[:, i]], key)


def _keep_scalar(e, p, seed, site, layer_id):
    blk = e >> 3
    o = _philox_int([blk % 2**32, blk >> 32, site, layer_id], [seed % 2**32, seed >> 32])
    r16 = (o[(e & 7) >> 1] >> (16 * (e & 1))) & 0xFFFF
    from fractions import Fraction
    import math
    thr = math.floor(Fraction(float(np.float32(p))) * 65536 + Fraction(1, 2))   # exact rational arithmetic
    return r16 >= thr


def test_mask_element_mapping():
    seed = 0x1234567890ABCDEF
    m = philox.keep_mask(4096, 0.3, seed, 1, 7)
    for e in list(range(40)) + [1023, 1024, 4095]:
        assert bool(m[e]) == _keep_scalar(e, 0.3, seed, 1, 7)


def test_mask_statistics_and_independence():
    n = 1 << 21
    p = 0.1
    thr = philox.dropout_threshold(p)
    assert thr == 6554
    q = 1.0 - thr / 65536.0
    m0 = philox.keep_mask(n, p, 0, 0, 0)
    m1 = philox.keep_mask(n, p, 0, 1, 0)
    m2 = philox.keep_mask(n, p, 0, 0, 1)
    m3 = philox.keep_mask(n, p, 1, 0, 0)
    sigma = np.sqrt(q * (1 - q) / n)
    for m in (m0, m1, m2, m3):
        assert abs(m.mean() - q) < 4 * sigma
    for other in (m1, m2, m3):
        both = (m0 & other).mean()
        assert abs(both - q * q) < 5 * np.sqrt(q * q * (1 - q * q) / n)
    # neighbouring elements within one 8-element block are not tied together
    pairs = (m0[0::2] & m0[1::2]).mean()
    assert abs(pairs - q * q) < 5 * np.sqrt(q * q * (1 - q * q) / (n // 2))
    assert philox.keep_mask(10000, 0.0, 3, 0, 0).all()
    assert philox.keep_mask(1 << 16, 0.5, 3, 0, 0).mean() == pytest_approx(0.5, 0.01)


def pytest_approx(v, tol):
    import pytest
    return pytest.approx(v, abs=tol)


def test_threshold_rounding():
    """The threshold is round-half-away-from-zero of the SINGLE-precision probability times 2^16 (values by hand)."""
    assert philox.dropout_threshold(0.0) == 0
    assert philox.dropout_threshold(0.1) == 6554          # 6553.6
    assert philox.dropout_threshold(0.5) == 32768
    assert philox.dropout_threshold(0.25 + 2.0 ** -17) == 16385     # exactly 16384.5: the half goes up, not to even
    assert philox.dropout_threshold(0.25 + 3 * 2.0 ** -17) == 16386  # exactly 16385.5: up as well
    # 13107 * 2^-17 = 6553.5 / 65536 is a single-precision number; a double a hair below it rounds to it first
    assert philox.dropout_threshold(13107 * 2.0 ** -17 - 1e-12) == 6554
    # and the mask follows the threshold: a draw equal to the threshold is kept, one below is dropped
    thr = philox.dropout_threshold(0.25 + 2.0 ** -17)
    m_lo = philox.keep_mask(1 << 16, 0.25, 9, 0, 0)
    m_hi = philox.keep_mask(1 << 16, 0.25 + 2.0 ** -17, 9, 0, 0)
    assert thr == philox.dropout_threshold(0.25) + 1 and (m_lo | ~m_hi).all() and m_lo.sum() >= m_hi.sum()
