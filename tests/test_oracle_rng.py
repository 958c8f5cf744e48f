"""Pins of the oracle's counter-based generator (oracle/rng.py), all CPU.

* the published known-answer vectors of Philox4x32-10 (tests/golden/philox4x32_10_kat.txt) catch any mistake in the
  round function, the multipliers, the key schedule or the number of rounds;
* a 64-bit-arithmetic restatement with numpy integer arrays (different code: vectorised, uint64 products) must agree
  on random counters and keys;
* the uniform mapping: value = top 24 bits * 2^-24, inside [0, 1), exactly a float32; counter layout: each of index,
  purpose, call (both halves) and seed (both halves) changes the number; first two moments and a coarse histogram of
  100 000 draws are those of U[0, 1).
"""
import os

import numpy as np

from oracle import rng

HERE = os.path.dirname(os.path.abspath(__file__))


def test_known_answer_vectors():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert list(rng.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def philox_vectorised(ctr, key):
    """ctr [n][4], key [n][2] uint64 arrays holding 32-bit words; the same function on whole arrays."""
    c = ctr.astype(np.uint64).copy()
    k = key.astype(np.uint64).copy()
    m32 = np.uint64(0xFFFFFFFF)
    for rnd in range(10):
        if rnd:
            k[:, 0] = (k[:, 0] + np.uint64(0x9E3779B9)) & m32
            k[:, 1] = (k[:, 1] + np.uint64(0xBB67AE85)) & m32
        p0 = np.uint64(0xD2511F53) * c[:, 0]
        p1 = np.uint64(0xCD9E8D57) * c[:, 2]
        n = np.empty_like(c)
        n[:, 0] = (p1 >> np.uint64(32)) ^ c[:, 1] ^ k[:, 0]
        n[:, 1] = p1 & m32
        n[:, 2] = (p0 >> np.uint64(32)) ^ c[:, 3] ^ k[:, 1]
        n[:, 3] = p0 & m32
        c = n
    return c


def test_against_vectorised_restatement():
    g = np.random.default_rng(5)
    ctr = g.integers(0, 2 ** 32, size=(200, 4), dtype=np.uint64)
    key = g.integers(0, 2 ** 32, size=(200, 2), dtype=np.uint64)
    out = philox_vectorised(ctr, key)
    for i in range(200):
        assert list(rng.philox4x32_10(ctr[i], key[i])) == [int(x) for x in out[i]]


def test_uniform_mapping_and_counter_layout():
    u = rng.uniform(seed=0x1234567890ABCDEF, call=7, purpose=rng.DRAFT, index=3)
    assert u.dtype == np.float32 and 0.0 <= float(u) < 1.0
    w0 = rng.philox4x32_10((3, rng.DRAFT, 7, 0), (0x90ABCDEF, 0x12345678))[0]
    assert float(u) == (w0 >> 8) / 2.0 ** 24
    assert float(u) * 2 ** 24 == int(float(u) * 2 ** 24)            # 24 bits: exact in float32
    base = dict(seed=0x1234567890ABCDEF, call=7, purpose=rng.DRAFT, index=3)
    for change in (dict(index=4), dict(purpose=rng.ACCEPT), dict(call=8), dict(call=7 + 2 ** 32), dict(seed=0x1234567890ABCDEE),
                   dict(seed=0x0234567890ABCDEF)):
        assert float(rng.uniform(**{**base, **change})) != float(u), change
    assert np.array_equal(rng.uniforms(9, 2, rng.ACCEPT, 5), np.array([rng.uniform(9, 2, rng.ACCEPT, i) for i in range(5)], np.float32))


def test_moments_and_histogram():
    n = 100000
    ctr = np.zeros((n, 4), np.uint64); ctr[:, 0] = np.arange(n); ctr[:, 1] = rng.DRAFT; ctr[:, 2] = 11
    key = np.tile(np.array([[42, 0]], np.uint64), (n, 1))
    u = (philox_vectorised(ctr, key)[:, 0] >> np.uint64(8)).astype(np.float64) / 2.0 ** 24
    assert float(u[17]) == float(rng.uniform(42, 11, rng.DRAFT, 17))
    assert abs(u.mean() - 0.5) < 4 * (1 / 12 / n) ** 0.5
    assert abs(u.var() - 1 / 12) < 0.002
    hist = np.bincount((u * 16).astype(int), minlength=16)
    chi2 = float(((hist - n / 16) ** 2 / (n / 16)).sum())
    assert chi2 < 45.0                                              # 15 degrees of freedom: P(chi2 > 45) < 1e-4
    assert len(np.unique(u)) > 0.99 * n
