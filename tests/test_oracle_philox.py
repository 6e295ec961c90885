"""Pins for the oracle's Philox4x32-10 (the randomness of every MH step)."""
import os

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors(oracle_mod):
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle_mod.philox4x32_10(v[0:4], v[4:6])
        assert out.tolist() == v[6:10]


def test_counter_and_key_sensitivity(oracle_mod):
    # every counter word and key word must change the output (plumbing check)
    base = oracle_mod.philox4x32_10([1, 2, 3, 4], [5, 6]).tolist()
    for i in range(4):
        c = [1, 2, 3, 4]
        c[i] ^= 1
        assert oracle_mod.philox4x32_10(c, [5, 6]).tolist() != base
    for i in range(2):
        k = [5, 6]
        k[i] ^= 1
        assert oracle_mod.philox4x32_10([1, 2, 3, 4], k).tolist() != base


def test_uniformity_smoke(oracle_mod):
    # 4 x 20000 words, 16 equiprobable cells: chi-square far from the tail
    n = 20000
    xs = np.array([oracle_mod.philox4x32_10([i, 0, 7, 1], [123, 456]) for i in range(n)])
    cells = (xs >> 28).ravel()
    obs = np.bincount(cells, minlength=16)
    exp = cells.size / 16.0
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert chi2 < 50.0  # 15 dof: P(chi2 > 50) ~ 1e-5
