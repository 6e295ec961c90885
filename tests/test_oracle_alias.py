"""Pins for the oracle's alias table (Sec. 4.2, Fig. 2 of the paper).

The table is pinned by what an alias table *is*: drawing a uniform bin and a
uniform height reproduces the bin weights.  With integer masses this is an
exact identity, checked here without reference to how the table was built.
A second, independent construction (closed-form prefix sums, written in this
file with Python integers) must give the identical table: that is the form a
parallel build uses.
"""
import bisect

import numpy as np
import pytest


def reconstruct_masses(split, alias, cap):
    """Mass that a (bin, height) draw assigns to every outcome."""
    n = len(split)
    m = [0] * n
    for k in range(n):
        s = int(split[k])
        assert 1 <= s <= cap
        m[k] += s
        if s < cap:
            a = int(alias[k])
            assert 0 <= a < n and a != k
            m[a] += cap - s
    return m


def masses_by_definition(q0):
    """Integer masses m_k from the quantised weights, with Python integers."""
    n = len(q0)
    q0 = [int(x) for x in q0]
    Q0 = sum(q0)
    sh = 0
    while (Q0 >> sh) >= (n << 31):
        sh += 1
    q = [max(1, x >> sh) for x in q0]
    Q = sum(q)
    cap = -(-Q // n)
    pad = n * cap - Q
    assert 0 <= pad < n
    m = [q[k] + (1 if k < pad else 0) for k in range(n)]
    assert sum(m) == n * cap
    return m, cap


def closed_form_table(m, cap):
    """Prefix-sum construction: no sequential dependence between bins.

    lights l_0<l_1<.. (m<cap) with exclusive deficit sums Delta_a,
    heavies h_0<h_1<.. (m>=cap) with inclusive excess sums X_b:
      light  a: split = m, alias = h_b with b = min{b : X_b > Delta_a}
      heavy  b: a = min{a : Delta_a >= X_b}, split = cap + X_b - Delta_a,
                alias = h_{b+1} if split < cap else itself
    """
    n = len(m)
    lights = [k for k in range(n) if m[k] < cap]
    heavies = [k for k in range(n) if m[k] >= cap]
    delta = [0]
    for l in lights:
        delta.append(delta[-1] + cap - m[l])
    X = []
    acc = 0
    for h in heavies:
        acc += m[h] - cap
        X.append(acc)
    split = [0] * n
    alias = [0] * n
    for a, l in enumerate(lights):
        b = bisect.bisect_right(X, delta[a])
        split[l] = m[l]
        alias[l] = heavies[b]
    for b, h in enumerate(heavies):
        a = bisect.bisect_left(delta, X[b])
        s = cap + X[b] - delta[a]
        split[h] = s
        alias[h] = heavies[b + 1] if s < cap else h
    return split, alias


def check_table(oracle_mod, q0):
    q0 = np.asarray(q0, np.uint64)
    split, alias, cap = oracle_mod.alias_from_q0(q0)
    m_def, cap_def = masses_by_definition(q0)
    assert cap == cap_def
    m_or, cap_or = oracle_mod.alias_masses(q0)
    assert cap_or == cap and [int(x) for x in m_or] == m_def
    # exact alias property
    assert reconstruct_masses(split, alias, cap) == m_def
    # closed form == sequential build
    s2, a2 = closed_form_table(m_def, cap)
    assert [int(x) for x in split] == s2
    # an alias is only meaningful where split < cap
    for k in range(len(q0)):
        if s2[k] < cap:
            assert int(alias[k]) == a2[k]
        else:
            assert int(alias[k]) == k == a2[k]
    return split, alias, cap, m_def


def test_adversarial_shapes(oracle_mod):
    one = 1 << 40
    cases = [
        [one],                                   # K = 1
        [one, one],                              # K = 2 equal
        [1, one],                                # K = 2 extreme
        [one, 1],
        [5] * 7,                                 # all equal (every bin full)
        [one] + [1] * 63,                        # one giant bin
        [1] * 63 + [one],
        [7, 7, 7, 100, 7, 7, 7],
        [10, 10, 10, 10, 40, 10, 10, 10, 10, 0],  # a zero weight is lifted to 1
        list(range(1, 200)),
        list(range(200, 0, -1)),
        [one] * 1000,                            # forces a right shift (sum >= n*2^31)
        [3, 9, 3, 9, 3, 9, 6, 6, 6],             # runs with m == cap
    ]
    for q0 in cases:
        check_table(oracle_mod, q0)


def test_random_tables_small_exhaustive_style(oracle_mod):
    rng = np.random.default_rng(11)
    for _ in range(3000):
        n = int(rng.integers(1, 13))
        kind = rng.integers(0, 3)
        if kind == 0:
            q0 = rng.integers(0, 20, n)
        elif kind == 1:
            q0 = rng.integers(0, 1 << 40, n)
        else:
            q0 = (rng.random(n) ** 8 * (1 << 40)).astype(np.uint64)
        if int(np.sum(q0)) == 0:
            q0[0] = 1
        check_table(oracle_mod, q0)


def test_random_tables_large(oracle_mod):
    rng = np.random.default_rng(12)
    for n in (64, 100, 1000, 4097):
        w = rng.gamma(0.05, 1.0, n) + 1e-9
        w /= w.max()
        q0 = np.floor(w * 2.0 ** 40).astype(np.uint64)
        check_table(oracle_mod, q0)


def test_dense_row_matches_word_proposal(oracle_mod):
    """Table of a word == (n_kw + beta)/(n_k + betabar), Eq. (6), to 2^-30."""
    rng = np.random.default_rng(13)
    K, V, beta = 50, 40, 0.01
    betabar = V * beta
    nk = rng.integers(0, 500, K).astype(np.int32)
    row = np.minimum(rng.integers(0, 30, K) * (rng.random(K) < 0.3), nk).astype(np.int32)
    split, alias, cap = oracle_mod.alias_build_dense_row(row, nk, beta, betabar)
    m = np.array(reconstruct_masses(split, alias, cap), dtype=np.float64)
    p_tab = m / (K * float(cap))
    a = (row + beta) / (nk + betabar)
    p = a / a.sum()
    assert np.max(np.abs(p_tab - p)) < 2.0 ** -30
    # and the order of magnitudes survives (a transposed n_kw / n_k would not)
    assert np.argmax(p_tab) == np.argmax(p)


def test_draws_follow_weights(oracle_mod):
    rng = np.random.default_rng(14)
    K = 12
    w = rng.random(K) ** 3 + 1e-3
    q0 = np.floor(w / w.max() * 2.0 ** 40).astype(np.uint64)
    split, alias, cap = oracle_mod.alias_from_q0(q0)
    R = 200_000
    xs = rng.integers(0, 1 << 32, (R, 2), dtype=np.uint64)
    draws = np.array([oracle_mod.alias_draw(split, alias, cap, a, b) for a, b in xs])
    obs = np.bincount(draws, minlength=K)
    exp = R * w / w.sum()
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert chi2 < 45.0  # 11 dof, P(chi2 > 45) ~ 5e-6
    # the draw rule itself: bin = floor(x0*K / 2^32), height = floor(x1*cap / 2^32)
    for a, b in xs[:2000]:
        bin_ = (int(a) * K) >> 32
        h = (int(b) * cap) >> 32
        want = bin_ if h < int(split[bin_]) else int(alias[bin_])
        assert oracle_mod.alias_draw(split, alias, cap, a, b) == want


def test_planted_mistake_is_caught(oracle_mod):
    """The mass check is sharp: moving one unit of mass breaks it."""
    q0 = np.array([3, 9, 2, 30, 1, 8], np.uint64)
    split, alias, cap = oracle_mod.alias_from_q0(q0)
    m_def, _ = masses_by_definition(q0)
    bad = split.copy()
    k = int(np.argmax(split < cap))
    bad[k] += 1
    assert reconstruct_masses(bad, alias, cap) != m_def
