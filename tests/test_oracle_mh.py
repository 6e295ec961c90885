"""Pins for the oracle's MH steps against the exact collapsed-Gibbs conditional.

Everything the oracle is compared with here is computed in this file from the
paper's definitions: the target p(k) of Eq. (1)/(4) from a numpy recount, the
word-proposal of Eq. (6) and the doc-proposal of Eq. (9).  The oracle's coded
acceptance (Eq. 8 and 11) enters only through its accept/reject answers.
"""
import numpy as np
import pytest

from test_oracle_alias import reconstruct_masses

K, V, D = 6, 8, 5
ALPHA, BETA = 0.3, 0.2


def tiny_corpus(seed=5):
    rng = np.random.default_rng(seed)
    lens = np.array([6, 1, 9, 4, 7])
    doff = np.zeros(D + 1, np.int64)
    doff[1:] = np.cumsum(lens)
    words = rng.integers(0, V, doff[-1]).astype(np.int32)
    return doff, words


def exact_setup(o, doff, words, g):
    """Counts by numpy recount and the exact conditional of token g (Eq. 4)."""
    z = o.get_z()
    d = int(np.searchsorted(doff, g, side="right") - 1)
    w = int(words[g])
    nk = np.bincount(z, minlength=K)
    nkw = np.bincount(z[words == w], minlength=K)
    ndk = np.bincount(z[doff[d]:doff[d + 1]], minlength=K)
    z0 = int(z[g])
    e = np.zeros(K)
    e[z0] = 1
    betabar = V * BETA
    p = (ndk - e + ALPHA) * (nkw - e + BETA) / (nk - e + betabar)
    p /= p.sum()
    qw = (nkw + BETA) / (nk + betabar)
    qw /= qw.sum()
    qd = (ndk + ALPHA) / (ndk.sum() + K * ALPHA)
    return dict(d=d, w=w, z0=z0, nk=nk, nkw=nkw, ndk=ndk, p=p, qw=qw, qd=qd)


def accept_probability(oracle_mod, word_step, s, t, st):
    """P(accept) of the coded test: the count of x2 values that accept / 2^32.

    The test is monotone in x2 (accept iff u*den < num, u increasing in x2),
    so the count is found by bisection over the 2^32 possible x2.
    """
    betabar = V * BETA

    def acc(x2):
        return oracle_mod.mh_accept(word_step, s, t, st["z0"], int(st["ndk"][s]), int(st["ndk"][t]),
                                    int(st["nkw"][s]), int(st["nkw"][t]), int(st["nk"][s]),
                                    int(st["nk"][t]), ALPHA, BETA, betabar, x2)

    if not acc(0):
        return 0.0
    if acc(2 ** 32 - 1):
        return 1.0
    lo, hi = 0, 2 ** 32 - 1  # acc(lo) = 1, acc(hi) = 0
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if acc(mid):
            lo = mid
        else:
            hi = mid
    return hi / 2.0 ** 32


def transition_matrix(oracle_mod, word_step, q, st):
    T = np.zeros((K, K))
    for s in range(K):
        for t in range(K):
            if t != s:
                T[s, t] = q[t] * accept_probability(oracle_mod, word_step, s, t, st)
        T[s, s] = 1.0 - T[s].sum()
    return T


@pytest.fixture(scope="module")
def setup(oracle_mod):
    doff, words = tiny_corpus()
    o = oracle_mod.Oracle(doff, words, V, K, ALPHA, BETA, seed=42)
    o.build_alias()
    return o, doff, words


@pytest.mark.parametrize("g", [0, 3, 6, 11, 26])
def test_detailed_balance_of_coded_acceptance(oracle_mod, setup, g):
    """p_s T(s,t) = p_t T(t,s) for both proposals: pins Eq. (8) and Eq. (11)."""
    o, doff, words = setup
    st = exact_setup(o, doff, words, g)
    for word_step, q in ((1, st["qw"]), (0, st["qd"])):
        T = transition_matrix(oracle_mod, word_step, q, st)
        flow = st["p"][:, None] * T
        assert np.max(np.abs(flow - flow.T)) < 1e-8
        assert np.max(np.abs(st["p"] @ T - st["p"])) < 1e-8
    # acceptance equals min(1, p(t) q(s) / (p(s) q(t))) -- Eq. (7) and (10)
    for word_step, q in ((1, st["qw"]), (0, st["qd"])):
        for s in range(K):
            for t in range(K):
                if s != t:
                    want = min(1.0, st["p"][t] * q[s] / (st["p"][s] * q[t]))
                    got = accept_probability(oracle_mod, word_step, s, t, st)
                    assert abs(got - want) < 1e-8


def test_uniform_proposal_special_case(oracle_mod, setup):
    """When the proposal factors cancel the ratio is p(t)/p(s) (Sec. 4.1)."""
    o, doff, words = setup
    st = exact_setup(o, doff, words, 8)
    # doc-step ratio with n_sd = n_td has equal proposal factors
    ndk = st["ndk"].copy()
    s, t = 1, 4
    ndk[s] = ndk[t] = 2
    st2 = dict(st, ndk=ndk, z0=0)
    e = np.zeros(K)
    e[0] = 1
    p = (ndk - e + ALPHA) * (st["nkw"] - e + BETA) / (st["nk"] - e + V * BETA)
    got = accept_probability(oracle_mod, 0, s, t, st2)
    assert abs(got - min(1.0, p[t] / p[s])) < 1e-8


def word_table_masses(o, w):
    split, alias, cap = o.get_alias_row(w)
    m = np.array(reconstruct_masses(split, alias, cap), dtype=np.float64)
    return m / m.sum()


def test_word_table_is_word_proposal(oracle_mod, setup):
    o, doff, words = setup
    for g in (0, 6, 26):
        st = exact_setup(o, doff, words, g)
        assert np.max(np.abs(word_table_masses(o, st["w"]) - st["qw"])) < 1e-8


def chain_histogram(o, g, m, R, first_sweep=1000):
    out = np.zeros(K, np.int64)
    tok = np.array([g], np.int64)
    for r in range(R):
        out[o.sweep_tokens(first_sweep + r, m, tok)[0]] += 1
    return out


def chi2_ok(obs, prob, R, limit):
    exp = R * prob
    keep = exp > 5
    chi2 = ((obs[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    return chi2 < limit, chi2


@pytest.mark.parametrize("g,m", [(0, 1), (0, 2), (6, 2), (11, 4), (26, 3)])
def test_chain_matches_exact_m_step_distribution(oracle_mod, setup, g, m):
    """Histogram of the token's final state over independent replicas (different
    sweep indices, frozen counts) vs e_z0 (T_w T_d)^(m/2) -- pins the RNG plumbing,
    the draw routines, the step order (word first) and the state carry-over."""
    o, doff, words = setup
    st = exact_setup(o, doff, words, g)
    Tw = transition_matrix(oracle_mod, 1, st["qw"], st)
    Td = transition_matrix(oracle_mod, 0, st["qd"], st)
    dist = np.zeros(K)
    dist[st["z0"]] = 1.0
    for j in range(m):
        dist = dist @ (Tw if j % 2 == 0 else Td)
    R = 120_000
    obs = chain_histogram(o, g, m, R)
    ok, chi2 = chi2_ok(obs, dist, R, 40.0)  # <= 5 dof: P(chi2 > 40) ~ 1e-7
    assert ok, (chi2, obs, R * dist)
    # the other step order is distinguishable at this sample size for m >= 2
    if m == 2:
        wrong = np.zeros(K)
        wrong[st["z0"]] = 1.0
        wrong = wrong @ Td @ Tw
        if np.abs(wrong - dist).max() > 0.02:
            assert not chi2_ok(obs, wrong, R, 40.0)[0]


@pytest.mark.parametrize("g", [3, 14])
def test_long_chain_reaches_exact_conditional(oracle_mod, setup, g):
    """After many cycles the token is distributed as Eq. (4) itself."""
    o, doff, words = setup
    st = exact_setup(o, doff, words, g)
    R = 60_000
    obs = chain_histogram(o, g, 64, R)
    ok, chi2 = chi2_ok(obs, st["p"], R, 40.0)
    assert ok, (chi2, obs, R * st["p"])


def test_doc_draw_histogram(oracle_mod):
    """Doc-proposal draws follow (n_dk + alpha)/(L + K alpha), Eq. (9) and (12)."""
    rng = np.random.default_rng(3)
    Kd, alpha = 7, 0.4
    zdoc = np.array([2, 2, 5, 0, 2, 5, 6, 6, 2], np.int32)
    L = len(zdoc)
    R = 200_000
    xs = rng.integers(0, 1 << 32, (R, 2), dtype=np.uint64)
    draws = np.array([oracle_mod.doc_draw(L, Kd, Kd * alpha, zdoc, a, b) for a, b in xs])
    want = (np.bincount(zdoc, minlength=Kd) + alpha) / (L + Kd * alpha)
    ok, chi2 = chi2_ok(np.bincount(draws, minlength=Kd), want, R, 45.0)
    assert ok, chi2
    # one-token document: either its own topic or a uniform one
    z1 = np.array([3], np.int32)
    d1 = np.array([oracle_mod.doc_draw(1, Kd, Kd * alpha, z1, a, b) for a, b in xs[:50_000]])
    want1 = (np.bincount(z1, minlength=Kd) + alpha) / (1 + Kd * alpha)
    assert chi2_ok(np.bincount(d1, minlength=Kd), want1, 50_000, 45.0)[0]


def test_mixture_word_proposal(oracle_mod):
    """Sparsified word-proposal (Sec. 4.2): sparse term + shared beta term have
    the same total distribution as Eq. (6), and the chain still has the exact
    m-step law."""
    doff, words = tiny_corpus()
    o = oracle_mod.Oracle(doff, words, V, K, ALPHA, BETA, seed=42, dense_alias_min_count=10 ** 6)
    o.build_alias()
    bs, ba, bc, QB = o.get_beta_table()
    mb = np.array(reconstruct_masses(bs, ba, bc), dtype=np.float64)
    for g in (0, 11):
        st = exact_setup(o, doff, words, g)
        topics, ss, sa, sc, QS = o.get_sparse_table(st["w"])
        assert topics.tolist() == np.nonzero(st["nkw"])[0].tolist()
        ms = np.array(reconstruct_masses(ss, sa, sc), dtype=np.float64)
        mix = np.zeros(K)
        mix[topics] += QS / (QS + QB) * ms / ms.sum()
        mix += QB / (QS + QB) * mb / mb.sum()
        assert np.max(np.abs(mix - st["qw"])) < 1e-8
        # term masses as defined: floor(weight * 2^40) summed
        betabar = V * BETA
        assert QB == sum(int(np.floor(BETA / (n + betabar) * 2.0 ** 40)) for n in st["nk"])
        assert QS == sum(int(np.floor(st["nkw"][k] / (st["nk"][k] + betabar) * 2.0 ** 40))
                         for k in topics)
        Tw = transition_matrix(oracle_mod, 1, st["qw"], st)
        Td = transition_matrix(oracle_mod, 0, st["qd"], st)
        dist = np.zeros(K)
        dist[st["z0"]] = 1.0
        dist = dist @ Tw @ Td
        R = 120_000
        obs = chain_histogram(o, g, 2, R)
        ok, chi2 = chi2_ok(obs, dist, R, 40.0)
        assert ok, (chi2, obs, R * dist)


def test_proposal_modes(oracle_mod):
    """word-only / doc-only chains use one transition matrix throughout."""
    doff, words = tiny_corpus()
    for mode in (1, 2):
        o = oracle_mod.Oracle(doff, words, V, K, ALPHA, BETA, seed=42, proposal_mode=mode)
        o.build_alias()
        st = exact_setup(o, doff, words, 6)
        T = transition_matrix(oracle_mod, 1 if mode == 1 else 0,
                              st["qw"] if mode == 1 else st["qd"], st)
        dist = np.zeros(K)
        dist[st["z0"]] = 1.0
        dist = dist @ T @ T
        R = 80_000
        obs = chain_histogram(o, 6, 2, R)
        ok, chi2 = chi2_ok(obs, dist, R, 40.0)
        assert ok, (mode, chi2)


def test_sweep_equals_per_token_chains_and_is_deterministic(oracle_mod):
    doff, words = tiny_corpus()
    a = oracle_mod.Oracle(doff, words, V, K, ALPHA, BETA, seed=9)
    b = oracle_mod.Oracle(doff, words, V, K, ALPHA, BETA, seed=9)
    a.build_alias()
    b.build_alias()
    per_token = b.sweep_tokens(0, 3, np.arange(b.N))
    a.sweep(3)
    assert a.get_z().tolist() == per_token.tolist()
    b.sweep(3)
    assert a.get_z().tolist() == b.get_z().tolist()
    c = oracle_mod.Oracle(doff, words, V, K, ALPHA, BETA, seed=10)
    c.build_alias()
    c.sweep(3)
    assert c.get_z().tolist() != a.get_z().tolist()
