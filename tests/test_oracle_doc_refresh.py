"""Pins for the oracle's sweep with the doc side refreshed after every token (Sec. 4.2,
footnote 4) and the word side kept at the snapshot (Sec. 6).

  * a token's chain against a given assignment of its document follows the exact m-step law
    e_z0 (T_w T_d)^(m/2) whose doc side -- n_kd in the target of Eq. (4) and in the
    doc-proposal of Eq. (9) -- is recounted here from THAT assignment, while the word side is
    recounted from the snapshot;
  * with the snapshot itself as the assignment it is the ordinary chain, bit for bit;
  * the sweep is those chains folded over a document in token order.
"""
import numpy as np
import pytest

import test_oracle_mh as mh

K, V = mh.K, mh.V


def state_with_doc(o, doff, words, g, zdoc):
    """exact_setup, with the document's counts taken from zdoc instead of the snapshot."""
    st = mh.exact_setup(o, doff, words, g)
    ndk = np.bincount(zdoc, minlength=K)
    e = np.zeros(K)
    e[st["z0"]] = 1
    p = (ndk - e + mh.ALPHA) * (st["nkw"] - e + mh.BETA) / (st["nk"] - e + V * mh.BETA)
    qd = (ndk + mh.ALPHA) / (ndk.sum() + K * mh.ALPHA)
    return dict(st, ndk=ndk, p=p / p.sum(), qd=qd)


@pytest.fixture(scope="module")
def setup(oracle_mod):
    doff, words = mh.tiny_corpus()
    o = oracle_mod.Oracle(doff, words, V, K, mh.ALPHA, mh.BETA, seed=42)
    o.build_alias()
    return o, doff, words


def test_snapshot_assignment_gives_the_ordinary_chain(oracle_mod, setup):
    o, doff, words = setup
    z = o.get_z()
    ids = np.arange(o.N)
    for m in (1, 2, 3, 4):
        want = o.sweep_tokens(7, m, ids)
        for g in ids:
            d = int(np.searchsorted(doff, g, side="right") - 1)
            assert o.chain_with_doc(g, 7, m, z[doff[d]:doff[d + 1]]) == want[g]


@pytest.mark.parametrize("g,m", [(8, 2), (12, 2), (20, 4), (24, 3)])
def test_chain_follows_the_law_of_the_refreshed_document(oracle_mod, setup, g, m):
    o, doff, words = setup
    z = o.get_z()
    d = int(np.searchsorted(doff, g, side="right") - 1)
    b = int(doff[d])
    rng = np.random.default_rng(g)
    zdoc = z[b:doff[d + 1]].copy()
    moved = [i for i in range(len(zdoc)) if i != g - b]
    for i in moved[: max(2, len(moved) // 2)]:       # earlier and later tokens given new topics
        zdoc[i] = rng.integers(0, K)
    assert not np.array_equal(np.bincount(zdoc, minlength=K), np.bincount(z[b:doff[d + 1]], minlength=K))
    st = state_with_doc(o, doff, words, g, zdoc)
    Tw = mh.transition_matrix(oracle_mod, 1, st["qw"], st)
    Td = mh.transition_matrix(oracle_mod, 0, st["qd"], st)
    dist = np.zeros(K)
    dist[st["z0"]] = 1.0
    for j in range(m):
        dist = dist @ (Tw if j % 2 == 0 else Td)
    R = 120_000
    obs = np.bincount([o.chain_with_doc(g, 1000 + r, m, zdoc) for r in range(R)], minlength=K)
    ok, chi2 = mh.chi2_ok(obs, dist, R, 40.0)
    assert ok, (chi2, obs, R * dist)
    # the law of the stale document is told apart at this sample size
    st0 = mh.exact_setup(o, doff, words, g)
    Td0 = mh.transition_matrix(oracle_mod, 0, st0["qd"], st0)
    Tw0 = mh.transition_matrix(oracle_mod, 1, st0["qw"], st0)
    stale = np.zeros(K)
    stale[st0["z0"]] = 1.0
    for j in range(m):
        stale = stale @ (Tw0 if j % 2 == 0 else Td0)
    if np.abs(stale - dist).max() > 0.02:
        assert not mh.chi2_ok(obs, stale, R, 40.0)[0]


def test_sweep_is_the_fold_of_chains_in_token_order(oracle_mod):
    doff, words = mh.tiny_corpus()
    a = oracle_mod.Oracle(doff, words, V, K, mh.ALPHA, mh.BETA, seed=9)
    b = oracle_mod.Oracle(doff, words, V, K, mh.ALPHA, mh.BETA, seed=9)
    snap = oracle_mod.Oracle(doff, words, V, K, mh.ALPHA, mh.BETA, seed=9)
    for it, m in enumerate((2, 3, 1, 4)):
        a.build_alias(); b.build_alias(); snap.build_alias()
        z = b.get_z()
        want = z.copy()
        for d in range(len(doff) - 1):
            lo, hi = int(doff[d]), int(doff[d + 1])
            zc = z[lo:hi].copy()
            for g in range(lo, hi):
                zc[g - lo] = b.chain_with_doc(g, it, m, zc)
            want[lo:hi] = zc
        a.sweep_doc_refresh(m)
        assert a.get_z().tolist() == want.tolist()
        # the first token of a document has no refreshed neighbour: the ordinary chain
        first = doff[:-1][np.diff(doff) > 0]
        assert a.get_z()[first].tolist() == snap.sweep_tokens(it, m, first).tolist()
        if it == 0:
            assert a.get_z().tolist() != snap.sweep_tokens(it, m, np.arange(snap.N)).tolist()
        # both keep the same state afterwards (b and snap follow a)
        a.rebuild_counts()
        for x in (b, snap):
            x.set_z(a.get_z(), it + 1)
            x.rebuild_counts()
        assert int(a.get_nk().sum()) == a.N
