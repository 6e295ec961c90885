"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle sweeps 10^8 tokens in half a minute (c2: every token is compared) but not 10^9,
so for the larger workloads, after an exhaustive comparison of the initial state (z, n_k),
it is asked for the chains of sampled tokens only, for n_kw rows and word-proposal tables
of sampled words (the most frequent word -- many rebuild tiles --, words of every storage
class, rare ones), and the GPU's post-sweep counts are checked against a numpy recount of
the GPU's own assignment (a property that holds at any size).  Where the V x K table does
not fit in host memory (c4, c5) the oracle counts a word's row when it is first needed
(lazy_rows; pinned to the plain oracle in tests/test_oracle_storage.py).
"""
import numpy as np
import pytest

from paper_1412_1576_amd import corpus

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lda_mod():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1412_1576_amd import lda
    lda.load_library()
    return lda


def sampled_check(lda_mod, oracle_mod, cfg, mh_steps, n_tokens=2000, n_words=12, seed=123,
                  min_count=0, dense_rows=0, lazy_rows=False, stream_block_tokens=0):
    """min_count > 0: words with fewer tokens draw from the mixture (bench.py's default form).
    min_count < 0: bench.py's rule for the hybrid store -- dense tables only for words with at
    least K tokens and more tokens than any word without a dense row.  dense_rows: as
    lda_options (the oracle has no such notion: storage does not change a result)."""
    rng = np.random.default_rng(seed)
    doff, words = corpus.make_corpus(cfg)
    N = int(doff[-1])
    freq = np.bincount(words, minlength=cfg.V)
    if min_count < 0:
        min_count = max(int(freq[max(dense_rows, 0):].max()) + 1, cfg.K)
    g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                    dense_rows=dense_rows, dense_alias_min_count=min_count,
                    stream_block_tokens=stream_block_tokens)
    o = oracle_mod.Oracle(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                          dense_alias_min_count=min_count, lazy_alias=True, lazy_rows=lazy_rows)
    # initial state: exhaustive
    z_init = g.get_z()
    assert np.array_equal(z_init, o.get_z())
    assert np.array_equal(g.get_nk(), o.get_nk())
    order = np.argsort(-freq, kind="stable")
    sample_words = list(order[:3]) + list(order[[len(order) // 2, -1]]) + \
        list(rng.choice(cfg.V, n_words - 5, replace=False))
    special = []   # words of every storage class of the hybrid store
    if dense_rows != 0:
        H = max(dense_rows, 0)
        below = np.flatnonzero(freq[:H] < min_count)     # dense row, mixture table
        if len(below):
            special += [int(below[0]), int(below[len(below) // 2]), int(below[-1])]
        tail = H + np.flatnonzero(freq[H:] > 0)          # sparse row (list + hash row)
        special += [int(tail[0]), int(tail[len(tail) // 2]), int(tail[-1])]
        special.append(int(H + np.argmax(freq[H:])))
        sample_words += special
    for w in sample_words:
        assert np.array_equal(g.get_nkw_row(w), o.get_nkw_row(w)), "n_kw row %d" % w
    docs = rng.choice(cfg.D, 20, replace=False)
    for d in docs:
        assert np.array_equal(g.get_ndk_row(d), o.get_ndk_row(d)), "n_dk row %d" % d
    # alias tables of the sampled words
    g.build_alias()
    o.build_alias()
    if min_count:
        assert g.get_beta_table()[2:] == o.get_beta_table()[2:]
    for w in sample_words:
        if min_count and freq[w] < min_count:   # mixture word: its own table over its non-zeros
            t, sp, at, c, qs = g.get_sparse_table(w)
            ot, osp, oal, oc, oqs = o.get_sparse_table(w)
            assert np.array_equal(t, ot) and np.array_equal(sp, osp), "mixture table %d" % w
            assert len(t) == 0 or ((c, qs) == (oc, oqs) and
                                   np.array_equal(at, ot[oal.astype(np.int64)])), "mixture table %d" % w
            continue
        sg, ag, cg = g.get_alias_row(w)
        so, ao, co = o.get_alias_row(w)
        assert cg == co and np.array_equal(sg, so) and np.array_equal(ag, ao), "alias row %d" % w
    # the sweep: sampled chains (tokens of the hottest word, of rare words, uniform ones)
    head = words[: 20_000_000]
    ids = np.unique(np.concatenate([
        rng.choice(N, n_tokens, replace=False),
        np.flatnonzero(head == order[0])[:200],
        np.flatnonzero(words == order[-1])[:50],
        np.array([0, N - 1]),
    ] + [np.flatnonzero(head == w)[:40] for w in special])).astype(np.int64)
    want = o.sweep_tokens(0, mh_steps, ids)
    g.sweep(mh_steps)
    z_new = g.get_z()
    assert np.array_equal(z_new[ids], want), \
        "%d of %d sampled tokens differ" % (int((z_new[ids] != want).sum()), len(ids))
    assert 0 <= z_new.min() and z_new.max() < cfg.K
    assert (z_new != z_init).mean() > 0.05  # the sweep did move tokens
    # rebuilt counts against a recount of the GPU's own assignment
    g.rebuild_counts()
    nk = g.get_nk()
    assert np.array_equal(nk, np.bincount(z_new, minlength=cfg.K))
    assert int(nk.sum()) == N
    for w in sample_words[:6]:
        row = np.bincount(z_new[words == w], minlength=cfg.K)
        assert np.array_equal(g.get_nkw_row(w), row), "rebuilt n_kw row %d" % w
    for d in docs[:8]:
        row = np.bincount(z_new[doff[d]:doff[d + 1]], minlength=cfg.K)
        assert np.array_equal(g.get_ndk_row(d), row), "rebuilt n_dk row %d" % d
    g.close()
    o.close()


@pytest.mark.timeout(600)
def test_c2_full_size_sampled(lda_mod, oracle_mod):
    cfg = corpus.CONFIGS["c2"]
    sampled_check(lda_mod, oracle_mod, cfg, cfg.mh_steps)


@pytest.mark.timeout(900)
def test_c3_full_size_sampled(lda_mod, oracle_mod):
    """The benchmark's workload (K = 10,000), with the config's own 4 MH steps."""
    cfg = corpus.CONFIGS["c3"]
    sampled_check(lda_mod, oracle_mod, cfg, cfg.mh_steps, n_tokens=1500, n_words=10)


@pytest.mark.timeout(900)
def test_c3_full_size_bench_configuration(lda_mod, oracle_mod):
    """The workload exactly as bench.py times it: 2 steps, dense tables for words with at
    least K tokens, the mixture for the others."""
    cfg = corpus.CONFIGS["c3"]
    sampled_check(lda_mod, oracle_mod, cfg, 2, n_tokens=1500, n_words=10, min_count=cfg.K)


@pytest.mark.timeout(900)
def test_c2_full_size_every_token(lda_mod, oracle_mod):
    """One whole iteration of c2 (9.9 * 10^7 tokens) against the oracle: every token's new
    topic, n_k, sampled n_kw rows, and the log-likelihood before and after."""
    cfg = corpus.CONFIGS["c2"]
    doff, words = corpus.make_corpus(cfg)
    rng = np.random.default_rng(11)
    for min_count in (cfg.K,):      # the form bench.py times
        g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                        dense_alias_min_count=min_count)
        o = oracle_mod.Oracle(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                              dense_alias_min_count=min_count, lazy_alias=True)
        lg, lo = g.loglik(), o.loglik()
        assert abs(lg[0] - lo[0]) <= 1e-9 * abs(lo[0]), (lg, lo)
        g.build_alias(); o.build_alias()
        g.sweep(cfg.mh_steps); o.sweep(cfg.mh_steps)
        g.rebuild_counts(); o.rebuild_counts()
        zg, zo = g.get_z(), o.get_z()
        assert np.array_equal(zg, zo), "%d of %d tokens differ" % (int((zg != zo).sum()), len(zg))
        assert np.array_equal(g.get_nk(), o.get_nk())
        freq = np.bincount(words, minlength=cfg.V)
        order = np.argsort(-freq, kind="stable")
        for w in list(order[:5]) + list(order[[1000, 20000, -1]]) + list(rng.choice(cfg.V, 42, replace=False)):
            assert np.array_equal(g.get_nkw_row(w), o.get_nkw_row(w)), "n_kw row %d" % w
        lg, lo = g.loglik(), o.loglik()
        assert abs(lg[0] - lo[0]) <= 1e-9 * abs(lo[0]), (lg, lo)
        for a, b in zip(lg[1:], lo[1:]):
            assert abs(a - b) <= 1e-9 * max(abs(b), abs(lo[0])), (lg, lo)
        g.close()
        o.close()


@pytest.mark.timeout(900)
def test_c3_loglik_and_every_token_on_600k_documents(lda_mod, oracle_mod):
    """The first 600 000 documents of c3 (5.4 * 10^7 tokens, the benchmark's V and K): the
    log-likelihood of 10^7..10^8 terms -- where the order of the block partial sums matters
    most -- within 1e-9 of the oracle, before and after one whole iteration in the form
    bench.py times, and every token of that iteration."""
    cfg = corpus.scaled(corpus.CONFIGS["c3"], D=600_000)
    doff, words = corpus.make_corpus(cfg)
    g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                    dense_alias_min_count=cfg.K)
    o = oracle_mod.Oracle(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                          dense_alias_min_count=cfg.K, lazy_alias=True, lazy_rows=True)
    for it in range(2):
        lg, lo = g.loglik(), o.loglik()
        assert abs(lg[0] - lo[0]) <= 1e-9 * abs(lo[0]), (it, lg, lo)
        for a, b in zip(lg[1:], lo[1:]):
            assert abs(a - b) <= 1e-9 * max(abs(b), abs(lo[0])), (it, lg, lo)
        if it == 1:
            break
        g.build_alias(); o.build_alias()
        g.sweep(2); o.sweep(2)
        g.rebuild_counts(); o.rebuild_counts()
        zg, zo = g.get_z(), o.get_z()
        assert np.array_equal(zg, zo), "%d of %d tokens differ" % (int((zg != zo).sum()), len(zg))
        assert np.array_equal(g.get_nk(), o.get_nk())
    g.close()
    o.close()


@pytest.mark.timeout(1100)
def test_c4_full_size_sampled(lda_mod, oracle_mod):
    """K = 100 000 on the hybrid store at full size (10^9 tokens, V = 10^6), as bench.py runs
    it: sampled chains, rows, dense / mixture / shared tables and n_k against the oracle."""
    cfg = corpus.CONFIGS["c4"]
    sampled_check(lda_mod, oracle_mod, cfg, cfg.mh_steps, n_tokens=1500, n_words=10, min_count=-1,
                  dense_rows=cfg.dense_rows, lazy_rows=True)


@pytest.mark.timeout(1100)
def test_c5_full_size_sampled(lda_mod, oracle_mod):
    """One K = 10^6 slice with no dense row at full size (5 * 10^8 tokens)."""
    cfg = corpus.CONFIGS["c5"]
    sampled_check(lda_mod, oracle_mod, cfg, cfg.mh_steps, n_tokens=1500, n_words=10, min_count=-1,
                  dense_rows=-1, lazy_rows=True)


@pytest.mark.timeout(1100)
def test_c5_full_size_streamed_blocks(lda_mod, oracle_mod):
    """The K = 10^6 slice as its workload words it: 5 * 10^8 tokens streamed from pinned host
    memory in five blocks of 10^8 tokens (lda_options.stream_block_tokens).  Same checks as
    the resident run: initial state, rows, tables, sampled chains and n_k against the oracle."""
    cfg = corpus.CONFIGS["c5"]
    sampled_check(lda_mod, oracle_mod, cfg, cfg.mh_steps, n_tokens=1500, n_words=10, min_count=-1,
                  dense_rows=-1, lazy_rows=True, stream_block_tokens=100_000_000)


def property_check(lda_mod, cfg, dense_rows, mh_steps, seed=5):
    """Invariants and numpy recounts of the GPU's own assignment over two iterations of the
    hybrid-store workloads (their chains, rows and tables meet the oracle in the tests above)."""
    rng = np.random.default_rng(seed)
    doff, words = corpus.make_corpus(cfg)
    N = int(doff[-1])
    cnt = np.bincount(words, minlength=cfg.V)
    # as bench.py: dense tables only for words with at least K tokens and a dense row
    min_count = max(int(cnt[max(dense_rows, 0):].max()) + 1, cfg.K)
    g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=cfg.lib_seed,
                    dense_rows=dense_rows, dense_alias_min_count=min_count)
    order = np.argsort(-cnt, kind="stable")
    sample_words = list(order[:2]) + [int(order[len(order) // 3])] + \
        list(rng.choice(cfg.V, 5, replace=False))
    docs = rng.choice(cfg.D, 6, replace=False)
    z_prev = g.get_z()
    for it in range(2):
        nk = g.get_nk()
        assert np.array_equal(nk, np.bincount(z_prev, minlength=cfg.K)) and int(nk.sum()) == N
        for w in sample_words:
            row = np.bincount(z_prev[words == w], minlength=cfg.K)
            assert np.array_equal(g.get_nkw_row(w), row), "n_kw row %d" % w
        for d in docs:
            row = np.bincount(z_prev[doff[d]:doff[d + 1]], minlength=cfg.K)
            assert np.array_equal(g.get_ndk_row(d), row), "n_dk row %d" % d
        if it == 1:
            break
        ll0 = g.loglik()[0]
        g.build_alias()
        # mixture tables: structural invariants of an alias table over the word's non-zeros
        for w in sample_words:
            if cnt[w] >= min_count:
                continue
            t, s, at, c, qs = g.get_sparse_table(w)
            nz = np.flatnonzero(np.bincount(z_prev[words == w], minlength=cfg.K))
            assert np.array_equal(t, nz)
            if len(t):
                assert s.min() >= 1 and s.max() <= c and np.isin(at, t).all()
                mass = s.astype(np.int64).copy()
                pos = np.searchsorted(t, at)
                np.add.at(mass, pos[s < c], (c - s[s < c]).astype(np.int64))
                assert mass.sum() == len(t) * c
        g.sweep(mh_steps)
        g.rebuild_counts()
        z_new = g.get_z()
        assert 0 <= z_new.min() and z_new.max() < cfg.K
        assert (z_new != z_prev).mean() > 0.05
        assert g.loglik()[0] > ll0  # one sweep from a uniform start improves the likelihood
        z_prev = z_new
    g.close()


@pytest.mark.timeout(900)
def test_c4_full_size_properties(lda_mod):
    cfg = corpus.CONFIGS["c4"]
    property_check(lda_mod, cfg, cfg.dense_rows, cfg.mh_steps)


@pytest.mark.timeout(900)
def test_c5_full_size_properties(lda_mod):
    cfg = corpus.CONFIGS["c5"]
    property_check(lda_mod, cfg, -1, cfg.mh_steps)


@pytest.mark.timeout(900)
def test_near_the_token_limit(lda_mod):
    """2.11 * 10^9 tokens (the limit is 2^31 - 2^20 - 1): token positions are 32-bit, so this
    is where an overflow in the index arithmetic would show.  No oracle at this size: counts
    and sampled rows against numpy recounts of the library's own z."""
    cfg = corpus.scaled(corpus.CONFIGS["c3"], D=23_500_000, K=1000, alpha=0.05)
    doff, words = corpus.make_corpus(cfg)
    N = int(doff[-1])
    assert 2_100_000_000 < N <= 2**31 - 2**20 - 1
    g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=1, dense_rows=0,
                    dense_alias_min_count=cfg.K)
    assert g.N == N
    ll0 = g.loglik()[0]
    for _ in range(2):
        g.build_alias()
        g.sweep(2)
        g.rebuild_counts()
    nk = g.get_nk()
    z = g.get_z()
    assert 0 <= z.min() and z.max() < cfg.K
    assert np.array_equal(np.bincount(z, minlength=cfg.K), nk)
    for d in (0, 1, cfg.D // 2, cfg.D - 1):
        assert np.array_equal(g.get_ndk_row(d),
                              np.bincount(z[doff[d]:doff[d + 1]], minlength=cfg.K)), d
    for w in (0, 5, 1000, cfg.V - 1):  # a dense-table word, mixture words, the rarest word
        assert np.array_equal(g.get_nkw_row(w), np.bincount(z[words == w], minlength=cfg.K)), w
    assert g.loglik()[0] > ll0
    g.close()
