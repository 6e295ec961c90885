"""GPU parity of the hybrid word-topic store (Sec. 5) and the sparsified mixture
word-proposal (Sec. 4.2) against the oracle: bit-exact z, counts, dense tables,
mixture tables (sparse term per word + shared beta term), log-likelihood to 1e-9.
"""
import numpy as np
import pytest

from paper_1412_1576_amd import corpus
from test_gpu_parity import check_state, check_alias

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lda_mod():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1412_1576_amd import lda
    lda.load_library()
    return lda


def classes(words, V, dense_rows):
    """dense_alias_min_count that makes every word without a dense row a mixture word."""
    cnt = np.bincount(words, minlength=V)
    H = 0 if dense_rows < 0 else (V if dense_rows == 0 else min(dense_rows, V))
    tail_max = int(cnt[H:].max()) if H < V else 0
    min_count = tail_max + 1
    dense_alias = cnt >= min_count
    assert not dense_alias[H:].any()
    return cnt, H, min_count, dense_alias


def check_mixture_tables(g, o, mix_words, tag=""):
    bs, ba, bc, QB = g.get_beta_table()
    os_, oa, oc, oQB = o.get_beta_table()
    assert (bc, QB) == (oc, oQB), tag + " beta table header"
    assert np.array_equal(bs, os_) and np.array_equal(ba, oa), tag + " beta table"
    for w in mix_words:
        t, s, at, c, qs = g.get_sparse_table(w)
        ot, osp, oal, oc, oqs = o.get_sparse_table(w)
        assert len(t) == len(ot) and (len(t) == 0 or (c, qs) == (oc, oqs)), \
            "%s sparse table header of word %d" % (tag, w)
        assert np.array_equal(t, ot), "%s sparse table topics of word %d" % (tag, w)
        assert np.array_equal(s, osp), "%s sparse table split of word %d" % (tag, w)
        assert np.array_equal(at, ot[oal.astype(np.int64)]), \
            "%s sparse table alias of word %d" % (tag, w)


def run_hybrid(lda_mod, oracle_mod, doff, words, V, K, alpha, beta, seed, sweeps, mh_steps,
               dense_rows, docs=(), nkw_words=None, table_words=None, **opt):
    cnt, H, min_count, dense_alias = classes(words, V, dense_rows)
    g = lda_mod.Lda(doff, words, V, K, alpha, beta, seed=seed, dense_rows=dense_rows,
                    dense_alias_min_count=min_count, **opt)
    o = oracle_mod.Oracle(doff, words, V, K, alpha, beta, seed=seed,
                          dense_alias_min_count=min_count)
    ws = list(range(V)) if table_words is None else list(table_words)
    dense_ws = [w for w in ws if dense_alias[w]]
    mix_ws = [w for w in ws if not dense_alias[w]]
    check_state(g, o, docs, nkw_words, tag="init")
    for it in range(sweeps):
        g.build_alias()
        o.build_alias()
        check_alias(g, o, dense_ws, tag="sweep %d" % it)
        check_mixture_tables(g, o, mix_ws, tag="sweep %d" % it)
        g.sweep(mh_steps)
        o.sweep(mh_steps)
        g.rebuild_counts()
        o.rebuild_counts()
        check_state(g, o, docs, nkw_words, tag="sweep %d" % it)
    g.close()
    o.close()
    return cnt, H, dense_alias


def test_hybrid_small(lda_mod, oracle_mod):
    """Head words dense (some of them mixture words with a dense row), tail sparse."""
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=600)
    doff, words = corpus.make_corpus(cfg)
    cnt, H, dense_alias = run_hybrid(lda_mod, oracle_mod, doff, words, cfg.V, cfg.K, cfg.alpha,
                                     cfg.beta, 0, 4, 2, dense_rows=150, docs=range(0, 600, 41))
    assert dense_alias[:150].any() and not dense_alias[:150].all()  # both kinds among dense rows


def test_hybrid_record_buckets(lda_mod, oracle_mod):
    """The bucketed record order on the hybrid store (not its default there)."""
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=600)
    doff, words = corpus.make_corpus(cfg)
    run_hybrid(lda_mod, oracle_mod, doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, 0, 3, 2,
               dense_rows=150, docs=range(0, 600, 41), record_bucket_tokens=2048)


def test_all_sparse_all_mixture(lda_mod, oracle_mod):
    """No dense row at all (the shape of one K = 10^6 model slice); the hottest words go
    through the scratch-row rebuild (more than 16384 tokens), the others through the LDS sorts."""
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=6000, V=20000, K=300)
    doff, words = corpus.make_corpus(cfg)
    cnt = np.bincount(words, minlength=cfg.V)
    assert cnt.max() > 16384 and (cnt == 0).any()
    run_hybrid(lda_mod, oracle_mod, doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, 5, 3, 3,
               dense_rows=-1, docs=range(0, 6000, 397),
               nkw_words=list(range(0, 40)) + list(range(40, cfg.V, 137)),
               table_words=list(range(0, 30)) + list(range(30, cfg.V, 253)))


def test_ragged_hybrid(lda_mod, oracle_mod):
    """Empty / one-token / long documents with mixture words, odd K."""
    from test_gpu_parity import ragged_corpus
    V = 60
    doff, words = ragged_corpus(V, seed=8, long_len=700)
    D = len(doff) - 1
    for K, dr in ((7, 4), (65, -1), (1, 3)):
        run_hybrid(lda_mod, oracle_mod, doff, words, V, K, 0.1, 0.05, 9, 3, 3, dense_rows=dr,
                   docs=range(D), sweep_chunk_tokens=128, sweep_block_threads=64,
                   rebuild_tile_tokens=64)


@pytest.mark.timeout(600)
def test_large_K_hybrid(lda_mod, oracle_mod):
    """K = 100,000 (the big-K hybrid store's shape at a small vocabulary): dense rows
    rebuilt by atomics, dense and mixture tables too large for LDS, n_k by topic ranges."""
    K, V = 100_000, 400
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=3000, V=V, K=K, T=10)
    doff, words = corpus.make_corpus(cfg)
    cnt = np.bincount(words, minlength=V)
    assert (cnt[2:] > 12288).any()      # a mixture table beyond the LDS limit
    run_hybrid(lda_mod, oracle_mod, doff, words, V, K, 0.01, 0.01, 2, 2, 2, dense_rows=2,
               docs=range(0, 3000, 499), nkw_words=list(range(0, 12)) + [100, 399],
               table_words=list(range(0, 10)) + [50, 200, 399])


@pytest.mark.timeout(600)
def test_million_topics_slice(lda_mod, oracle_mod):
    """K = 1,000,000, all rows sparse, mixture only: the shared beta table has 10^6 bins."""
    K, V = 1_000_000, 120
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=1500, V=V, K=K, T=10)
    doff, words = corpus.make_corpus(cfg)
    run_hybrid(lda_mod, oracle_mod, doff, words, V, K, 0.01, 0.01, 4, 2, 2, dense_rows=-1,
               docs=range(0, 1500, 301), nkw_words=[0, 1, 2, 50, 119],
               table_words=[0, 1, 7, 60, 119])


def test_option_validation(lda_mod):
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=100)
    doff, words = corpus.make_corpus(cfg)
    # a frequent word outside the dense rows cannot draw from a dense table
    with pytest.raises(lda_mod.LdaError) as e:
        lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, dense_rows=10,
                    dense_alias_min_count=1)
    assert e.value.code == lda_mod.LDA_ERR_ARG
    # more dense row entries than the library allocates
    with pytest.raises(lda_mod.LdaError) as e:
        lda_mod.Lda(doff, words, 20000, 600000, cfg.alpha, cfg.beta)
    assert e.value.code == lda_mod.LDA_ERR_UNSUPPORTED
