"""lda_options.stream_block_tokens: streamed data blocks (Sec. 3; Sec. 6, Fig. 7) give the
resident run's results bit for bit -- and with them the oracle's."""
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


def compare(lda_mod, oracle_mod, cfg, doff, words, block_tokens, steps, **opt):
    s = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=6,
                    stream_block_tokens=block_tokens, **opt)
    r = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=6, **opt)
    o = oracle_mod.Oracle(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=6,
                          dense_alias_min_count=opt.get("dense_alias_min_count", 0))
    rng = np.random.default_rng(1)
    some_words = rng.choice(cfg.V, 25, replace=False)
    some_docs = rng.choice(len(doff) - 1, 10, replace=False)
    assert np.array_equal(s.get_z(), o.get_z())
    for it, m in enumerate(steps):
        if it == 2:   # another assignment through lda_set_z
            z = rng.integers(0, cfg.K, s.N).astype(np.int32)
            for x in (s, r, o):
                x.set_z(z, 40)
                x.rebuild_counts()
        assert s.loglik() == r.loglik()
        for x in (s, r, o):
            x.build_alias()
            x.sweep(m)
            x.rebuild_counts()
        zs = s.get_z()
        assert np.array_equal(zs, o.get_z()), (it, m)
        assert np.array_equal(zs, r.get_z()), (it, m)
        assert np.array_equal(s.get_nk(), o.get_nk()), (it, m)
        for w in some_words:
            assert np.array_equal(s.get_nkw_row(w), o.get_nkw_row(w)), (it, w)
        for d in some_docs:
            assert np.array_equal(s.get_ndk_row(d), o.get_ndk_row(d)), (it, d)
    ls, lo = s.loglik(), o.loglik()
    assert abs(ls[0] - lo[0]) <= 1e-9 * abs(lo[0])
    assert s.loglik() == r.loglik()
    for x in (s, r, o):
        x.close()


def test_dense_store_in_blocks(lda_mod, oracle_mod):
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=700)
    doff, words = corpus.make_corpus(cfg)
    for block in (9000, 25000, 10**9):     # 8 blocks with a short last one, 3 blocks, one block
        compare(lda_mod, oracle_mod, cfg, doff, words, block, [2, 4, 1, 3])


def test_hybrid_store_in_blocks(lda_mod, oracle_mod):
    """Dense rows for the head, sparse rows (lists and hash rows) for the tail, the mixture
    proposal; and no dense row at all with K above the n_k histogram's range."""
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=500, K=300)
    doff, words = corpus.make_corpus(cfg)
    cnt = np.bincount(words, minlength=cfg.V)
    compare(lda_mod, oracle_mod, cfg, doff, words, 7000, [2, 2, 3],
            dense_rows=100, dense_alias_min_count=int(cnt[100:].max()) + 1)
    compare(lda_mod, oracle_mod, cfg, doff, words, 12000, [2, 1, 2],
            dense_rows=-1, dense_alias_min_count=int(cnt.max()) + 1)
    big = corpus.scaled(corpus.CONFIGS["c1"], D=150, V=200, K=300_000)
    doff, words = corpus.make_corpus(big)
    cnt = np.bincount(words, minlength=big.V)
    compare(lda_mod, oracle_mod, big, doff, words, 4000, [2, 2],
            dense_rows=-1, dense_alias_min_count=int(cnt.max()) + 1)


def test_what_streaming_refuses(lda_mod):
    cfg = corpus.scaled(corpus.CONFIGS["c1"], D=60)
    doff, words = corpus.make_corpus(cfg)
    with pytest.raises(lda_mod.LdaError) as e:
        lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, stream_block_tokens=1000, doc_refresh=1)
    assert e.value.code == lda_mod.LDA_ERR_ARG
    long_doff = np.array([0, 3000, 3010], np.int64)   # a document longer than a sweep tile
    with pytest.raises(lda_mod.LdaError) as e:
        lda_mod.Lda(long_doff, np.zeros(3010, np.int32), 4, 8, 0.1, 0.1, stream_block_tokens=1000)
    assert e.value.code == lda_mod.LDA_ERR_UNSUPPORTED
    g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, stream_block_tokens=1000)
    g.build_alias(); g.sweep(2)
    with pytest.raises(lda_mod.LdaError) as e:
        g.update_counts()
    assert e.value.code == lda_mod.LDA_ERR_UNSUPPORTED
    g.rebuild_counts()
    g.close()
