"""The synthetic corpus generator: shapes, determinism, Zipf head."""
import numpy as np

from paper_1412_1576_amd import corpus


def test_c1_shape_and_determinism():
    cfg = corpus.CONFIGS["c1"]
    doff, w = corpus.make_corpus(cfg)
    doff2, w2 = corpus.make_corpus(cfg, threads=1)
    assert doff.tolist() == doff2.tolist() and w.tolist() == w2.tolist()
    assert doff.dtype == np.int64 and w.dtype == np.int32
    assert len(doff) == cfg.D + 1 and doff[0] == 0 and len(w) == doff[-1]
    L = np.diff(doff)
    assert L.min() >= 1 and abs(L.mean() - cfg.lam) < 2.0
    assert w.min() >= 0 and w.max() < cfg.V
    c = np.bincount(w, minlength=cfg.V)
    assert c[0] == c.max() and c[:10].sum() > 5 * c[100:110].sum()


def test_multi_chunk_thread_independence():
    cfg = corpus.scaled(corpus.CONFIGS["c3"], D=70_000, lam=8, V=3000)
    a = corpus.make_corpus(cfg, threads=1)
    b = corpus.make_corpus(cfg, threads=4)
    assert a[0].tolist() == b[0].tolist() and np.array_equal(a[1], b[1])


def test_planted_topics_concentrate_documents():
    cfg = corpus.scaled(corpus.CONFIGS["c2"], D=300, V=4000)
    doff, w = corpus.make_corpus(cfg)
    cls = w % cfg.T
    # a document's tokens crowd into few classes compared with the corpus
    ent = []
    for d in range(50):
        p = np.bincount(cls[doff[d]:doff[d + 1]], minlength=cfg.T) / (doff[d + 1] - doff[d])
        ent.append(-(p[p > 0] * np.log(p[p > 0])).sum())
    pc = np.bincount(cls, minlength=cfg.T) / len(cls)
    assert np.mean(ent) < -(pc[pc > 0] * np.log(pc[pc > 0])).sum() - 0.5
