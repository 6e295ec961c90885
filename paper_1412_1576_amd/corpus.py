"""Seeded synthetic corpora with the shapes of the paper's workloads (Table 1).

This module is the only code shared by the CPU oracle's tests and the GPU
path's tests and benchmark.  It holds input generation only -- none of the
sampler's arithmetic -- and depends on numpy alone.

Recipe (all configs):
  * document lengths  L_d ~ Poisson(lam), clipped to >= 1;
  * word frequencies  Zipf: pi(r) ~ r^-s for rank r = 1..V, word id = r - 1
    (id order is frequency order);
  * T planted topics (T = 0: none): word w belongs to class w mod T,
    phi_t = pi restricted to class t and renormalised, theta_d ~ Dirichlet(0.1);
    every token is a background draw from pi with probability 1/2, otherwise
    t ~ theta_d and w ~ phi_t;
  * CSR output: int64 doc_offsets[D+1], int32 word_ids[N].
Documents are generated in fixed-size chunks, each from its own child of
numpy's SeedSequence(seed), so the result does not depend on the thread count.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class CorpusConfig:
    name: str
    D: int            # documents
    lam: float        # mean document length
    V: int            # vocabulary size
    s: float          # Zipf exponent
    T: int            # planted topics (0: pure Zipf)
    K: int            # LDA topics
    alpha: float
    beta: float
    mh_steps: int
    sweeps: int
    gen_seed: int     # corpus generator seed
    lib_seed: int = 0  # sampler seed
    dense_rows: int = 0
    dense_alias_min_count: int = 0


# The five workloads: a tiny case, NYTimes-, PubMed-shaped corpora (Table 1),
# a big-K hybrid-store case and one K = 10^6 model slice.
CONFIGS = {
    "c1": CorpusConfig("c1", D=1_000, lam=100, V=5_000, s=1.07, T=20, K=100, alpha=0.1,
                       beta=0.01, mh_steps=2, sweeps=10, gen_seed=1001),
    "c2": CorpusConfig("c2", D=300_000, lam=330, V=100_000, s=1.07, T=200, K=1_000,
                       alpha=50.0 / 1_000, beta=0.01, mh_steps=2, sweeps=20, gen_seed=1002),
    "c3": CorpusConfig("c3", D=8_200_000, lam=90, V=141_000, s=1.05, T=0, K=10_000, alpha=0.01,
                       beta=0.01, mh_steps=4, sweeps=5, gen_seed=1003),
    "c4": CorpusConfig("c4", D=10_000_000, lam=100, V=1_000_000, s=1.1, T=0, K=100_000,
                       alpha=0.01, beta=0.01, mh_steps=2, sweeps=1, gen_seed=1004,
                       dense_rows=20_000),
    "c5": CorpusConfig("c5", D=5_000_000, lam=100, V=50_000, s=1.1, T=0, K=1_000_000,
                       alpha=0.01, beta=0.01, mh_steps=2, sweeps=1, gen_seed=1005),
}


def scaled(cfg: CorpusConfig, **kw) -> CorpusConfig:
    """A copy of a config with some fields replaced (e.g. fewer documents)."""
    return replace(cfg, **kw)


def zipf_cdf(V: int, s: float) -> np.ndarray:
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    c /= c[-1]
    c[-1] = 1.0
    return c


_CHUNK_DOCS = 32_768


def _class_tables(V: int, s: float, T: int):
    """Flattened per-class inverse-CDF tables: entry [t*M + i] = t + cdf_t(i)."""
    M = (V + T - 1) // T
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    tab = np.zeros((T, M), np.float64)
    for t in range(T):
        pc = p[t::T]
        c = np.cumsum(pc)
        c /= c[-1]
        tab[t, : len(c)] = c
        tab[t, len(c) - 1:] = 1.0
    tab[:, -1] = 1.0
    tab += np.arange(T, dtype=np.float64)[:, None]
    return tab.ravel(), M


def _gen_chunk(args):
    ss, nd, lam, V, T, cdf, class_tab, M = args
    rng = np.random.default_rng(ss)
    lens = np.maximum(rng.poisson(lam, nd), 1).astype(np.int64)
    n = int(lens.sum())
    u = rng.random(n)
    if T <= 0:
        w = np.searchsorted(cdf, u, side="right")
        np.minimum(w, V - 1, out=w)
        return lens, w.astype(np.int32)
    background = rng.random(n) < 0.5
    w = np.empty(n, np.int64)
    wb = np.searchsorted(cdf, u[background], side="right")
    w[background] = np.minimum(wb, V - 1)
    # planted part: topic from the document's theta, then a word of that class
    doc_idx = np.repeat(np.arange(nd, dtype=np.int64), lens)[~background]
    theta = rng.dirichlet(np.full(T, 0.1), nd)
    cth = np.cumsum(theta, axis=1)
    cth /= cth[:, -1:]
    cth[:, -1] = 1.0
    cth += np.arange(nd, dtype=np.float64)[:, None]
    ut = rng.random(len(doc_idx))
    t = np.searchsorted(cth.ravel(), doc_idx + ut, side="right") - doc_idx * T
    np.clip(t, 0, T - 1, out=t)
    i = np.searchsorted(class_tab, t + u[~background], side="right") - t * M
    np.clip(i, 0, M - 1, out=i)
    wp = t + i * T
    # the last class rows can be one entry shorter than M
    over = wp >= V
    wp[over] -= T
    w[~background] = wp
    return lens, w.astype(np.int32)


def make_corpus(cfg: CorpusConfig, threads: int | None = None):
    """Return (doc_offsets int64[D+1], word_ids int32[N]) for a config."""
    nchunks = (cfg.D + _CHUNK_DOCS - 1) // _CHUNK_DOCS
    seeds = np.random.SeedSequence(cfg.gen_seed).spawn(nchunks)
    cdf = zipf_cdf(cfg.V, cfg.s)
    class_tab, M = _class_tables(cfg.V, cfg.s, cfg.T) if cfg.T > 0 else (None, 0)
    jobs = []
    for c in range(nchunks):
        nd = min(_CHUNK_DOCS, cfg.D - c * _CHUNK_DOCS)
        jobs.append((seeds[c], nd, cfg.lam, cfg.V, cfg.T, cdf, class_tab, M))
    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if threads > 1 and nchunks > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            parts = list(ex.map(_gen_chunk, jobs))
    else:
        parts = [_gen_chunk(j) for j in jobs]
    lens = np.concatenate([p[0] for p in parts])
    doc_offsets = np.zeros(cfg.D + 1, np.int64)
    np.cumsum(lens, out=doc_offsets[1:])
    word_ids = np.concatenate([p[1] for p in parts])
    assert len(word_ids) == doc_offsets[-1]
    return doc_offsets, word_ids
