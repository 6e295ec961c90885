"""GPU parity on seeded random configurations: corpus shape, K, store (all dense rows, head
dense / tail sparse, all sparse), proposal form (dense tables, mixture below a random corpus
frequency), number of MH steps changing from sweep to sweep, proposal mode, launch geometry
and the order of the records the two passes exchange are all drawn from the case's seed.
Every case compares z, n_k, sampled n_kw and n_kd rows and the log-likelihood with the
oracle after every sweep (bit-exact / 1e-9).
"""
import numpy as np
import pytest

from test_gpu_parity import check_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lda_mod():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1412_1576_amd import lda
    lda.load_library()
    return lda


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([1, 3, 40, 200, 900]))
    K = int(rng.choice([1, 2, 5, 33, 100, 257, 1000, 4096, 20000, 70000]))
    while V * K > 12_000_000:  # the oracle's dense V x K tables
        V = max(1, V // 2)
    D = int(rng.integers(1, 400))
    shape = rng.choice(["short", "mixed", "long"])
    if shape == "short":
        lens = rng.integers(0, 12, D)
    elif shape == "mixed":
        lens = rng.poisson(rng.choice([20, 90, 330]), D)
        lens[rng.integers(0, D, max(1, D // 10))] = 0
    else:
        lens = rng.poisson(60, D)
        for L in (1023, 1024, 1025, 1536, 1537, 2100):
            lens[rng.integers(0, D)] = L
    if lens.sum() == 0:
        lens[0] = 3
    doff = np.zeros(D + 1, np.int64)
    doff[1:] = np.cumsum(lens)
    s = float(rng.choice([0.0, 0.8, 1.1, 1.6]))
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    words = rng.choice(V, int(doff[-1]), p=p / p.sum()).astype(np.int32)
    cnt = np.bincount(words, minlength=V)
    store = rng.choice(["dense", "hybrid", "sparse"])
    opt = {}
    if store == "dense":
        H = V
        opt["dense_rows"] = 0
    elif store == "hybrid":
        H = int(rng.integers(1, V + 1))
        opt["dense_rows"] = H
    else:
        H = 0
        opt["dense_rows"] = -1
    # words without a dense row must be mixture words; above that any threshold is legal
    tail_max = int(cnt[H:].max()) if H < V else 0
    lowest = tail_max + 1
    form = rng.choice(["all dense tables", "threshold", "all mixture"])
    if form == "all dense tables" and H == V:
        min_count = 0
    elif form == "all mixture":
        min_count = int(cnt.max()) + 1
    else:
        min_count = int(rng.integers(lowest, max(lowest, int(cnt.max())) + 2))
    opt["dense_alias_min_count"] = min_count
    mode = int(rng.choice([0, 0, 0, 1, 2]))
    if mode:
        opt["proposal_mode"] = mode
    if rng.random() < 0.4:
        opt["sweep_chunk_tokens"] = int(rng.choice([64, 128, 512, 1024, 2016]))
        opt["sweep_block_threads"] = int(rng.choice([64, 256, 512, 1024]))
    if rng.random() < 0.4:
        opt["rebuild_tile_tokens"] = int(rng.choice([64, 1000, 65536]))
    if rng.random() < 0.5:
        opt["record_bucket_tokens"] = int(rng.choice([-1, 64, 512, 8192]))
    steps = [int(x) for x in rng.integers(1, 6, 3)]
    alpha = float(rng.choice([0.01, 0.1, 1.0]))
    beta = float(rng.choice([0.01, 0.1]))
    return doff, words, V, K, alpha, beta, steps, mode, opt


@pytest.mark.parametrize("seed", range(36))
def test_random_configuration(lda_mod, oracle_mod, seed):
    doff, words, V, K, alpha, beta, steps, mode, opt = random_case(seed)
    D = len(doff) - 1
    lib_seed = 7 * seed + 1
    g = lda_mod.Lda(doff, words, V, K, alpha, beta, seed=lib_seed, **opt)
    o = oracle_mod.Oracle(doff, words, V, K, alpha, beta, seed=lib_seed, proposal_mode=mode,
                          dense_alias_min_count=opt["dense_alias_min_count"])
    rng = np.random.default_rng(seed)
    docs = sorted(set(int(d) for d in rng.integers(0, D, 6)) | {0, D - 1})
    ws = sorted(set(int(w) for w in rng.integers(0, V, 12)) | {0, V - 1})
    tag = "case %d (V=%d K=%d N=%d %s)" % (seed, V, K, len(words), opt)
    check_state(g, o, docs, ws, tag=tag + " init")
    for it, m in enumerate(steps):
        g.build_alias()
        o.build_alias()
        g.sweep(m)
        o.sweep(m)
        g.rebuild_counts()
        o.rebuild_counts()
        check_state(g, o, docs, ws, tag="%s sweep %d (%d steps)" % (tag, it, m))
    g.close()
    o.close()
