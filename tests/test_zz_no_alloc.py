"""lda_loglik_noalloc (the entry point for callers that cannot allocate) against lda_loglik.

Called through the C ABI on two contexts in a row, the second smaller than the first, so
that the static scratch array still holds the first call's partial sums when the second
runs; then on the hybrid store, and on a corpus with more document tiles than the array
holds, which must be refused.  The contexts take their device memory from a counting
allocator, which shows that the call allocates nothing through the library's allocator.
"""
import ctypes as C

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


class CountingAllocator:
    """Device memory from torch's caching allocator, every request counted."""

    def __init__(self):
        import torch
        self.torch = torch
        self.live = {}
        self.calls = 0

    def alloc(self, nbytes):
        self.calls += 1
        t = self.torch.empty(max(nbytes, 1), dtype=self.torch.uint8, device="cuda")
        self.live[t.data_ptr()] = t
        return t.data_ptr()

    def free(self, ptr):
        self.calls += 1
        self.live.pop(ptr, None)


def both(lda_mod, g):
    """(lda_loglik, lda_loglik_noalloc) through the C ABI."""
    lib = lda_mod.load_library()
    out = []
    for f in (lib.lda_loglik, lib.lda_loglik_noalloc):
        t, d, w = C.c_double(), C.c_double(), C.c_double()
        rc = f(g._h, C.byref(t), C.byref(d), C.byref(w))
        assert rc == lda_mod.LDA_OK, (lib.lda_last_error(g._h) or b"").decode()
        out.append((t.value, d.value, w.value))
    return out


def check(lda_mod, cfg, **opt):
    doff, words = corpus.make_corpus(cfg)
    a = CountingAllocator()
    g = lda_mod.Lda(doff, words, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed=4, dev_alloc=a.alloc,
                    dev_free=a.free, **opt)
    for it in range(2):
        g.loglik()                       # the context's own buffers exist before the count
        before = a.calls
        ref, got = both(lda_mod, g)
        assert a.calls == before
        for x, y in zip(got, ref):       # same kernels, same order of summation
            assert abs(x - y) <= 1e-9 * max(abs(y), abs(ref[0])), (got, ref)
            assert x == y, (got, ref)
        before = a.calls
        lib = lda_mod.load_library()
        t = C.c_double()
        assert lib.lda_loglik_noalloc(g._h, C.byref(t), None, None) == lda_mod.LDA_OK
        assert a.calls == before and t.value == ref[0]
        g.build_alias()
        g.sweep(2)
        g.rebuild_counts()
    g.close()


def test_noalloc_matches_loglik_two_calls_in_a_row(lda_mod):
    big = corpus.scaled(corpus.CONFIGS["c1"], D=6000)        # about 6 * 10^5 tokens, 600 tiles
    small = corpus.scaled(corpus.CONFIGS["c1"], D=150, V=700, K=33)
    check(lda_mod, big)
    check(lda_mod, small)                                    # the array keeps the first call's sums
    check(lda_mod, corpus.scaled(small, D=40), dense_rows=50, dense_alias_min_count=40)  # sparse rows
    check(lda_mod, corpus.scaled(big, D=900), sweep_chunk_tokens=64)   # many small tiles


def test_noalloc_refuses_more_tiles_than_the_array_holds(lda_mod):
    # 1.1 * 10^6 documents of 64 tokens on tiles of 64 tokens: one tile per document
    D = 1_100_000
    doff = np.arange(D + 1, dtype=np.int64) * 64
    words = np.tile(np.arange(64, dtype=np.int32), D)
    g = lda_mod.Lda(doff, words, 64, 8, 0.1, 0.01, seed=1, sweep_chunk_tokens=64)
    lib = lda_mod.load_library()
    t = C.c_double()
    assert lib.lda_loglik_noalloc(g._h, C.byref(t), None, None) == lda_mod.LDA_ERR_UNSUPPORTED
    assert b"static scratch" in lib.lda_last_error(g._h)
    ref = g.loglik()[0]                                      # the allocating entry point still works
    assert np.isfinite(ref) and ref < 0
    # state checks come first
    g.build_alias(); g.sweep(1)
    assert lib.lda_loglik_noalloc(g._h, C.byref(t), None, None) == lda_mod.LDA_ERR_STATE
    g.close()
