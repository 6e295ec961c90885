"""MI355X-native LightLDA cycle Metropolis-Hastings sweep (arXiv 1412.1576).

`paper_1412_1576_amd.lda` is the thin ctypes binding over the C-ABI library
built from `csrc/` (hand-written HIP for gfx950); `paper_1412_1576_amd.corpus`
generates the seeded synthetic corpora.  Importing the package loads nothing
native; the binding fails loudly when the library has not been built.
"""
__all__ = ["corpus", "lda"]
