"""Thin ctypes binding over the C ABI of liblda_mi355x.so (include/lda_mi355x.h).

Argument marshalling only: every step of the method runs in the library's HIP
kernels.  There is no CPU fallback -- loading fails loudly when the library has
not been built (`python -m paper_1412_1576_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblda_mi355x.so")

LDA_OK = 0
LDA_ERR_ARG = -1
LDA_ERR_STATE = -2
LDA_ERR_OOM = -3
LDA_ERR_HIP = -4
LDA_ERR_UNSUPPORTED = -5

EXPORTS = [
    "lda_init", "lda_build_alias", "lda_sweep", "lda_sweep_pass_ms", "lda_rebuild_counts",
    "lda_update_counts", "lda_loglik", "lda_loglik_noalloc",
    "lda_num_tokens", "lda_sweep_index", "lda_get_z", "lda_set_z", "lda_get_nk",
    "lda_get_nkw_row", "lda_get_ndk_row", "lda_get_alias_row", "lda_get_sparse_table",
    "lda_get_beta_table", "lda_sync", "lda_last_error", "lda_destroy",
]


DEV_ALLOC = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
DEV_FREE = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class lda_options(C.Structure):
    _fields_ = [
        ("hip_stream", C.c_void_p),
        ("dev_alloc", DEV_ALLOC),
        ("dev_free", DEV_FREE),
        ("alloc_user", C.c_void_p),
        ("dense_rows", C.c_int32),
        ("dense_alias_min_count", C.c_int32),
        ("proposal_mode", C.c_int32),
        ("sweep_chunk_tokens", C.c_int32),
        ("sweep_block_threads", C.c_int32),
        ("rebuild_tile_tokens", C.c_int32),
        ("time_sweep_passes", C.c_int32),
        ("record_bucket_tokens", C.c_int32),
        ("doc_refresh", C.c_int32),
        ("stream_block_tokens", C.c_int32),
        ("reserved", C.c_int32 * 5),
    ]


class LdaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("lda error %d: %s" % (code, msg))
        self.code = code


_lib = None
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")


def load_library():
    """Load liblda_mi355x.so; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s not found: build it with `python -m paper_1412_1576_amd.build`; "
            "there is no CPU fallback" % LIB_PATH)
    # PyTorch supplies device memory and streams to callers and ships its own HIP
    # runtime; import it first so that this library binds to the runtime the
    # process already uses (two HIP/HSA runtimes in one process cannot share the GPU).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    dp = C.POINTER(C.c_double)
    sig = {
        "lda_init": (C.c_int, [C.POINTER(vp), C.c_int64, C.c_int32, C.c_int32, _i64p, _i32p,
                               C.c_double, C.c_double, C.c_uint64, C.POINTER(lda_options)]),
        "lda_build_alias": (C.c_int, [vp]),
        "lda_sweep": (C.c_int, [vp, C.c_int32]),
        "lda_sweep_pass_ms": (C.c_int, [vp, C.POINTER(C.c_float), C.POINTER(C.c_float)]),
        "lda_rebuild_counts": (C.c_int, [vp]),
        "lda_update_counts": (C.c_int, [vp]),
        "lda_loglik": (C.c_int, [vp, dp, dp, dp]),
        "lda_loglik_noalloc": (C.c_int, [vp, dp, dp, dp]),
        "lda_num_tokens": (C.c_int64, [vp]),
        "lda_sweep_index": (C.c_int64, [vp]),
        "lda_get_z": (C.c_int, [vp, _i32p]),
        "lda_set_z": (C.c_int, [vp, _i32p, C.c_int64]),
        "lda_get_nk": (C.c_int, [vp, _i32p]),
        "lda_get_nkw_row": (C.c_int, [vp, C.c_int32, _i32p]),
        "lda_get_ndk_row": (C.c_int, [vp, C.c_int64, _i32p]),
        "lda_get_alias_row": (C.c_int, [vp, C.c_int32, _u32p, _u32p, C.POINTER(C.c_uint32)]),
        "lda_get_sparse_table": (C.c_int, [vp, C.c_int32, C.c_int32, C.POINTER(C.c_int32), _i32p,
                                           _u32p, _i32p, C.POINTER(C.c_uint32),
                                           C.POINTER(C.c_uint64)]),
        "lda_get_beta_table": (C.c_int, [vp, _u32p, _u32p, C.POINTER(C.c_uint32),
                                         C.POINTER(C.c_uint64)]),
        "lda_sync": (C.c_int, [vp]),
        "lda_last_error": (C.c_char_p, [vp]),
        "lda_destroy": (None, [vp]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype = res
        f.argtypes = args
    _lib = L
    return L


class Lda:
    """One corpus on one GPU.  Methods mirror the C entry points one to one."""

    def __init__(self, doc_offsets, word_ids, V, K, alpha, beta, seed=0, stream=None,
                 dense_rows=0, dense_alias_min_count=0, proposal_mode=0, sweep_chunk_tokens=0,
                 sweep_block_threads=0, rebuild_tile_tokens=0, time_sweep_passes=0,
                 record_bucket_tokens=0, doc_refresh=0, stream_block_tokens=0, dev_alloc=None,
                 dev_free=None):
        """dev_alloc(bytes) -> device address (0: failure) and dev_free(address): the
        caller's device allocator for every buffer of the context (both or neither)."""
        L = load_library()
        self._h = C.c_void_p()
        doc_offsets = np.ascontiguousarray(doc_offsets, np.int64)
        word_ids = np.ascontiguousarray(word_ids, np.int32)
        opt = lda_options()
        opt.hip_stream = C.c_void_p(int(stream)) if stream else None
        opt.dense_rows = dense_rows
        opt.dense_alias_min_count = dense_alias_min_count
        opt.proposal_mode = proposal_mode
        opt.sweep_chunk_tokens = sweep_chunk_tokens
        opt.sweep_block_threads = sweep_block_threads
        opt.rebuild_tile_tokens = rebuild_tile_tokens
        opt.time_sweep_passes = time_sweep_passes
        opt.record_bucket_tokens = record_bucket_tokens
        opt.doc_refresh = doc_refresh
        opt.stream_block_tokens = stream_block_tokens
        # the ctypes thunks must outlive the context: the library calls them until lda_destroy
        self._alloc_cb = self._free_cb = None
        if dev_alloc is not None:
            self._alloc_cb = DEV_ALLOC(lambda nbytes, user: int(dev_alloc(int(nbytes))) or None)
            opt.dev_alloc = self._alloc_cb
        if dev_free is not None:
            self._free_cb = DEV_FREE(lambda ptr, user: dev_free(int(ptr or 0)))
            opt.dev_free = self._free_cb
        self.D = len(doc_offsets) - 1
        self.V, self.K = int(V), int(K)
        rc = L.lda_init(C.byref(self._h), self.D, self.V, self.K, doc_offsets, word_ids,
                        float(alpha), float(beta), int(seed), C.byref(opt))
        if rc != LDA_OK:
            raise LdaError(rc, (L.lda_last_error(None) or b"").decode())
        self.N = int(L.lda_num_tokens(self._h))

    def _ck(self, rc):
        if rc != LDA_OK:
            raise LdaError(rc, (load_library().lda_last_error(self._h) or b"").decode())

    def close(self):
        if self._h:
            load_library().lda_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def build_alias(self):
        self._ck(_lib.lda_build_alias(self._h))

    def sweep(self, mh_steps):
        self._ck(_lib.lda_sweep(self._h, int(mh_steps)))

    def sweep_pass_ms(self):
        w, d = C.c_float(), C.c_float()
        self._ck(_lib.lda_sweep_pass_ms(self._h, C.byref(w), C.byref(d)))
        return w.value, d.value

    def rebuild_counts(self):
        self._ck(_lib.lda_rebuild_counts(self._h))

    def update_counts(self):
        self._ck(_lib.lda_update_counts(self._h))

    def loglik(self):
        t, d, w = C.c_double(), C.c_double(), C.c_double()
        self._ck(_lib.lda_loglik(self._h, C.byref(t), C.byref(d), C.byref(w)))
        return t.value, d.value, w.value

    def loglik_noalloc(self):
        t, d, w = C.c_double(), C.c_double(), C.c_double()
        self._ck(_lib.lda_loglik_noalloc(self._h, C.byref(t), C.byref(d), C.byref(w)))
        return t.value, d.value, w.value

    def sync(self):
        self._ck(_lib.lda_sync(self._h))

    @property
    def sweep_index(self):
        return int(_lib.lda_sweep_index(self._h))

    def get_z(self):
        z = np.empty(self.N, np.int32)
        self._ck(_lib.lda_get_z(self._h, z))
        return z

    def set_z(self, z, next_sweep_index):
        z = np.ascontiguousarray(z, np.int32)
        if len(z) != self.N:
            raise ValueError("z must have N entries")
        self._ck(_lib.lda_set_z(self._h, z, int(next_sweep_index)))

    def get_nk(self):
        nk = np.empty(self.K, np.int32)
        self._ck(_lib.lda_get_nk(self._h, nk))
        return nk

    def get_nkw_row(self, w):
        row = np.empty(self.K, np.int32)
        self._ck(_lib.lda_get_nkw_row(self._h, int(w), row))
        return row

    def get_ndk_row(self, d):
        row = np.empty(self.K, np.int32)
        self._ck(_lib.lda_get_ndk_row(self._h, int(d), row))
        return row

    def get_alias_row(self, w):
        split = np.empty(self.K, np.uint32)
        alias = np.empty(self.K, np.uint32)
        cap = C.c_uint32()
        self._ck(_lib.lda_get_alias_row(self._h, int(w), split, alias, C.byref(cap)))
        return split, alias, cap.value

    def get_sparse_table(self, w):
        """(topics, split, alias_topic, capacity, mass) of a mixture-form word."""
        n = C.c_int32()
        cap = C.c_uint32()
        mass = C.c_uint64()
        d = np.empty(1, np.int32)
        u = np.empty(1, np.uint32)
        self._ck(_lib.lda_get_sparse_table(self._h, int(w), 0, C.byref(n), d, u, d.copy(),
                                           C.byref(cap), C.byref(mass)))
        k = max(n.value, 1)
        topics = np.empty(k, np.int32)
        split = np.empty(k, np.uint32)
        alias_topic = np.empty(k, np.int32)
        self._ck(_lib.lda_get_sparse_table(self._h, int(w), k, C.byref(n), topics, split,
                                           alias_topic, C.byref(cap), C.byref(mass)))
        k = n.value
        return topics[:k], split[:k], alias_topic[:k], cap.value, mass.value

    def get_beta_table(self):
        split = np.empty(self.K, np.uint32)
        alias = np.empty(self.K, np.uint32)
        cap = C.c_uint32()
        mass = C.c_uint64()
        self._ck(_lib.lda_get_beta_table(self._h, split, alias, C.byref(cap), C.byref(mass)))
        return split, alias, cap.value, mass.value
