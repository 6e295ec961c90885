"""CPU oracle for the LightLDA cycle Metropolis-Hastings sweep (arXiv 1412.1576).

TEST INFRASTRUCTURE ONLY: a ctypes wrapper around ``ldaref.c``.  Nothing in the
product package imports this module; only the tests, the smoke check and the
benchmark's cpu_baseline leg do.  It shares no code with the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ldaref.c")
_LIB = os.path.join(_HERE, "libldaref.so")

# -ffp-contract=off: the accept test and the alias quotients are defined with
# separately rounded fp64 operations (no fused multiply-add).
CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build_oracle(force: bool = False) -> str:
    """Compile ldaref.c with gcc into libldaref.so (next to the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None

_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_u64p = np.ctypeslib.ndpointer(np.uint64, flags="C_CONTIGUOUS")


def bind(path):
    """Load an oracle shared library and declare its signatures."""
    L = C.CDLL(path)
    vp = C.c_void_p
    sig = {
        "ldaref_philox4x32_10": (None, [_u32p, _u32p, _u32p]),
        "ldaref_alias_masses": (C.c_int, [C.c_int32, _u64p, _u64p, C.POINTER(C.c_uint32)]),
        "ldaref_alias_from_q0": (C.c_int, [C.c_int32, _u64p, _u32p, _u32p, C.POINTER(C.c_uint32)]),
        "ldaref_alias_build_dense_row": (C.c_int, [C.c_int32, _i32p, _i32p, C.c_double, C.c_double,
                                                   _u32p, _u32p, C.POINTER(C.c_uint32)]),
        "ldaref_alias_draw": (C.c_uint32, [C.c_int32, _u32p, _u32p, C.c_uint32, C.c_uint32, C.c_uint32]),
        "ldaref_doc_draw": (C.c_int32, [C.c_int32, C.c_int32, C.c_double, _i32p, C.c_uint32, C.c_uint32]),
        "ldaref_mh_accept": (C.c_int, [C.c_int] + [C.c_int32] * 9 + [C.c_double] * 3 + [C.c_uint32]),
        "ldaref_init": (C.c_int, [C.POINTER(vp), C.c_int64, C.c_int32, C.c_int32, _i64p, _i32p,
                                  C.c_double, C.c_double, C.c_uint64, C.c_int32, C.c_int32]),
        "ldaref_init_ex": (C.c_int, [C.POINTER(vp), C.c_int64, C.c_int32, C.c_int32, _i64p, _i32p,
                                     C.c_double, C.c_double, C.c_uint64, C.c_int32, C.c_int32,
                                     C.c_int32]),
        "ldaref_destroy": (None, [vp]),
        "ldaref_set_lazy_alias": (None, [vp, C.c_int32]),
        "ldaref_build_alias": (C.c_int, [vp]),
        "ldaref_sweep": (C.c_int, [vp, C.c_int32]),
        "ldaref_sweep_tokens": (C.c_int, [vp, C.c_uint32, C.c_int32, C.c_int64, _i64p, _i32p]),
        "ldaref_sweep_doc_refresh": (C.c_int, [vp, C.c_int32]),
        "ldaref_chain_with_doc": (C.c_int, [vp, C.c_int64, C.c_uint32, C.c_int32, C.c_int32, _i32p,
                                            C.POINTER(C.c_int32)]),
        "ldaref_rebuild_counts": (C.c_int, [vp]),
        "ldaref_update_counts": (C.c_int, [vp]),
        "ldaref_loglik": (C.c_int, [vp] + [C.POINTER(C.c_double)] * 3),
        "ldaref_num_tokens": (C.c_int64, [vp]),
        "ldaref_sweep_index": (C.c_uint32, [vp]),
        "ldaref_get_z": (C.c_int, [vp, _i32p]),
        "ldaref_set_z": (C.c_int, [vp, _i32p, C.c_int64]),
        "ldaref_get_nk": (C.c_int, [vp, _i32p]),
        "ldaref_get_nkw_row": (C.c_int, [vp, C.c_int32, _i32p]),
        "ldaref_get_ndk_row": (C.c_int, [vp, C.c_int64, _i32p]),
        "ldaref_get_alias_row": (C.c_int, [vp, C.c_int32, _u32p, _u32p, C.POINTER(C.c_uint32)]),
        "ldaref_get_sparse_table": (C.c_int, [vp, C.c_int32, C.c_int32, C.POINTER(C.c_int32), _i32p,
                                              _u32p, _u32p, C.POINTER(C.c_uint32),
                                              C.POINTER(C.c_uint64)]),
        "ldaref_get_beta_table": (C.c_int, [vp, _u32p, _u32p, C.POINTER(C.c_uint32),
                                            C.POINTER(C.c_uint64)]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype = res
        f.argtypes = args
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = bind(build_oracle())
    return _lib


class OracleError(RuntimeError):
    pass


def _ck(rc, what):
    if rc != 0:
        raise OracleError("%s failed with code %d" % (what, rc))


def philox4x32_10(ctr, key):
    out = np.zeros(4, np.uint32)
    lib().ldaref_philox4x32_10(np.asarray(ctr, np.uint32), np.asarray(key, np.uint32), out)
    return out


def alias_masses(q0):
    q0 = np.ascontiguousarray(q0, np.uint64)
    m = np.zeros_like(q0)
    cap = C.c_uint32()
    _ck(lib().ldaref_alias_masses(len(q0), q0, m, C.byref(cap)), "alias_masses")
    return m, cap.value


def alias_from_q0(q0):
    q0 = np.ascontiguousarray(q0, np.uint64)
    split = np.zeros(len(q0), np.uint32)
    alias = np.zeros(len(q0), np.uint32)
    cap = C.c_uint32()
    _ck(lib().ldaref_alias_from_q0(len(q0), q0, split, alias, C.byref(cap)), "alias_from_q0")
    return split, alias, cap.value


def alias_build_dense_row(nkw_row, nk, beta, betabar):
    nkw_row = np.ascontiguousarray(nkw_row, np.int32)
    nk = np.ascontiguousarray(nk, np.int32)
    K = len(nk)
    split = np.zeros(K, np.uint32)
    alias = np.zeros(K, np.uint32)
    cap = C.c_uint32()
    _ck(lib().ldaref_alias_build_dense_row(K, nkw_row, nk, beta, betabar, split, alias,
                                           C.byref(cap)), "alias_build_dense_row")
    return split, alias, cap.value


def alias_draw(split, alias, cap, x0, x1):
    return int(lib().ldaref_alias_draw(len(split), split, alias, cap, int(x0), int(x1)))


def doc_draw(L, K, alphabar, z_doc, x0, x1):
    z_doc = np.ascontiguousarray(z_doc, np.int32)
    return int(lib().ldaref_doc_draw(L, K, alphabar, z_doc, int(x0), int(x1)))


def mh_accept(word_step, s, t, z0, ndk_s, ndk_t, nkw_s, nkw_t, nk_s, nk_t, alpha, beta, betabar, x2):
    return int(lib().ldaref_mh_accept(int(bool(word_step)), s, t, z0, ndk_s, ndk_t, nkw_s, nkw_t,
                                      nk_s, nk_t, alpha, beta, betabar, int(x2)))


class Oracle:
    """Host-memory LDA state with the same call sequence as the GPU library."""

    def __init__(self, doc_offsets, word_ids, V, K, alpha, beta, seed=0,
                 dense_alias_min_count=0, proposal_mode=0, lazy_alias=False, lazy_rows=False):
        """lazy_alias: a word's table is built when a draw first needs it.  lazy_rows: a
        word's n_kw row (and dense table) is allocated and counted when first needed, for
        vocabularies whose V x K table does not fit in memory.  Neither changes a result."""
        self._h = C.c_void_p()
        doc_offsets = np.ascontiguousarray(doc_offsets, np.int64)
        word_ids = np.ascontiguousarray(word_ids, np.int32)
        self.D = len(doc_offsets) - 1
        self.V, self.K = int(V), int(K)
        _ck(lib().ldaref_init_ex(C.byref(self._h), self.D, self.V, self.K, doc_offsets, word_ids,
                                 float(alpha), float(beta), int(seed), int(dense_alias_min_count),
                                 int(proposal_mode), 1 if lazy_rows else 0), "ldaref_init")
        self.N = int(lib().ldaref_num_tokens(self._h))
        if lazy_alias:
            lib().ldaref_set_lazy_alias(self._h, 1)

    def close(self):
        if self._h:
            lib().ldaref_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def build_alias(self):
        _ck(lib().ldaref_build_alias(self._h), "ldaref_build_alias")

    def sweep(self, mh_steps):
        _ck(lib().ldaref_sweep(self._h, mh_steps), "ldaref_sweep")

    def sweep_tokens(self, sweep_index, mh_steps, token_ids):
        token_ids = np.ascontiguousarray(token_ids, np.int64)
        out = np.zeros(len(token_ids), np.int32)
        _ck(lib().ldaref_sweep_tokens(self._h, int(sweep_index), mh_steps, len(token_ids),
                                      token_ids, out), "ldaref_sweep_tokens")
        return out

    def sweep_doc_refresh(self, mh_steps):
        _ck(lib().ldaref_sweep_doc_refresh(self._h, mh_steps), "ldaref_sweep_doc_refresh")

    def chain_with_doc(self, g, sweep_index, mh_steps, zdoc):
        zdoc = np.ascontiguousarray(zdoc, np.int32)
        out = C.c_int32()
        _ck(lib().ldaref_chain_with_doc(self._h, int(g), int(sweep_index), mh_steps, len(zdoc), zdoc,
                                        C.byref(out)), "ldaref_chain_with_doc")
        return out.value

    def rebuild_counts(self):
        _ck(lib().ldaref_rebuild_counts(self._h), "ldaref_rebuild_counts")

    def update_counts(self):
        _ck(lib().ldaref_update_counts(self._h), "ldaref_update_counts")

    def loglik(self):
        t, d, w = C.c_double(), C.c_double(), C.c_double()
        _ck(lib().ldaref_loglik(self._h, C.byref(t), C.byref(d), C.byref(w)), "ldaref_loglik")
        return t.value, d.value, w.value

    @property
    def sweep_index(self):
        return int(lib().ldaref_sweep_index(self._h))

    def get_z(self):
        z = np.zeros(self.N, np.int32)
        _ck(lib().ldaref_get_z(self._h, z), "ldaref_get_z")
        return z

    def set_z(self, z, next_sweep_index):
        _ck(lib().ldaref_set_z(self._h, np.ascontiguousarray(z, np.int32), int(next_sweep_index)),
            "ldaref_set_z")

    def get_nk(self):
        nk = np.zeros(self.K, np.int32)
        _ck(lib().ldaref_get_nk(self._h, nk), "ldaref_get_nk")
        return nk

    def get_nkw_row(self, w):
        row = np.zeros(self.K, np.int32)
        _ck(lib().ldaref_get_nkw_row(self._h, int(w), row), "ldaref_get_nkw_row")
        return row

    def get_ndk_row(self, d):
        row = np.zeros(self.K, np.int32)
        _ck(lib().ldaref_get_ndk_row(self._h, int(d), row), "ldaref_get_ndk_row")
        return row

    def get_alias_row(self, w):
        split = np.zeros(self.K, np.uint32)
        alias = np.zeros(self.K, np.uint32)
        cap = C.c_uint32()
        _ck(lib().ldaref_get_alias_row(self._h, int(w), split, alias, C.byref(cap)),
            "ldaref_get_alias_row")
        return split, alias, cap.value

    def get_sparse_table(self, w):
        n = C.c_int32()
        cap = C.c_uint32()
        qs = C.c_uint64()
        e = np.zeros(1, np.int32)
        u = np.zeros(1, np.uint32)
        _ck(lib().ldaref_get_sparse_table(self._h, int(w), 0, C.byref(n), e, u, u.copy(),
                                          C.byref(cap), C.byref(qs)), "ldaref_get_sparse_table")
        cnt = max(n.value, 1)
        topics = np.zeros(cnt, np.int32)
        split = np.zeros(cnt, np.uint32)
        alias = np.zeros(cnt, np.uint32)
        _ck(lib().ldaref_get_sparse_table(self._h, int(w), cnt, C.byref(n), topics, split, alias,
                                          C.byref(cap), C.byref(qs)), "ldaref_get_sparse_table")
        k = n.value
        return topics[:k], split[:k], alias[:k], cap.value, qs.value

    def get_beta_table(self):
        split = np.zeros(self.K, np.uint32)
        alias = np.zeros(self.K, np.uint32)
        cap = C.c_uint32()
        qb = C.c_uint64()
        _ck(lib().ldaref_get_beta_table(self._h, split, alias, C.byref(cap), C.byref(qb)),
            "ldaref_get_beta_table")
        return split, alias, cap.value, qb.value
