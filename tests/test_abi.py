"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before touching
the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1412_1576_amd import lda
    if not os.path.exists(lda.LIB_PATH):
        from paper_1412_1576_amd import build
        build.build_library()
    return lda.load_library()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "lda_mi355x.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lda_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    from paper_1412_1576_amd import lda
    names = header_symbols()
    assert "lda_init" in names and "lda_sweep" in names and len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(lda.EXPORTS) == names


def test_options_struct_layout():
    from paper_1412_1576_amd import lda
    # stream, the three allocator fields, 10 int32, 5 reserved int32
    assert C.sizeof(lda.lda_options) == 4 * 8 + 15 * 4 + 4  # padded to 8-byte alignment
    assert lda.lda_options.dev_alloc.offset == 8
    assert lda.lda_options.dense_rows.offset == 32


def test_bad_arguments_are_rejected_on_the_host(lib):
    from paper_1412_1576_amd import lda
    doff = np.array([0, 2, 3], np.int64)
    w = np.array([0, 1, 1], np.int32)

    def init(D=2, V=2, K=2, doff=doff, w=w, alpha=0.1, beta=0.1, **opt):
        h = C.c_void_p()
        o = lda.lda_options()
        for k, v in opt.items():
            setattr(o, k, v)
        rc = lib.lda_init(C.byref(h), D, V, K, doff, w, alpha, beta, 0, C.byref(o))
        assert not h.value
        return rc, lib.lda_last_error(None).decode()

    assert init(K=0)[0] == lda.LDA_ERR_ARG
    assert init(V=0)[0] == lda.LDA_ERR_ARG
    assert init(alpha=0.0)[0] == lda.LDA_ERR_ARG
    assert init(beta=-1.0)[0] == lda.LDA_ERR_ARG
    assert init(alpha=float("nan"))[0] == lda.LDA_ERR_ARG
    assert init(doff=np.array([1, 2, 3], np.int64))[0] == lda.LDA_ERR_ARG
    assert init(doff=np.array([0, 3, 2], np.int64))[0] == lda.LDA_ERR_ARG
    assert init(doff=np.array([0, 0, 0], np.int64))[0] == lda.LDA_ERR_ARG  # empty corpus
    assert init(proposal_mode=3)[0] == lda.LDA_ERR_ARG
    assert init(record_bucket_tokens=1000)[0] == lda.LDA_ERR_ARG  # not a power of two
    only_alloc = lda.DEV_ALLOC(lambda nbytes, user: None)
    assert init(dev_alloc=only_alloc)[0] == lda.LDA_ERR_ARG  # dev_free missing
    rc, msg = init(K=0)
    assert "K" in msg
    # calls on a NULL context
    assert lib.lda_build_alias(None) == lda.LDA_ERR_ARG
    assert lib.lda_sweep(None, 2) == lda.LDA_ERR_ARG
    assert lib.lda_num_tokens(None) == -1
    lib.lda_destroy(None)
