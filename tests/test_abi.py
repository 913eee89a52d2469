"""The C ABI without a GPU: the library loads, exports every function that
include/maddness.h declares, and rejects bad arguments on the host before any
launch (so these calls never touch a device)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mad():
    import paper_2106_10860_amd as m
    if not os.path.exists(m.LIB_PATH):
        from paper_2106_10860_amd.build import build
        build()
    return m


def declared_functions():
    text = open(os.path.join(ROOT, "include", "maddness.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(maddness_[a-z_]+)\s*\(", text)))


def test_header_and_library_agree(mad):
    names = declared_functions()
    assert set(names) == set(mad.EXPORTS)
    L = mad.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in maddness.h but not exported"


def test_workspace_size(mad):
    L = mad.lib()
    need = L.maddness_build_luts_workspace(512, 32, 256)
    assert need >= 8 * (32 * 16 * 256 + 32 * 256) + 4 * 256
    assert L.maddness_build_luts_workspace(0, 32, 256) == 0


def test_argument_errors_are_reported_on_the_host(mad):
    L = mad.lib()
    P = mad._Params
    fake = 0x1000   # never dereferenced: every call below fails validation first
    ok_params = P(16, 4, fake, fake, fake)

    def err():
        return L.maddness_last_error().decode()

    assert L.maddness_encode(None, fake, 10, 16, fake, None) == mad.MADDNESS_E_INVAL
    assert "params" in err()
    assert L.maddness_encode(C.byref(P(16, 0, fake, fake, fake)), fake, 10, 16, fake, None) == mad.MADDNESS_E_UNSUPPORTED
    assert L.maddness_encode(C.byref(P(16, 257, fake, fake, fake)), fake, 10, 16, fake, None) == mad.MADDNESS_E_UNSUPPORTED
    assert L.maddness_encode(C.byref(P(0, 4, fake, fake, fake)), fake, 10, 16, fake, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_encode(C.byref(ok_params), fake, -1, 16, fake, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_encode(C.byref(ok_params), fake, 10, 15, fake, None) == mad.MADDNESS_E_INVAL
    assert "lda" in err()
    assert L.maddness_encode(C.byref(ok_params), None, 10, 16, fake, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_encode(C.byref(ok_params), fake + 2, 10, 16, fake, None) == mad.MADDNESS_E_ALIGN
    assert L.maddness_encode(C.byref(ok_params), fake, 10, 16, None, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_encode(C.byref(P(16, 4, None, fake, fake)), fake, 10, 16, fake, None) == mad.MADDNESS_E_INVAL
    # N = 0 is a valid no-op
    assert L.maddness_encode(C.byref(ok_params), None, 0, 16, None, None) == mad.MADDNESS_OK

    assert L.maddness_scan(4, 8, fake, 10, fake, fake, fake, None, 8, None, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_scan(4, 8, fake, 10, fake, fake, fake, fake, 7, None, None) == mad.MADDNESS_E_INVAL
    assert "ldo" in err()
    assert L.maddness_scan(4, 0, fake, 10, fake, fake, fake, fake, 8, None, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_scan(300, 8, fake, 10, fake, fake, fake, fake, 8, None, None) == mad.MADDNESS_E_UNSUPPORTED
    assert L.maddness_scan(4, 8, fake, 10, fake, fake, fake, None, 0, fake + 1, None) == mad.MADDNESS_E_ALIGN
    assert L.maddness_scan(4, 8, None, 0, fake, fake, fake, fake, 8, None, None) == mad.MADDNESS_OK

    assert L.maddness_encode_scan(C.byref(ok_params), fake, 10, 16, 8, fake, fake, fake, None, 8, None,
                                  None, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_encode_scan(C.byref(ok_params), fake, 10, 8, 8, fake, fake, fake, fake, 8, None,
                                  None, None) == mad.MADDNESS_E_INVAL

    need = L.maddness_build_luts_workspace(16, 4, 8)
    assert L.maddness_build_luts(C.byref(ok_params), fake, 8, 8, fake, fake, fake, fake, need - 1,
                                 None) == mad.MADDNESS_E_UNSUPPORTED
    assert "workspace" in err()
    assert L.maddness_build_luts(C.byref(P(16, 4, fake, fake, None)), fake, 8, 8, fake, fake, fake, fake,
                                 need, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_build_luts(C.byref(ok_params), fake, 8, 7, fake, fake, fake, fake, need,
                                 None) == mad.MADDNESS_E_INVAL


def test_options(mad):
    L = mad.lib()
    for opt in range(4):
        assert L.maddness_get_option(opt) == 0
    assert L.maddness_get_option(4) == -1 and L.maddness_get_option(-1) == -1
    assert L.maddness_set_option(9, 0) == mad.MADDNESS_E_INVAL
    assert L.maddness_set_option(mad.MADDNESS_OPT_KERNELS, 3) == mad.MADDNESS_E_INVAL
    assert L.maddness_set_option(mad.MADDNESS_OPT_PHASED_ROWS, 1) == mad.MADDNESS_E_INVAL
    assert L.maddness_set_option(mad.MADDNESS_OPT_COLS_RUN, 3) == mad.MADDNESS_E_INVAL
    assert L.maddness_set_option(mad.MADDNESS_OPT_MAX_WORKGROUPS, -1) == mad.MADDNESS_E_INVAL
    assert L.maddness_set_option(mad.MADDNESS_OPT_COLS_RUN, 2) == mad.MADDNESS_OK
    assert L.maddness_get_option(mad.MADDNESS_OPT_COLS_RUN) == 2
    assert L.maddness_set_option(mad.MADDNESS_OPT_COLS_RUN, 0) == mad.MADDNESS_OK
    assert L.maddness_get_option(mad.MADDNESS_OPT_COLS_RUN) == 0


def test_binding_fails_loudly_without_the_library(mad, monkeypatch):
    import paper_2106_10860_amd as m
    monkeypatch.setattr(m, "_lib", None)
    monkeypatch.setattr(m, "LIB_PATH", "/nonexistent/libmaddness.so")
    with pytest.raises(ImportError):
        m.lib()


def test_static_workspace_entry_rejects_on_the_host(mad):
    """maddness_build_luts_static: argument and size errors come before any device call."""
    L = mad.lib()
    P = mad._Params
    fake = 0x1000
    assert L.maddness_build_luts_static(None, fake, 8, 8, fake, fake, fake, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_build_luts_static(C.byref(P(16, 4, fake, fake, None)), fake, 8, 8, fake, fake, fake,
                                        None) == mad.MADDNESS_E_INVAL
    assert L.maddness_build_luts_static(C.byref(P(16, 4, fake, fake, fake)), fake, 0, 8, fake, fake, fake,
                                        None) == mad.MADDNESS_E_INVAL
    # 64 codebooks x 2048 columns need 17.8 MB of workspace; the library holds 8 MiB
    assert L.maddness_build_luts_workspace(16, 64, 2048) > mad.STATIC_WORKSPACE_BYTES
    assert L.maddness_build_luts_static(C.byref(P(16, 64, fake, fake, fake)), fake, 2048, 2048, fake, fake, fake,
                                        None) == mad.MADDNESS_E_UNSUPPORTED
    assert "workspace" in L.maddness_last_error().decode()


def test_learning_calls_reject_on_the_host(mad):
    L = mad.lib()
    fake = 0x1000
    ok = (C.c_int32 * 4)(0, 8, 8, 16)
    assert L.maddness_learn_trees_workspace(1000, 16, 2, ok) > 1000 * 2
    assert L.maddness_learn_trees_workspace(0, 16, 2, ok) == 0
    assert L.maddness_learn_prototypes_workspace(16, 2) >= 8 * (32 * 32 * 2 + 32 * 16)
    assert L.maddness_learn_trees(fake, 0, 16, 16, 2, ok, fake, fake, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_trees(fake, 10, 15, 16, 2, ok, fake, fake, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_trees(None, 10, 16, 16, 2, ok, fake, fake, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_trees(fake, 10, 16, 16, 2, None, fake, fake, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    bad = (C.c_int32 * 4)(0, 8, 8, 17)
    assert L.maddness_learn_trees(fake, 10, 16, 16, 2, bad, fake, fake, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert "codebook 1" in L.maddness_last_error().decode()
    assert L.maddness_learn_trees(fake, 10, 16, 16, 2, ok, None, fake, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_trees(fake, 10, 16, 16, 2, ok, fake, fake, None, fake, 16, None) == mad.MADDNESS_E_UNSUPPORTED
    assert L.maddness_learn_trees(fake, 10, 16, 16, 2, ok, fake, fake, None, fake + 8, 1 << 30, None) == mad.MADDNESS_E_ALIGN
    assert L.maddness_learn_prototypes(fake, fake, 10, 16, 16, 2, ok, 1, -1.0, fake, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_prototypes(fake, fake, 10, 16, 16, 2, ok, 1, 1.0, None, fake, 1 << 30, None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_prototypes(fake, fake, 10, 16, 16, 2, ok, 0, 0.0, fake, fake, 16, None) == mad.MADDNESS_E_UNSUPPORTED
