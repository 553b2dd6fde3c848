"""The C-ABI library: it loads, exports every symbol the header declares, and rejects bad arguments
on the host before anything is launched (so all of this runs without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2202_10217_amd import binding as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tb.LIB_PATH):
        from paper_2202_10217_amd import build
        build.build()
    return tb.load()


def _declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(tbs_[a-z0-9_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_symbols()
    assert declared == set(tb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = {tb.tbs_status_string(s) for s in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert tb.tbs_status_string(99) == "unknown status"


def _syrk(lib, entry, dtype, N, M, A, lda, C, ldc):
    return getattr(lib, entry)(dtype, N, M, 1.0, ctypes.c_void_p(A), lda, 1.0, ctypes.c_void_p(C), ldc,
                               None, 0, None)


@pytest.mark.parametrize("entry", ["tbs_syrk_lower", "tbs_syrk_lower_square"])
def test_syrk_argument_checks(lib, entry):
    fake = 0x1000                                             # never dereferenced: checks come first
    assert _syrk(lib, entry, 7, 4, 4, fake, 4, fake, 4) == tb.TBS_EINVAL      # dtype
    assert _syrk(lib, entry, 0, -1, 4, fake, 4, fake, 4) == tb.TBS_EINVAL     # N < 0
    assert _syrk(lib, entry, 0, 4, -1, fake, 4, fake, 4) == tb.TBS_EINVAL     # M < 0
    assert _syrk(lib, entry, 0, 4, 8, fake, 7, fake, 4) == tb.TBS_EINVAL      # lda < M
    assert _syrk(lib, entry, 0, 4, 8, fake, 8, fake, 3) == tb.TBS_EINVAL      # ldc < N
    assert _syrk(lib, entry, 0, 4, 8, None, 8, fake, 4) == tb.TBS_EINVAL      # A NULL
    assert _syrk(lib, entry, 0, 4, 8, fake, 8, None, 4) == tb.TBS_EINVAL      # C NULL
    assert _syrk(lib, entry, 0, 1 << 40, 8, fake, 8, fake, 1 << 40) == tb.TBS_EINVAL
    assert _syrk(lib, entry, 0, 0, 8, None, 8, None, 1) == tb.TBS_OK          # N = 0: nothing to do


def test_noalloc_argument_checks(lib, monkeypatch):
    fake = ctypes.c_void_p(0x1000)                            # never dereferenced: checks come first
    f = lib.tbs_syrk_lower_noalloc
    assert f(7, 4, 4, 1.0, fake, 4, 1.0, fake, 4, None) == tb.TBS_EINVAL      # dtype
    assert f(0, -1, 4, 1.0, fake, 4, 1.0, fake, 4, None) == tb.TBS_EINVAL     # N < 0
    assert f(0, 4, 8, 1.0, fake, 7, 1.0, fake, 4, None) == tb.TBS_EINVAL      # lda < M
    assert f(0, 4, 8, 1.0, fake, 8, 1.0, fake, 3, None) == tb.TBS_EINVAL      # ldc < N
    assert f(0, 4, 8, 1.0, None, 8, 1.0, fake, 4, None) == tb.TBS_EINVAL      # A NULL
    assert f(0, 0, 8, 1.0, None, 8, 1.0, None, 1, None) == tb.TBS_OK          # N = 0: nothing to do
    # a plan whose parts do not fit the library's scratch array is refused before anything is launched
    monkeypatch.setenv("TBS_PLAN_TUNING", "1,2,3,0,2,3,16,1,0,1")
    assert tb.tbs_syrk_lower_workspace(tb.TBS_F64, 4096, 4096) > tb.NOALLOC_WORKSPACE_BYTES
    assert f(0, 4096, 4096, 1.0, fake, 4096, 1.0, fake, 4096, None) == tb.TBS_EWORKSPACE
    # the header's constant is the binding's
    text = open(os.path.join(ROOT, "include", "tbs_syrk.h")).read()
    assert re.search(r"#define TBS_NOALLOC_WORKSPACE_BYTES \(\(size_t\)128 << 20\)", text)
    assert tb.NOALLOC_WORKSPACE_BYTES == 128 << 20


def test_workspace_queries(lib):
    big = tb.tbs_syrk_lower_query(tb.TBS_F64, 32768, 512)
    assert tb.tbs_syrk_lower_workspace(tb.TBS_F64, 32768, 512) == 0 == big["workspace_bytes"]   # many blocks per unit
    small = tb.tbs_syrk_lower_query(tb.TBS_F64, 2048, 4096)
    assert tb.tbs_syrk_lower_workspace(tb.TBS_F64, 2048, 4096) == small["workspace_bytes"]
    assert small["workspace_bytes"] == small["n_sliced_blocks"] * small["max_slices"] * 6 * 4096 * 8
    assert tb.tbs_syrk_lower_query(tb.TBS_F64, 2048, 4096, 2)["workspace_bytes"] == 0        # plan without workspace
    n64 = tb.tbs_potrf_lower_workspace(tb.TBS_F64, 1000)
    n32 = tb.tbs_potrf_lower_workspace(tb.TBS_F32, 1000)
    assert n64 >= 4 and n32 >= 4                              # at least the info word
    with pytest.raises(tb.TbsError):
        tb.tbs_potrf_lower_workspace(tb.TBS_F64, -1)
    with pytest.raises(tb.TbsError):
        tb.tbs_syrk_lower_workspace(5, 1, 1)


def test_potrf_argument_checks(lib):
    fake = ctypes.c_void_p(0x1000)
    info = ctypes.c_int32(123)
    f = lib.tbs_potrf_lower
    assert f(0, -1, fake, 1, fake, 1 << 20, ctypes.byref(info), None) == tb.TBS_EINVAL
    assert f(3, 8, fake, 8, fake, 1 << 20, ctypes.byref(info), None) == tb.TBS_EINVAL
    assert f(0, 8, fake, 7, fake, 1 << 20, ctypes.byref(info), None) == tb.TBS_EINVAL
    assert f(0, 8, None, 8, fake, 1 << 20, ctypes.byref(info), None) == tb.TBS_EINVAL
    assert f(0, 8, fake, 8, fake, 2, ctypes.byref(info), None) == tb.TBS_EWORKSPACE
    assert f(0, 8, fake, 8, None, 0, ctypes.byref(info), None) == tb.TBS_EWORKSPACE
    assert f(0, 0, None, 1, None, 0, ctypes.byref(info), None) == tb.TBS_OK and info.value == 0


def test_query_and_enumerate_reject_bad_arguments(lib):
    with pytest.raises(tb.TbsError):
        tb.tbs_syrk_lower_query(tb.TBS_F64, -5, 3)
    with pytest.raises(tb.TbsError):
        tb.tbs_syrk_lower_enumerate(9, 100, 10)
    n = ctypes.c_int64(0)
    buf = (ctypes.c_int32 * 8)()
    st = lib.tbs_syrk_lower_enumerate(0, 4096, 4096, 0, buf, 1, ctypes.byref(n))
    assert st == tb.TBS_EWORKSPACE and n.value > 1
