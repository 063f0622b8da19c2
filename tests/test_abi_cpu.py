"""CPU-only checks of the C ABI: the library loads, exports what include/*.h declare,
and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2602_13692_amd import binding as ta

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"TA_API[^;(]*?\b(ta_\w+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(ta.LIB_PATH):
        pytest.fail(f"{ta.LIB_PATH} missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(ta.LIB_PATH)
    declared = _declared_symbols()
    assert declared, "no TA_API declarations found"
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared under include/ but not exported"
    assert set(declared) == set(ta.EXPORTS)


def test_version_and_error_strings():
    assert ta.ta_version() >= 100
    assert ta.ta_strerror(ta.TA_OK) == "ok"
    for code in (ta.TA_ERR_INVALID_ARG, ta.TA_ERR_UNSUPPORTED, ta.TA_ERR_HIP, -99):
        assert ta.ta_strerror(code)


def test_workspace_size_and_descriptor_validation():
    good = ta.Desc(32, 8)
    n = ta.ta_workspace_bytes(good, 64, 1, 32768)
    assert n > 0 and n % 256 == 0
    # partials dominate: chunks * Hq * 130 floats
    assert n >= 64 * 32 * 32 * 130 * 4
    assert ta.ta_workspace_bytes(good, 64, 2048, 34816) > 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, head_dim=64), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, page_size=32), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 5), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(48, 1), 4, 1, 100) == 0       # group 48 unsupported
    assert ta.ta_workspace_bytes(good, -1, 1, 100) == 0


def test_host_side_rejections_need_no_device():
    lib = ta._lib()
    d = ta.Desc(32, 8).c()
    null = ctypes.c_void_p(None)
    # batch 0 is a no-op, checked before any pointer
    assert lib.ta_paged_decode(ctypes.byref(d), null, null, null, null, 0, null, 0, 0, null, null, null, 0, null) == ta.TA_OK
    # null pointers with batch > 0
    assert lib.ta_paged_decode(ctypes.byref(d), null, null, null, null, 4, null, 2, 64, null, null, null, 0, null) == ta.TA_ERR_INVALID_ARG
    bad = ta.Desc(32, 8, head_dim=256).c()
    assert lib.ta_paged_decode(ctypes.byref(bad), null, null, null, null, 4, null, 2, 64, null, null, null, 0, null) == ta.TA_ERR_UNSUPPORTED
    neg = ta.Desc(32, 8, scale=-1.0).c()
    assert lib.ta_paged_decode(ctypes.byref(neg), null, null, null, null, 4, null, 2, 64, null, null, null, 0, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_append_prefill(ctypes.byref(d), null, null, null, null, null, 0, null, 0, 0, 0, 0, null, null, null, 0, null) == ta.TA_OK
    assert lib.ta_append_prefill(ctypes.byref(d), null, null, null, null, null, 4, null, 2, 10, 5, 64, null, null, null, 0, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_kv_page_restore(null, null, 32768, null, null, null, 0, 10, null, 0, null) == ta.TA_OK
    assert lib.ta_kv_page_restore(null, null, 32768, null, null, null, 3, 10, null, 0, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_kv_page_restore(null, null, 32768, null, null, null, -1, 10, null, 0, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_restore_staging_min_bytes(1000) == 4096
    assert lib.ta_restore_staging_full_bytes(1000, 32768) == 4096 + 2 * 32768
    # the matrix-core probe rejects missing or misaligned buffers and a non-positive count
    assert lib.ta_matrix_core_probe(null, 10, null, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_matrix_core_probe(ctypes.c_void_p(4096), 0, ctypes.c_void_p(8192), null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_matrix_core_probe(ctypes.c_void_p(4100), 10, ctypes.c_void_p(8192), null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_stream_read_probe(null, 4096, null, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_stream_read_probe(ctypes.c_void_p(4096), 24, ctypes.c_void_p(8192), null) == ta.TA_ERR_INVALID_ARG
