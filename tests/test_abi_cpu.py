"""CPU-only checks of the C ABI: the library loads, exports what include/*.h declare,
and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2602_13692_amd import binding as ta

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(macro):
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(macro + r"\b[^;(]*?\b(ta_\w+)\s*\(", text))
    return sorted(names)


@pytest.mark.parametrize("path,macro,exports", [(ta.LIB_PATH, "TA_API", ta.EXPORTS),
                                                (ta.PROBE_LIB_PATH, "TA_PROBE_API", ta.PROBE_EXPORTS)])
def test_library_exports_every_declared_symbol(path, macro, exports):
    if not os.path.exists(path):
        pytest.fail(f"{path} missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(path)
    declared = _declared_symbols(macro)
    assert declared, f"no {macro} declarations found"
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared under include/ but not exported"
    assert set(declared) == set(exports)


def test_the_hot_path_library_holds_no_measurement_aid():
    lib = ctypes.CDLL(ta.LIB_PATH)
    for name in ta.PROBE_EXPORTS:
        assert not hasattr(lib, name)


def test_version_and_error_strings():
    assert ta.ta_version() >= 100
    assert ta.ta_strerror(ta.TA_OK) == "ok"
    for code in (ta.TA_ERR_INVALID_ARG, ta.TA_ERR_UNSUPPORTED, ta.TA_ERR_HIP, -99):
        assert ta.ta_strerror(code)


def test_workspace_size_and_descriptor_validation():
    good = ta.Desc(32, 8)
    n = ta.ta_workspace_bytes(good, 64, 1, 32768)
    assert n > 0 and n % 256 == 0
    # partials dominate: slots * Hq * 130 floats.  A batch this large streams on the tile kernel:
    # a program of 32k tokens has 4 bulk chunks of 512 pages and one leftover item (plus room for the
    # about 150 more slots that a chunk shortened on the device can need)
    assert 64 * (4 + 1) * 32 * 130 * 4 <= n < (64 * (4 + 2) + 160) * 32 * 130 * 4
    # four programs stay on the vector-ALU kernel: 16 bulk chunks of 128 pages and up to 4 pieces of
    # the leftover each
    assert ta.ta_workspace_bytes(good, 4, 1, 32768) >= 4 * (16 + 4) * 32 * 130 * 4
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, decode_chunk_pages=64), 64, 1, 32768) >= 64 * 36 * 32 * 130 * 4
    assert ta.ta_workspace_bytes(good, 64, 2048, 34816) > 0
    # append-prefill of few query tiles cuts every tile's keys into chunks and keeps a partial
    # (130 floats) per row and chunk: one program's 64 new tokens on 32k cached tokens fill the
    # chip with about 256 workgroups, 8 kv heads x 32 chunks; a batch that fills it anyway needs none
    few = ta.ta_workspace_bytes(good, 1, 64, 32832)
    assert 64 * 32 * 24 * 130 * 4 <= few <= 64 * 32 * 40 * 130 * 4
    assert ta.ta_workspace_bytes(good, 64, 64, 32832) < 64 * 64 * 32 * 130 * 4
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
    assert lib.ta_restore_staging_min_bytes(1000) == 0      # the slot list travels in the kernel arguments
    assert lib.ta_restore_staging_full_bytes(1000, 32768) == 2 * 32768
    # staging may be absent only together with a size of zero
    one = ctypes.c_void_p(4096)
    slot = (ctypes.c_int32 * 1)(0)
    assert lib.ta_kv_page_restore(one, one, 32768, one, one, slot, 1, 10, null, 512, null) == ta.TA_ERR_INVALID_ARG
    assert lib.ta_kv_page_evict(one, one, 32768, one, one, slot, 1, 10, null, 512, null) == ta.TA_ERR_INVALID_ARG
    # a chunk length the split-K plan does not offer; with a bf16 cache 256 and 512 pages ask for the tile
    # kernel (any head shape), with an FP8 cache they are item lengths of its own kernel
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, decode_chunk_pages=24), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, decode_chunk_pages=1024), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, decode_chunk_pages=256), 4, 1, 100) > 0
    assert ta.ta_workspace_bytes(ta.Desc(64, 8, decode_chunk_pages=512), 4, 1, 100) > 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, pool_pages=-1), 4, 1, 100) == 0
    # the number of key chunks of append-prefill: 0 .. 1024; asking for chunks costs their partials
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, prefill_key_chunks=-1), 4, 64, 5000) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, prefill_key_chunks=1025), 4, 64, 5000) == 0
    uncut = ta.ta_workspace_bytes(ta.Desc(32, 8, prefill_key_chunks=1), 64, 64, 5000)
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, prefill_key_chunks=4), 64, 64, 5000) >= uncut + 64 * 64 * 32 * 4 * 130 * 4
    # the FP8 cache format needs its two scales, positive and finite; other formats do not exist
    fp8 = dict(kv_format=ta.KV_FP8_E4M3)
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, k_scale=0.02, v_scale=0.02, **fp8), 4, 1, 100) > 0
    assert ta.ta_workspace_bytes(ta.Desc(64, 8, k_scale=0.02, v_scale=0.02, **fp8), 64, 1, 32768) > 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, k_scale=0.0, v_scale=0.02, **fp8), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, k_scale=0.02, v_scale=-1.0, **fp8), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, k_scale=float("inf"), v_scale=1.0, **fp8), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(32, 8, kv_format=2, k_scale=1.0, v_scale=1.0), 4, 1, 100) == 0
    assert ta.ta_workspace_bytes(ta.Desc(64, 8, decode_chunk_pages=256, k_scale=1.0, v_scale=1.0, **fp8), 4, 1, 100) > 0
    assert ta.ta_workspace_bytes(ta.Desc(64, 8, decode_chunk_pages=1024, k_scale=1.0, v_scale=1.0, **fp8), 4, 1, 100) == 0
    # the measurement aids (their own library) reject missing or misaligned buffers and bad sizes
    probe = ta._probe_lib()
    assert probe.ta_matrix_core_probe(null, 10, null, null) == -1
    assert probe.ta_matrix_core_probe(ctypes.c_void_p(4096), 0, ctypes.c_void_p(8192), null) == -1
    assert probe.ta_matrix_core_probe(ctypes.c_void_p(4100), 10, ctypes.c_void_p(8192), null) == -1
    assert probe.ta_stream_read_probe(null, 4096, null, null) == -1
    assert probe.ta_stream_read_probe(ctypes.c_void_p(4096), 24, ctypes.c_void_p(8192), null) == -1
