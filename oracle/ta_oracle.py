"""ctypes front end of ta_oracle.c (test infrastructure only).

Arrays are numpy: bf16 data travels as uint16 bit patterns, results are float64.
The arithmetic lives in the C file; this module only marshals arguments.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ta_oracle.c")
_LIB = os.path.join(_HERE, "libta_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ta_oracle.c with gcc (OpenMP, -O2) into libta_oracle.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Geom(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("scale", ctypes.c_double),
        ("stride_page", ctypes.c_int64),
        ("stride_head", ctypes.c_int64),
        ("stride_token", ctypes.c_int64),
    ]


@dataclass
class Geometry:
    """Head counts and pool layout.  Default pool layout is [P][Hkv][page][d]."""

    num_q_heads: int
    num_kv_heads: int
    head_dim: int = 128
    page_size: int = 16
    scale: float | None = None  # None -> 1/sqrt(head_dim)
    stride_page: int | None = None
    stride_head: int | None = None
    stride_token: int | None = None

    def c_struct(self) -> _Geom:
        st = self.stride_token if self.stride_token is not None else self.head_dim
        sh = self.stride_head if self.stride_head is not None else self.page_size * self.head_dim
        sp = (
            self.stride_page
            if self.stride_page is not None
            else self.num_kv_heads * self.page_size * self.head_dim
        )
        scale = self.scale if self.scale is not None else 1.0 / math.sqrt(self.head_dim)
        return _Geom(
            self.num_q_heads, self.num_kv_heads, self.head_dim, self.page_size, scale, sp, sh, st
        )


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ta_oracle_num_threads.restype = ctypes.c_int
        _lib.ta_oracle_kv_page_restore.restype = ctypes.c_int
        _lib.ta_oracle_kv_page_evict.restype = ctypes.c_int
        _lib.ta_oracle_kv_append.restype = None
        _lib.ta_oracle_widen_e4m3.restype = None
        _lib.ta_oracle_quantise_e4m3.restype = None
        _lib.ta_oracle_kv_append_fp8.restype = None
        _lib.ta_oracle_append_prefill_fp8.restype = None
        _lib.ta_oracle_paged_decode_fp8.restype = None
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 data must be passed as uint16 bit patterns"
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_load().ta_oracle_num_threads())


def paged_decode(geom: Geometry, q, k_pool, v_pool, block_table, context_lens):
    """q uint16 [B,Hq,d] -> (out f64 [B,Hq,d], lse f64 [B,Hq])."""
    lib = _load()
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    block_table = _i32(block_table)
    context_lens = _i32(context_lens)
    B = int(context_lens.shape[0])
    stride = int(block_table.shape[1]) if block_table.ndim == 2 else 0
    out = np.zeros((B, geom.num_q_heads, geom.head_dim), dtype=np.float64)
    lse = np.zeros((B, geom.num_q_heads), dtype=np.float64)
    g = geom.c_struct()
    lib.ta_oracle_paged_decode(
        ctypes.byref(g), _p(q), _p(k_pool), _p(v_pool), _p(block_table),
        ctypes.c_int64(stride), _p(context_lens), ctypes.c_int32(B), _p(out), _p(lse),
    )
    return out, lse


def widen_e4m3(codes) -> np.ndarray:
    """Values (float64) of OCP E4M3 codes given as uint8."""
    lib = _load()
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    values = np.zeros(codes.shape, dtype=np.float64)
    lib.ta_oracle_widen_e4m3(_p(codes), ctypes.c_int64(codes.size), _p(values))
    return values


def quantise_e4m3(x, scale) -> np.ndarray:
    """E4M3 codes (uint8) of x / scale: x float32, the division in float32, nearest value with ties to
    the even code, saturating at +-448, NaN kept."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.zeros(x.shape, dtype=np.uint8)
    lib.ta_oracle_quantise_e4m3(_p(x), ctypes.c_int64(x.size), ctypes.c_float(float(np.float32(scale))), _p(codes))
    return codes


def kv_append_fp8(geom: Geometry, new_k, new_v, cu_new_lens, k_pool, v_pool, k_scale, v_scale, block_table,
                  context_lens) -> None:
    """Quantise the new tokens' bf16 rows (uint16 [total_new,Hkv,d]) into the uint8 code pools in place."""
    lib = _load()
    new_k, new_v = _u16(new_k), _u16(new_v)
    for a in (k_pool, v_pool):
        assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    cu_new_lens = _i32(cu_new_lens)
    block_table = _i32(block_table)
    context_lens = _i32(context_lens)
    B = int(context_lens.shape[0])
    stride = int(block_table.shape[1]) if block_table.ndim == 2 else 0
    g = geom.c_struct()
    lib.ta_oracle_kv_append_fp8(
        ctypes.byref(g), _p(new_k), _p(new_v), _p(cu_new_lens), _p(k_pool), _p(v_pool),
        ctypes.c_float(float(np.float32(k_scale))), ctypes.c_float(float(np.float32(v_scale))),
        _p(block_table), ctypes.c_int64(stride), _p(context_lens), ctypes.c_int32(B),
    )


def paged_decode_fp8(geom: Geometry, q, k_pool, v_pool, k_scale, v_scale, block_table, context_lens):
    """Decode over an FP8 cache: q uint16 bf16 [B,Hq,d]; pools uint8 E4M3 codes; scales are the
    call's fp32 scales (the value of a cached element is code value * scale)."""
    lib = _load()
    q = _u16(q)
    k_pool, v_pool = np.ascontiguousarray(k_pool), np.ascontiguousarray(v_pool)
    assert k_pool.dtype == np.uint8 and v_pool.dtype == np.uint8, "FP8 pools travel as uint8 codes"
    block_table = _i32(block_table)
    context_lens = _i32(context_lens)
    B = int(context_lens.shape[0])
    stride = int(block_table.shape[1]) if block_table.ndim == 2 else 0
    out = np.zeros((B, geom.num_q_heads, geom.head_dim), dtype=np.float64)
    lse = np.zeros((B, geom.num_q_heads), dtype=np.float64)
    g = geom.c_struct()
    lib.ta_oracle_paged_decode_fp8(
        ctypes.byref(g), _p(q), _p(k_pool), _p(v_pool), ctypes.c_double(float(np.float32(k_scale))),
        ctypes.c_double(float(np.float32(v_scale))), _p(block_table), ctypes.c_int64(stride),
        _p(context_lens), ctypes.c_int32(B), _p(out), _p(lse),
    )
    return out, lse


def append_prefill(geom: Geometry, q, cu_q_lens, k_pool, v_pool, block_table, context_lens):
    """q uint16 [total_q,Hq,d] -> (out f64 [total_q,Hq,d], lse f64 [total_q,Hq])."""
    lib = _load()
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    block_table = _i32(block_table)
    context_lens = _i32(context_lens)
    cu_q_lens = _i32(cu_q_lens)
    B = int(context_lens.shape[0])
    total_q = int(cu_q_lens[B]) if B > 0 else 0
    stride = int(block_table.shape[1]) if block_table.ndim == 2 else 0
    out = np.zeros((total_q, geom.num_q_heads, geom.head_dim), dtype=np.float64)
    lse = np.zeros((total_q, geom.num_q_heads), dtype=np.float64)
    g = geom.c_struct()
    lib.ta_oracle_append_prefill(
        ctypes.byref(g), _p(q), _p(cu_q_lens), _p(k_pool), _p(v_pool), _p(block_table),
        ctypes.c_int64(stride), _p(context_lens), ctypes.c_int32(B), _p(out), _p(lse),
    )
    return out, lse


def append_prefill_fp8(geom: Geometry, q, cu_q_lens, k_pool, v_pool, k_scale, v_scale, block_table, context_lens):
    """Append-prefill over an FP8 cache: q uint16 bf16 [total_q,Hq,d]; pools uint8 E4M3 codes."""
    lib = _load()
    q = _u16(q)
    k_pool, v_pool = np.ascontiguousarray(k_pool), np.ascontiguousarray(v_pool)
    assert k_pool.dtype == np.uint8 and v_pool.dtype == np.uint8, "FP8 pools travel as uint8 codes"
    block_table = _i32(block_table)
    context_lens = _i32(context_lens)
    cu_q_lens = _i32(cu_q_lens)
    B = int(context_lens.shape[0])
    total_q = int(cu_q_lens[B]) if B > 0 else 0
    stride = int(block_table.shape[1]) if block_table.ndim == 2 else 0
    out = np.zeros((total_q, geom.num_q_heads, geom.head_dim), dtype=np.float64)
    lse = np.zeros((total_q, geom.num_q_heads), dtype=np.float64)
    g = geom.c_struct()
    lib.ta_oracle_append_prefill_fp8(
        ctypes.byref(g), _p(q), _p(cu_q_lens), _p(k_pool), _p(v_pool), ctypes.c_double(float(np.float32(k_scale))),
        ctypes.c_double(float(np.float32(v_scale))), _p(block_table), ctypes.c_int64(stride), _p(context_lens),
        ctypes.c_int32(B), _p(out), _p(lse),
    )
    return out, lse


def attend_rows(geom: Geometry, q, k_pool, v_pool, block_table, row_b, row_t, row_h, row_visible):
    """Selected rows: (program, packed query token, query head, visible keys) each.

    Returns (out f64 [n,d], lse f64 [n]).
    """
    lib = _load()
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    block_table = _i32(block_table)
    row_b = _i32(row_b)
    row_h = _i32(row_h)
    row_t = np.ascontiguousarray(row_t, dtype=np.int64)
    row_visible = np.ascontiguousarray(row_visible, dtype=np.int64)
    n = int(row_b.shape[0])
    stride = int(block_table.shape[1])
    out = np.zeros((n, geom.head_dim), dtype=np.float64)
    lse = np.zeros((n,), dtype=np.float64)
    g = geom.c_struct()
    lib.ta_oracle_attend_rows(
        ctypes.byref(g), _p(q), _p(k_pool), _p(v_pool), _p(block_table), ctypes.c_int64(stride),
        ctypes.c_int64(n), _p(row_b), _p(row_t), _p(row_h), _p(row_visible), _p(out), _p(lse),
    )
    return out, lse


def row_probs(geom: Geometry, q_row, h, k_pool, v_pool, table_row, visible):
    """Softmax probabilities of one row: (probs f64 [visible], out f64 [d], lse)."""
    lib = _load()
    q_row, k_pool, v_pool = _u16(q_row), _u16(k_pool), _u16(v_pool)
    table_row = _i32(table_row)
    probs = np.zeros((max(int(visible), 1),), dtype=np.float64)
    out = np.zeros((geom.head_dim,), dtype=np.float64)
    lse = ctypes.c_double(0.0)
    g = geom.c_struct()
    lib.ta_oracle_row_probs(
        ctypes.byref(g), _p(q_row), ctypes.c_int32(int(h)), _p(k_pool), _p(v_pool), _p(table_row),
        ctypes.c_int64(int(visible)), _p(probs), _p(out), ctypes.byref(lse),
    )
    return probs[: int(visible)], out, float(lse.value)


def kv_page_restore(k_pool, v_pool, page_bytes, host_k, host_v, dst_slots, pool_pages) -> int:
    """Scatter pages into the uint8 pools in place; returns 0 or -1 (bad slot list)."""
    lib = _load()
    for a in (k_pool, v_pool, host_k, host_v):
        assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    dst_slots = _i32(dst_slots)
    return int(
        lib.ta_oracle_kv_page_restore(
            _p(k_pool), _p(v_pool), ctypes.c_int64(int(page_bytes)), _p(host_k), _p(host_v),
            _p(dst_slots), ctypes.c_int32(int(dst_slots.shape[0])), ctypes.c_int32(int(pool_pages)),
        )
    )


def kv_page_evict(k_pool, v_pool, page_bytes, host_k, host_v, src_slots, pool_pages) -> int:
    """Gather pages out of the uint8 pools into host_k / host_v in place; returns 0 or -1."""
    lib = _load()
    for a in (k_pool, v_pool, host_k, host_v):
        assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    src_slots = _i32(src_slots)
    return int(
        lib.ta_oracle_kv_page_evict(
            _p(k_pool), _p(v_pool), ctypes.c_int64(int(page_bytes)), _p(host_k), _p(host_v),
            _p(src_slots), ctypes.c_int32(int(src_slots.shape[0])), ctypes.c_int32(int(pool_pages)),
        )
    )


def kv_append(geom: Geometry, new_k, new_v, cu_new_lens, k_pool, v_pool, block_table, context_lens) -> None:
    """Write the new tokens' rows (uint16 [total_new,Hkv,d]) into the uint16 pools in place."""
    lib = _load()
    new_k, new_v = _u16(new_k), _u16(new_v)
    for a in (k_pool, v_pool):
        assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    cu_new_lens = _i32(cu_new_lens)
    block_table = _i32(block_table)
    context_lens = _i32(context_lens)
    B = int(context_lens.shape[0])
    stride = int(block_table.shape[1]) if block_table.ndim == 2 else 0
    g = geom.c_struct()
    lib.ta_oracle_kv_append(
        ctypes.byref(g), _p(new_k), _p(new_v), _p(cu_new_lens), _p(k_pool), _p(v_pool),
        _p(block_table), ctypes.c_int64(stride), _p(context_lens), ctypes.c_int32(B),
    )
