"""ctypes binding of the HIP library: same names as the C ABI, argument marshalling only.

Tensors are torch tensors (device memory and streams are torch's); every step
of the computation runs in the library's kernels.  If the library is missing
the import of any entry point fails loudly; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TA_LIB_PATH selects another build of the same library (kernel experiments); default: in-tree
LIB_PATH = os.environ.get("TA_LIB_PATH", os.path.join(_HERE, "libta_hip.so"))
# the benchmark's measurement aids live in a library of their own
PROBE_LIB_PATH = os.path.join(_HERE, "libta_probe.so")

TA_OK = 0
TA_ERR_INVALID_ARG = -1
TA_ERR_UNSUPPORTED = -2
TA_ERR_HIP = -3
TA_ERR_TOO_LARGE = -4
KV_BF16, KV_FP8_E4M3 = 0, 1
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = (
    "ta_version", "ta_strerror", "ta_last_hip_error", "ta_workspace_bytes", "ta_paged_decode",
    "ta_append_prefill", "ta_restore_staging_min_bytes", "ta_restore_staging_full_bytes",
    "ta_kv_page_restore", "ta_kv_page_evict", "ta_kv_append", "ta_profile_events",
    "ta_set_debug_checks", "ta_sched_tick", "ta_paged_decode_static",
    "ta_sim_create", "ta_sim_destroy", "ta_sim_tick", "ta_sim_fetch", "ta_sim_programs", "ta_sim_page_table",
)
PROBE_EXPORTS = ("ta_matrix_core_probe", "ta_stream_read_probe", "ta_issue_port_probe")


class TaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        text = _lib().ta_strerror(status).decode()
        extra = f" (hipError {_lib().ta_last_hip_error()})" if status == TA_ERR_HIP else ""
        super().__init__(f"{where}: {text}{extra}")


class AttnDesc(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("pool_pages", ctypes.c_int32),
        ("pool_stride_page", ctypes.c_int64),
        ("pool_stride_head", ctypes.c_int64),
        ("pool_stride_token", ctypes.c_int64),
        ("decode_chunk_pages", ctypes.c_int32),
        ("kv_format", ctypes.c_int32),
        ("k_scale", ctypes.c_float),
        ("v_scale", ctypes.c_float),
        ("prefill_key_chunks", ctypes.c_int32),
    ]


@dataclass
class Desc:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int = 128
    page_size: int = 16
    scale: float = 0.0
    pool_stride_page: int = 0
    pool_stride_head: int = 0
    pool_stride_token: int = 0
    pool_pages: int = 0
    decode_chunk_pages: int = 0
    kv_format: int = 0          # KV_BF16 or KV_FP8_E4M3
    k_scale: float = 0.0
    v_scale: float = 0.0
    prefill_key_chunks: int = 0

    def c(self) -> AttnDesc:
        return AttnDesc(self.num_q_heads, self.num_kv_heads, self.head_dim, self.page_size,
                        self.scale, self.pool_pages, self.pool_stride_page, self.pool_stride_head,
                        self.pool_stride_token, self.decode_chunk_pages, self.kv_format, self.k_scale,
                        self.v_scale, self.prefill_key_chunks)


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2602_13692_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lib.ta_version.restype = i32
        lib.ta_strerror.restype = ctypes.c_char_p
        lib.ta_strerror.argtypes = [ctypes.c_int]
        lib.ta_last_hip_error.restype = ctypes.c_int
        lib.ta_workspace_bytes.restype = sz
        lib.ta_workspace_bytes.argtypes = [vp, i32, i32, i32]
        lib.ta_paged_decode.restype = ctypes.c_int
        lib.ta_paged_decode.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, sz, vp]
        lib.ta_paged_decode_static.restype = ctypes.c_int
        lib.ta_paged_decode_static.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp, vp]
        lib.ta_append_prefill.restype = ctypes.c_int
        lib.ta_append_prefill.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, vp, vp,
                                          vp, sz, vp]
        lib.ta_restore_staging_min_bytes.restype = sz
        lib.ta_restore_staging_min_bytes.argtypes = [i32]
        lib.ta_restore_staging_full_bytes.restype = sz
        lib.ta_restore_staging_full_bytes.argtypes = [i32, sz]
        lib.ta_kv_page_restore.restype = ctypes.c_int
        lib.ta_kv_page_restore.argtypes = [vp, vp, sz, vp, vp, vp, i32, i32, vp, sz, vp]
        lib.ta_kv_page_evict.restype = ctypes.c_int
        lib.ta_kv_page_evict.argtypes = [vp, vp, sz, vp, vp, vp, i32, i32, vp, sz, vp]
        lib.ta_kv_append.restype = ctypes.c_int
        lib.ta_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, i32, vp]
        lib.ta_sched_tick.restype = ctypes.c_int
        lib.ta_sched_tick.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp]
        lib.ta_sim_create.restype = vp
        lib.ta_sim_create.argtypes = [vp, vp, vp, vp, vp]
        lib.ta_sim_destroy.restype = None
        lib.ta_sim_destroy.argtypes = [vp]
        lib.ta_sim_tick.restype = ctypes.c_int
        lib.ta_sim_tick.argtypes = [vp, vp, vp]
        lib.ta_sim_fetch.restype = ctypes.c_int
        lib.ta_sim_fetch.argtypes = [vp, vp, vp]
        lib.ta_sim_programs.restype = ctypes.c_int
        lib.ta_sim_programs.argtypes = [vp, vp]
        lib.ta_sim_page_table.restype = i32
        lib.ta_sim_page_table.argtypes = [vp, i32, vp, i32]
        lib.ta_profile_events.restype = None
        lib.ta_profile_events.argtypes = [vp, vp]
        lib.ta_set_debug_checks.restype = ctypes.c_int
        lib.ta_set_debug_checks.argtypes = [ctypes.c_int]
        _LIB = lib
    return _LIB


_PROBE_LIB = None


def _probe_lib():
    global _PROBE_LIB
    if _PROBE_LIB is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise ImportError(f"{PROBE_LIB_PATH} is missing: build it with `python -m paper_2602_13692_amd.build`")
        lib = ctypes.CDLL(PROBE_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lib.ta_matrix_core_probe.restype = ctypes.c_int
        lib.ta_matrix_core_probe.argtypes = [vp, i32, vp, vp]
        lib.ta_stream_read_probe.restype = ctypes.c_int
        lib.ta_stream_read_probe.argtypes = [vp, sz, vp, vp]
        lib.ta_issue_port_probe.restype = ctypes.c_int
        lib.ta_issue_port_probe.argtypes = [i32, i32, i32, vp, vp]
        _PROBE_LIB = lib
    return _PROBE_LIB


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != TA_OK:
        raise TaError(status, where)


def ta_version() -> int:
    return int(_lib().ta_version())


def ta_strerror(status: int) -> str:
    return _lib().ta_strerror(status).decode()


def ta_last_hip_error() -> int:
    return int(_lib().ta_last_hip_error())


def ta_set_debug_checks(on: bool) -> bool:
    """Switches the metadata checks of the whole process on or off; returns the previous mode."""
    return bool(_lib().ta_set_debug_checks(1 if on else 0))


def ta_workspace_bytes(desc: Desc, batch: int, max_q_len: int, max_context_len: int) -> int:
    d = desc.c()
    return int(_lib().ta_workspace_bytes(ctypes.byref(d), batch, max_q_len, max_context_len))


def ta_paged_decode(desc: Desc, q, k_pool, v_pool, block_table, context_lens, max_context_len: int,
                    out, lse, workspace, stream=None, check: bool = True) -> int:
    """q,out bf16 [B,Hq,128]; pools bf16; block_table int32 [B,stride]; context_lens int32 [B]."""
    d = desc.c()
    rc = _lib().ta_paged_decode(
        ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
        int(block_table.shape[1]) if block_table is not None and block_table.dim() == 2 else 0,
        _ptr(context_lens), int(context_lens.shape[0]) if context_lens is not None else 0,
        int(max_context_len), _ptr(out), _ptr(lse), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream(stream))
    if check:
        _check(rc, "ta_paged_decode")
    return rc


def ta_paged_decode_static(desc: Desc, q, k_pool, v_pool, block_table, context_lens, max_context_len: int,
                           out, lse, stream=None, check: bool = True) -> int:
    """ta_paged_decode without a workspace: the library's own device array holds the split-K scratch."""
    d = desc.c()
    rc = _lib().ta_paged_decode_static(
        ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
        int(block_table.shape[1]) if block_table is not None and block_table.dim() == 2 else 0,
        _ptr(context_lens), int(context_lens.shape[0]) if context_lens is not None else 0,
        int(max_context_len), _ptr(out), _ptr(lse), _stream(stream))
    if check:
        _check(rc, "ta_paged_decode_static")
    return rc


def ta_append_prefill(desc: Desc, q, cu_q_lens, k_pool, v_pool, block_table, context_lens,
                      total_q: int, max_q_len: int, max_context_len: int, out, lse, workspace,
                      stream=None, check: bool = True) -> int:
    """q,out bf16 [total_q,Hq,128]; cu_q_lens int32 [B+1]; the rest as for ta_paged_decode."""
    d = desc.c()
    rc = _lib().ta_append_prefill(
        ctypes.byref(d), _ptr(q), _ptr(cu_q_lens), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
        int(block_table.shape[1]) if block_table is not None and block_table.dim() == 2 else 0,
        _ptr(context_lens), int(context_lens.shape[0]) if context_lens is not None else 0,
        int(total_q), int(max_q_len), int(max_context_len), _ptr(out), _ptr(lse), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()) if workspace is not None else 0,
        _stream(stream))
    if check:
        _check(rc, "ta_append_prefill")
    return rc


def ta_restore_staging_min_bytes(n_pages: int) -> int:
    return int(_lib().ta_restore_staging_min_bytes(n_pages))


def ta_restore_staging_full_bytes(n_pages: int, page_bytes: int) -> int:
    return int(_lib().ta_restore_staging_full_bytes(n_pages, page_bytes))


def ta_kv_page_restore(k_pool, v_pool, page_bytes: int, host_k, host_v, dst_slots, pool_pages: int,
                       staging, stream=None, check: bool = True) -> int:
    """host_k/host_v: pinned CPU tensors [n,...]; dst_slots: CPU int32 tensor [n]."""
    n = int(dst_slots.shape[0]) if dst_slots is not None else 0
    rc = _lib().ta_kv_page_restore(
        _ptr(k_pool), _ptr(v_pool), int(page_bytes), _ptr(host_k), _ptr(host_v), _ptr(dst_slots), n,
        int(pool_pages), _ptr(staging),
        int(staging.numel() * staging.element_size()) if staging is not None else 0, _stream(stream))
    if check:
        _check(rc, "ta_kv_page_restore")
    return rc


def ta_kv_page_evict(k_pool, v_pool, page_bytes, host_k, host_v, src_slots, pool_pages, staging,
                     stream=None, check: bool = True) -> int:
    """src_slots: CPU int32 tensor; host_k / host_v: pinned CPU tensors that receive the pages."""
    n = int(src_slots.shape[0]) if src_slots is not None else 0
    rc = _lib().ta_kv_page_evict(
        _ptr(k_pool), _ptr(v_pool), int(page_bytes), _ptr(host_k), _ptr(host_v), _ptr(src_slots), n,
        int(pool_pages), _ptr(staging),
        int(staging.numel() * staging.element_size()) if staging is not None else 0, _stream(stream))
    if check:
        _check(rc, "ta_kv_page_evict")
    return rc


def ta_kv_append(desc: Desc, new_k, new_v, cu_new_lens, k_pool, v_pool, block_table, context_lens,
                 total_new: int, stream=None, check: bool = True) -> int:
    d = desc.c()
    batch = int(context_lens.shape[0])
    stride = int(block_table.shape[1]) if block_table.dim() == 2 else 0
    rc = _lib().ta_kv_append(ctypes.byref(d), _ptr(new_k), _ptr(new_v), _ptr(cu_new_lens), _ptr(k_pool),
                             _ptr(v_pool), _ptr(block_table), stride, _ptr(context_lens), batch,
                             int(total_new), _stream(stream))
    if check:
        _check(rc, "ta_kv_append")
    return rc


def ta_profile_events(start_event, stop_event) -> None:
    """start/stop: raw hipEvent_t handles (ints) or None to switch recording off."""
    _lib().ta_profile_events(ctypes.c_void_p(start_event), ctypes.c_void_p(stop_event))


PROBE_FLOP_PER_ITER = 256.0 * 4.0 * 16.0 * 2.0 * 32.0 * 32.0 * 16.0
PROBE_SINK_BYTES = 256 * 256 * 4


def ta_matrix_core_probe(operands, iters: int, sink, stream=None, check: bool = True) -> int:
    """operands: 8192-byte device tensor of bf16 operand values; sink: PROBE_SINK_BYTES device bytes."""
    rc = _probe_lib().ta_matrix_core_probe(_ptr(operands), int(iters), _ptr(sink), _stream(stream))
    if check:
        _check(rc, "ta_matrix_core_probe")
    return rc


STREAM_SINK_BYTES = 8192 * 256 * 4
ISSUE_SINK_BYTES = 256 * 512 * 4


def ta_issue_port_probe(matrix_per_iter: int, vector_per_iter: int, iters: int, sink, stream=None, check: bool = True) -> int:
    """Two waves per SIMD issuing matrix and vector instructions side by side; sink: ISSUE_SINK_BYTES."""
    rc = _probe_lib().ta_issue_port_probe(int(matrix_per_iter), int(vector_per_iter), int(iters), _ptr(sink),
                                          _stream(stream))
    if check:
        _check(rc, "ta_issue_port_probe")
    return rc



def ta_stream_read_probe(src, sink, stream=None, check: bool = True) -> int:
    """src: device tensor whose bytes (a multiple of 16) are read once; sink: STREAM_SINK_BYTES."""
    rc = _probe_lib().ta_stream_read_probe(_ptr(src), int(src.numel() * src.element_size()), _ptr(sink),
                                     _stream(stream))
    if check:
        _check(rc, "ta_stream_read_probe")
    return rc


# ---- program-aware scheduling tick (host code) ----
PHASE_REASONING, PHASE_ACTING = 0, 1
STATUS_ACTIVE, STATUS_PAUSED, STATUS_TERMINATED = 0, 1, 2
# numpy layout of ta_program
PROGRAM_DTYPE = np.dtype([("id", "<i4"), ("context", "<i4"), ("backend", "<i4"), ("phase", "<i4"),
                          ("status", "<i4"), ("acting_time", "<f4")])


class SchedConfig(ctypes.Structure):
    _fields_ = [("capacity_tokens", ctypes.c_double), ("lambda_max", ctypes.c_double),
                ("lambda_min", ctypes.c_double), ("decay_base", ctypes.c_double)]


def ta_sched_tick(programs: np.ndarray, n_backends: int, capacity_tokens: float, lambda_max: float = 1.0,
                  lambda_min: float = 1.0, decay_base: float = 2.0, check: bool = True):
    """programs: C-contiguous array of PROGRAM_DTYPE, updated in place.
    Returns (status, paused ids, restored ids, restored backends) as numpy int32 arrays."""
    assert programs.dtype == PROGRAM_DTYPE and programs.flags["C_CONTIGUOUS"]
    n = int(programs.shape[0])
    cfg = SchedConfig(capacity_tokens, lambda_max, lambda_min, decay_base)
    paused = np.zeros(max(n, 1), np.int32)
    restored = np.zeros(max(n, 1), np.int32)
    backends = np.zeros(max(n, 1), np.int32)
    n_p, n_r = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = _lib().ta_sched_tick(ctypes.byref(cfg), programs.ctypes.data_as(ctypes.c_void_p), n, int(n_backends),
                              paused.ctypes.data_as(ctypes.c_void_p), ctypes.byref(n_p),
                              restored.ctypes.data_as(ctypes.c_void_p),
                              backends.ctypes.data_as(ctypes.c_void_p), ctypes.byref(n_r))
    if check:
        _check(rc, "ta_sched_tick")
    return rc, paused[: n_p.value], restored[: n_r.value], backends[: n_r.value]


# ---- trace-driven simulator of the policy (host code) ----
SIM_EVICT, SIM_EVICT_FORCED, SIM_RESTORE, SIM_PREFILL, SIM_DECODE, SIM_RELEASE = 1, 2, 3, 4, 5, 6
SIM_EVENT_DTYPE = np.dtype([("kind", "<i4"), ("program", "<i4"), ("backend", "<i4"), ("tokens", "<i4"),
                            ("context", "<i4"), ("first_slot", "<i4"), ("n_slots", "<i4")])


class SimConfig(ctypes.Structure):
    _fields_ = [("n_programs", ctypes.c_int32), ("n_backends", ctypes.c_int32), ("n_turns", ctypes.c_int32),
                ("pool_pages", ctypes.c_int32), ("steps_per_tick", ctypes.c_int32), ("max_context", ctypes.c_int32),
                ("time_per_tick", ctypes.c_double), ("sched", SchedConfig)]


class Sim:
    """Owner of a ta_sim handle: argument marshalling only, the decisions are the library's."""

    def __init__(self, n_backends: int, pool_pages: int, steps_per_tick: int, max_context: int, time_per_tick: float,
                 capacity_tokens: float, lambda_max: float, lambda_min: float, decay_base: float,
                 initial_context, turn_tokens, tool_ticks, tool_tokens):
        init = np.ascontiguousarray(initial_context, dtype=np.int32)
        arrays = [np.ascontiguousarray(a, dtype=np.int32) for a in (turn_tokens, tool_ticks, tool_tokens)]
        self.n_programs, self.n_turns = int(arrays[0].shape[0]), int(arrays[0].shape[1])
        cfg = SimConfig(self.n_programs, n_backends, self.n_turns, pool_pages, steps_per_tick, max_context,
                        time_per_tick, SchedConfig(capacity_tokens, lambda_max, lambda_min, decay_base))
        self._h = _lib().ta_sim_create(ctypes.byref(cfg), init.ctypes.data_as(ctypes.c_void_p),
                                       *[a.ctypes.data_as(ctypes.c_void_p) for a in arrays])
        if not self._h:
            raise TaError(TA_ERR_INVALID_ARG, "ta_sim_create")

    def close(self):
        if getattr(self, "_h", None):
            _lib().ta_sim_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: the library may already be gone
            pass

    def tick(self):
        """Advances one tick; returns (events as SIM_EVENT_DTYPE array, slots int32 array)."""
        n_e, n_s = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(_lib().ta_sim_tick(self._h, ctypes.byref(n_e), ctypes.byref(n_s)), "ta_sim_tick")
        events = np.zeros(n_e.value, SIM_EVENT_DTYPE)
        slots = np.zeros(max(n_s.value, 1), np.int32)
        _check(_lib().ta_sim_fetch(self._h, events.ctypes.data_as(ctypes.c_void_p),
                                   slots.ctypes.data_as(ctypes.c_void_p)), "ta_sim_fetch")
        return events, slots[: n_s.value]

    def programs(self) -> np.ndarray:
        out = np.zeros(self.n_programs, PROGRAM_DTYPE)
        _check(_lib().ta_sim_programs(self._h, out.ctypes.data_as(ctypes.c_void_p)), "ta_sim_programs")
        return out

    def page_table(self, program: int, max_pages: int = 1 << 16) -> np.ndarray:
        out = np.zeros(max_pages, np.int32)
        n = int(_lib().ta_sim_page_table(self._h, int(program), out.ctypes.data_as(ctypes.c_void_p), max_pages))
        if n < 0:
            raise TaError(TA_ERR_INVALID_ARG, "ta_sim_page_table")
        return out[:n]


def alloc_workspace(desc: Desc, batch: int, max_q_len: int, max_context_len: int, device="cuda"):
    """A uint8 device tensor of ta_workspace_bytes (torch's allocator aligns to 512 bytes)."""
    n = ta_workspace_bytes(desc, batch, max_q_len, max_context_len)
    if n == 0:
        raise TaError(TA_ERR_INVALID_ARG, "ta_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)
