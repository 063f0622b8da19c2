#!/usr/bin/env python3
"""One-GPU benchmark of the paged-KV attention hot path on MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only decode|prefill|all] [--calibrate-copy]

A step is one ta_paged_decode call (work plan, the split-K kernel that streams
the chunks, merge) on the Llama-3-8B-shaped decode batch: 64 programs, 32 q / 8 kv heads, context
lengths uniform in 4k..32k, 16-token pages scattered over the pool by a seeded
permutation.  All inputs are resident in HBM before the timed region.  The
headline value is KV bytes read per second (K and V of every cached token once).

The same JSON line carries
  roofline      the streaming kernel's own duration (HIP events recorded inside
                the library around that kernel) against the 8 TB/s HBM peak;
  cpu_baseline  the fp64 oracle timed on this host's cores on the same batch;
  extra         the same batch on the vector-ALU kernel and over an FP8 cache,
                append-prefill (MFMA, TFLOP/s), forked-prefix decode,
                restore-then-decode (also: restore and evict on a second stream while
                the resident programs decode), restore against recompute, the policy
                simulator.
Other modes print a table of their own: --decode-sweep, --prefill-sweep, --crossover,
--schedule-demo.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16

# HBM bytes per launch of the kernel that streams the decode batch, from rocprofv3 --pmc
# (FETCH_SIZE + WRITE_SIZE, each scaled by the same counter on a 1 GiB device copy), keyed by the
# hash of the kernel source's code (comments aside) they were taken with.  A changed kernel gives
# null until the counters are taken again.
TRAFFIC_BYTES = {"bf4ede3c947c6fcb": 5081000000}
# The same batch on the vector-ALU kernel (the library's choice for smaller batches).
VECTOR_TRAFFIC_BYTES = {"3c00f0907d8a1e28": 5081000000}
# The same for the FP8-cache decode kernel.
FP8_TRAFFIC_BYTES = {"cd0f3df5654f75cc": 2554000000}
# The same for the append-prefill tile kernel: bytes that left the L2 per launch (FETCH_SIZE scaled).
PREFILL_TRAFFIC_BYTES = {"bf4ede3c947c6fcb": 16480000000}


def source_hash(name: str) -> str:
    """Hash of a kernel source's code: // comments and blank space do not count."""
    path = os.path.join(ROOT, "paper_2602_13692_amd", "csrc", name)
    code = []
    for line in open(path, encoding="utf-8"):
        line = line.split("//", 1)[0].strip()
        if line:
            code.append(" ".join(line.split()))
    return hashlib.sha256("\n".join(code).encode()).hexdigest()[:16]


def time_steps(fn, steps: int, warmup: int, torch):
    """W untimed steps, then exactly K steps between synchronisations; returns ms per step."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


class KernelTimer:
    """Per-step HIP event pairs recorded by the library around its dominant kernel."""

    def __init__(self, steps: int, torch, ta):
        self.torch, self.ta = torch, ta
        self.pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                      for _ in range(steps)]
        for a, b in self.pairs:      # the first record creates the underlying hipEvent_t
            a.record()
            b.record()
        torch.cuda.synchronize()
        self.i = 0

    def arm(self):
        a, b = self.pairs[self.i]
        self.ta.ta_profile_events(a.cuda_event, b.cuda_event)
        self.i += 1

    def disarm(self):
        self.ta.ta_profile_events(None, None)

    def times_ms(self):
        self.torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in self.pairs[: self.i]]

    def mean_ms(self) -> float:
        t = self.times_ms()
        return sum(t) / max(len(t), 1)


def run_decode(wb, steps, warmup, torch, ta, fp8_cache=None, chunk_pages=0, events_in_timed_steps=True):
    """Times ta_paged_decode on a batch; with fp8_cache (workloads.Fp8Cache) over its E4M3 codes.
    chunk_pages is the descriptor's decode_chunk_pages (0: the library chooses chunk and kernel).
    The library records HIP events around its dominant kernel inside every timed call; with
    events_in_timed_steps=False the calls are timed as a caller issues them and the events are
    taken in a second pass of the same steps (two event records between kernels cost a short call
    some microseconds)."""
    dev = wb.q.device
    if fp8_cache is None:
        desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads, decode_chunk_pages=chunk_pages)
        k_pool, v_pool = wb.k_pool, wb.v_pool
    else:
        desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads, kv_format=ta.KV_FP8_E4M3, k_scale=fp8_cache.k_scale,
                       v_scale=fp8_cache.v_scale)
        k_pool, v_pool = fp8_cache.k_codes, fp8_cache.v_codes
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    out = torch.empty_like(wb.q)
    lse = torch.empty((wb.batch, wb.num_q_heads), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, dev)
    timer = KernelTimer(steps, torch, ta)

    def step():
        ta.ta_paged_decode(desc, wb.q, k_pool, v_pool, bt, cl, wb.max_context_len, out, lse, ws)

    def timed_step():
        timer.arm()
        step()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        (timed_step if events_in_timed_steps else step)()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    if not events_in_timed_steps:
        for _ in range(steps):
            timed_step()
        torch.cuda.synchronize()
    timer.disarm()
    run_decode.last_kernel_times = sorted(timer.times_ms())
    return ms, timer.mean_ms(), out, lse


def run_prefill(wb, steps, warmup, torch, ta, fp8_cache=None):
    """Times ta_append_prefill on a batch; with fp8_cache (workloads.Fp8Cache) over its E4M3 codes."""
    dev = wb.q.device
    if fp8_cache is None:
        desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads)
        k_pool, v_pool = wb.k_pool, wb.v_pool
    else:
        desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads, kv_format=ta.KV_FP8_E4M3, k_scale=fp8_cache.k_scale,
                       v_scale=fp8_cache.v_scale)
        k_pool, v_pool = fp8_cache.k_codes, fp8_cache.v_codes
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    cu = torch.from_numpy(wb.cu_q_lens).to(dev)
    out = torch.empty_like(wb.q)
    lse = torch.empty((wb.total_q, wb.num_q_heads), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, max(wb.max_q_len, 2), wb.max_context_len, dev)
    timer = KernelTimer(steps, torch, ta)

    def step():
        ta.ta_append_prefill(desc, wb.q, cu, k_pool, v_pool, bt, cl, wb.total_q, wb.max_q_len,
                             wb.max_context_len, out, lse, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        timer.arm()
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    timer.disarm()
    return ms, timer.mean_ms(), out, lse


def cpu_model() -> str:
    """The host CPU's model string (first "model name" line of /proc/cpuinfo)."""
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def oracle_baseline(wb, wl):
    """The fp64 oracle as it stands, on this host's cores, on the whole decode batch."""
    import oracle

    q, kp, vp = wl.as_u16(wb.q), wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool)
    geom = oracle.Geometry(wb.num_q_heads, wb.num_kv_heads)
    t0 = time.perf_counter()
    out, lse = oracle.paged_decode(geom, q, kp, vp, wb.block_table, wb.context_lens)
    dt = time.perf_counter() - t0
    kv_bytes = int(wb.context_lens.astype("int64").sum()) * wb.kv_bytes_per_token
    return {
        "value": kv_bytes / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "cpu": cpu_model(),
        "kind": "oracle",
        "sample": f"all {wb.batch} programs x {wb.num_q_heads} query heads of the same batch, "
                  f"{dt:.2f} s wall",
    }, out, lse


def prefill_sample_check(wb, wl, out, lse, torch, rows_per_program: int = 48, n_programs: int = 6):
    """The oracle on a seeded sample of (new token, query head) rows of the prefill batch: parity of
    those rows, and the oracle's own rate on them (the whole batch would take it minutes)."""
    import numpy as np

    import oracle

    rng = np.random.default_rng(wl.SEED_BASE + 33)
    programs = sorted(rng.choice(wb.batch, size=n_programs, replace=False).tolist())
    # host copy of just the pages these programs name, block tables renumbered (input plumbing)
    remap, tables = {}, []
    for b in programs:
        npg = (int(wb.context_lens[b]) + wb.page_size - 1) // wb.page_size
        row = np.full(wb.block_table.shape[1], -1, dtype=np.int32)
        for i in range(npg):
            row[i] = remap.setdefault(int(wb.block_table[b, i]), len(remap))
        tables.append(row)
    idx = torch.from_numpy(np.array(list(remap.keys()), dtype=np.int64)).to(wb.k_pool.device)
    k_small, v_small = wl.as_u16(wb.k_pool.index_select(0, idx)), wl.as_u16(wb.v_pool.index_select(0, idx))
    cu = wb.cu_q_lens
    row_b, row_t, row_h, row_vis = [], [], [], []
    for local, b in enumerate(programs):
        n, L = int(wb.q_lens[b]), int(wb.context_lens[b])
        for i in [0, n - 1] + [int(x) for x in rng.integers(0, n, size=rows_per_program - 2)]:
            row_b.append(local); row_t.append(int(cu[b]) + i)
            row_h.append(int(rng.integers(0, wb.num_q_heads))); row_vis.append(L - n + i + 1)
    geom = oracle.Geometry(wb.num_q_heads, wb.num_kv_heads)
    t0 = time.perf_counter()
    ref, ref_lse = oracle.attend_rows(geom, wl.as_u16(wb.q), k_small, v_small, np.stack(tables),
                                      row_b, row_t, row_h, row_vis)
    dt = time.perf_counter() - t0
    t = torch.tensor(row_t, device=out.device)
    h = torch.tensor(row_h, device=out.device)
    check = spot_check(out[t, h], lse[t, h], ref, ref_lse, torch)
    check["rows_checked"] = len(row_t)
    flops = 4.0 * wb.head_dim * float(sum(row_vis))
    base = {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "cpu": cpu_model(), "kind": "oracle",
            "sample": f"{len(row_t)} (new token, query head) rows of {n_programs} programs, {dt:.2f} s wall"}
    return check, base


def spot_check(out, lse, ref_out, ref_lse, torch):
    import numpy as np

    got = out.float().cpu().numpy().astype("float64").reshape(ref_out.shape)
    err = np.abs(got - ref_out)
    ok = bool(np.all(err <= 2e-2 + 1e-2 * np.abs(ref_out)))
    lse_err = float(np.max(np.abs(lse.cpu().numpy().reshape(ref_lse.shape) - ref_lse)))
    return {"within_tolerance": ok, "max_abs_err": float(err.max()), "max_lse_err": lse_err}


def stream_read_gbps(torch, ta, buf, reps: int = 5) -> float:
    """Best of a few timed ta_stream_read_probe passes over `buf` (GB/s)."""
    sink = torch.empty(ta.STREAM_SINK_BYTES, dtype=torch.uint8, device=buf.device)
    ta.ta_stream_read_probe(buf, sink)
    torch.cuda.synchronize()
    best = 0.0
    nbytes = buf.numel() * buf.element_size()
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ta.ta_stream_read_probe(buf, sink)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, nbytes / e0.elapsed_time(e1) / 1e6)
    return best


def tiny_decode_latency(torch, ta, wl, dev, reps: int = 200):
    """Config 1 (4 programs, 960 cached tokens) is cache resident and launch bound: microseconds per call."""
    wb = wl.tiny_decode(dev)
    desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads)
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    out = torch.empty_like(wb.q)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, dev)

    def call(stream=None):
        ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, wb.max_context_len, out, None, ws, stream)

    eager_ms = time_steps(call, reps, 10, torch)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call(side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call(side)
    torch.cuda.synchronize()
    graph_ms = time_steps(graph.replay, reps, 10, torch)
    # what a replay costs on this runtime whatever it holds: a graph of one one-element fill kernel
    one = torch.zeros(1, device=dev)
    floor = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        one.fill_(1.0)
        side.synchronize()
        with torch.cuda.graph(floor, stream=side):
            one.fill_(1.0)
    torch.cuda.synchronize()
    floor_ms = time_steps(floor.replay, reps, 10, torch)
    fill_ms = time_steps(lambda: one.fill_(1.0), reps, 10, torch)
    return {"us_per_replay_of_a_graph_with_one_trivial_kernel": round(floor_ms * 1e3, 1),
            "us_per_trivial_kernel_launched_eagerly": round(fill_ms * 1e3, 1),
            "workload": "config 1: 4 programs, 8 q / 2 kv heads, contexts 64-512 (one kernel per call: every "
                        "context fits a single item, the chunk kernel writes the output itself)",
            "us_per_call_eager": round(eager_ms * 1e3, 1), "us_per_call_hip_graph": round(graph_ms * 1e3, 1)}


def matrix_core_sustained_tflops(torch, ta, dev, iters: int = 60000, operands: str = "normal") -> float:
    """Rate of ta_matrix_core_probe over roughly 20 ms on operands of one kind: N(0,1) in bf16 (what
    attention feeds the matrix cores), all zero, or all 1.0."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(260213692)
    if operands == "normal":
        ops = torch.randn(8 * 64 * 8, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    else:
        ops = torch.full((8 * 64 * 8,), 0.0 if operands == "zero" else 1.0, device=dev, dtype=torch.bfloat16)
    sink = torch.empty(ta.PROBE_SINK_BYTES, dtype=torch.uint8, device=dev)
    ta.ta_matrix_core_probe(ops, 1000, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ta.ta_matrix_core_probe(ops, iters, sink)
    e1.record()
    torch.cuda.synchronize()
    return ta.PROBE_FLOP_PER_ITER * iters / e0.elapsed_time(e1) / 1e9


def issue_port_ns(torch, ta, dev, iters: int = 20000):
    """ta_issue_port_probe: nanoseconds per iteration and SIMD (two waves, 16 matrix instructions and / or
    160 FMAs per iteration) for matrix only, vector only and both."""
    sink = torch.empty(ta.ISSUE_SINK_BYTES, dtype=torch.uint8, device=dev)
    out = {}
    for name, (nm, nv) in (("matrix_only", (8, 0)), ("vector_only", (0, 80)), ("both", (8, 80))):
        ta.ta_issue_port_probe(nm, nv, 1000, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ta.ta_issue_port_probe(nm, nv, iters, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(e0.elapsed_time(e1) * 1e6 / iters, 1)
    # time the vector port was unavailable per matrix instruction, as a share of that instruction's time
    out["vector_port_blocked_share_of_a_matrix_instruction"] = round(
        (out["both"] - out["vector_only"]) / max(out["matrix_only"], 1e-9), 3)
    return out


def crossover(torch, ta, wl, dev, contexts=(1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072)):
    """Restore against recompute for one program and one layer, context c = 1k .. 128k.

    Recompute is ta_append_prefill with an empty prefix (the attention part of re-prefilling the
    whole context, quadratic in c: a lower bound, the linear layers of a model come on top);
    restore is ta_kv_page_restore of the same c tokens from pinned host memory (linear in c).
    Small contexts are batched so the GPU is full; times are per program.
    """
    rows = []
    for c in contexts:
        batch = max(1, 16384 // c)
        wb = wl.append_prefill(dev, seed=wl.SEED_BASE + 60, batch=batch, new_lo=c, new_hi=c,
                               prefix_lo=0, prefix_hi=0)
        flops = 4.0 * wb.head_dim * wb.num_q_heads * wb.unmasked_pairs()
        ms, kernel_ms, out, lse = run_prefill(wb, 2 if c >= 65536 else 3, 1, torch, ta)
        del out, lse
        page_bytes = wb.num_kv_heads * wb.page_size * wb.head_dim * 2
        n = wb.pool_pages
        host_k = torch.empty((n, page_bytes), dtype=torch.uint8).pin_memory()
        host_v = torch.empty((n, page_bytes), dtype=torch.uint8).pin_memory()
        slots = torch.arange(n, dtype=torch.int32)
        staging = torch.empty(ta.ta_restore_staging_min_bytes(n) + 2 * (64 << 20), dtype=torch.uint8, device=dev)
        r_ms = time_steps(lambda: ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, host_k, host_v, slots,
                                                        wb.pool_pages, staging), 3, 1, torch)
        rows.append({"context": c, "programs": batch,
                     "recompute_attention_ms_per_program": round(ms / batch, 4),
                     "recompute_tflops": round(flops / ms / 1e9, 1),
                     "restore_ms_per_program": round(r_ms / batch, 4),
                     "restore_gbps": round(2.0 * n * page_bytes / r_ms / 1e6, 2),
                     "restore_over_recompute": round(r_ms / ms, 3)})
        del wb, host_k, host_v, staging
        torch.cuda.empty_cache()
    return rows


def decode_sweep(torch, ta, wl, dev, batches=(4, 8, 16, 32, 64, 128),
                 ranges=((1024, 4096), (4096, 16384), (16384, 65536)), chunks=(32, 64, 128, 256, 512, 0)):
    """ta_paged_decode (32 q / 8 kv heads) on batches of every size with the chunk length left to the
    library (0) and forced to every value: microseconds per call, best of three runs of twenty calls.
    Chunks of 256 and 512 pages run on the tile kernel, shorter ones on the vector-ALU kernel."""
    rows = []
    for batch in batches:
        for lo, hi in ranges:
            if batch * hi > 6_000_000:
                continue
            wb = wl.llama8b_decode(dev, seed=wl.SEED_BASE + 9, batch=batch, len_lo=lo, len_hi=hi)
            kv = int(wb.context_lens.astype("int64").sum()) * wb.kv_bytes_per_token
            bt = torch.from_numpy(wb.block_table).to(dev)
            cl = torch.from_numpy(wb.context_lens).to(dev)
            out = torch.empty_like(wb.q)
            us = {}
            for cp in chunks:
                desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads, decode_chunk_pages=cp)
                ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, dev)
                best = min(time_steps(lambda: ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl,
                                                                 wb.max_context_len, out, None, ws), 20, 6, torch)
                           for _ in range(3))
                us[cp] = best * 1e3
            forced = {cp: t for cp, t in us.items() if cp != 0}
            best_cp = min(forced, key=forced.get)
            rows.append({"programs": batch, "tokens": [lo, hi], "pages": int(((wb.context_lens + 15) // 16).sum()),
                         "us_library_choice": round(us[0], 1), "frac_of_hbm_peak": round(kv / us[0] / 1e3 / HBM_PEAK_GBPS, 3),
                         "best_forced_chunk_pages": best_cp, "us_best_forced": round(forced[best_cp], 1),
                         "library_over_best": round(us[0] / forced[best_cp], 3),
                         "us_by_forced_chunk_pages": {str(cp): round(t, 1) for cp, t in forced.items()}})
            del wb, out
            torch.cuda.empty_cache()
    return rows


def prefill_sweep(torch, ta, wl, dev,
                  shapes=((1, 1, 32768), (1, 16, 131072), (1, 64, 32768), (1, 256, 32768), (1, 1024, 32768),
                          (2, 128, 20000), (4, 64, 4096), (4, 256, 16384), (8, 64, 32768), (3, 200, 40000),
                          (6, 100, 12000), (10, 32, 24000), (5, 256, 20000), (12, 256, 16384), (8, 512, 16384),
                          (16, 256, 8192)),
                  chunk_counts=(0, 1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64)):
    """ta_append_prefill (32 q / 8 kv heads) of a few programs, each appending the same number of new
    tokens onto a cached prefix: microseconds per call, best of two runs of thirty calls, with the
    number of key chunks per query tile left to the library (0), switched off (1) and forced."""
    rows = []
    for batch, new, prefix in shapes:
        wb = wl.append_prefill(dev, seed=wl.SEED_BASE + 77, batch=batch, new_lo=new, new_hi=new,
                               prefix_lo=prefix, prefix_hi=prefix)
        flops = 4.0 * wb.head_dim * wb.num_q_heads * wb.unmasked_pairs()
        bt = torch.from_numpy(wb.block_table).to(dev)
        cl = torch.from_numpy(wb.context_lens).to(dev)
        cu = torch.from_numpy(wb.cu_q_lens).to(dev)
        out = torch.empty_like(wb.q)
        key_tiles = (wb.max_context_len + 63) // 64
        us = {}
        for n in chunk_counts:
            if n > 1 and (key_tiles // n < 4 or n * batch * ((new + 63) // 64) * wb.num_kv_heads > 4096):
                continue
            desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads, prefill_key_chunks=n)
            ws = ta.alloc_workspace(desc, wb.batch, max(wb.max_q_len, 2), wb.max_context_len, dev)
            us[n] = 1e3 * min(time_steps(lambda: ta.ta_append_prefill(desc, wb.q, cu, wb.k_pool, wb.v_pool, bt, cl,
                                                                       wb.total_q, wb.max_q_len, wb.max_context_len,
                                                                       out, None, ws), 30, 5, torch)
                              for _ in range(2))
            del ws
        forced = {n: t for n, t in us.items() if n != 0}
        best_n = min(forced, key=forced.get)
        rows.append({"programs": batch, "new_tokens": new, "cached_tokens": prefix,
                     "us_library_choice": round(us[0], 1), "tflops": round(flops / us[0] / 1e6, 1),
                     "us_uncut": round(us[1], 1), "best_forced_chunks": best_n,
                     "us_best_forced": round(forced[best_n], 1),
                     "library_over_best": round(us[0] / forced[best_n], 3),
                     "us_by_forced_chunks": {str(n): round(t, 1) for n, t in forced.items()}})
        del wb, out
        torch.cuda.empty_cache()
    return rows


def restore_while_decoding(wb, torch, ta, page_bytes, slots, back_k, back_v):
    """The restore of config 5 (and the eviction of the same pages: the Pause side) on one stream while
    the programs that stayed resident keep decoding on another (both at the default priority): what each
    loses to the other.  Decode steps are issued one at a time until the transfer's last event has
    passed; only steps that began and ended inside the transfer count."""
    import numpy as np

    dev = wb.q.device
    rs = wb.restore
    n = int(rs.dst_slots.shape[0])
    resident = np.setdiff1d(np.arange(wb.batch), rs.programs)
    idx = torch.from_numpy(resident).to(dev)
    q = wb.q[idx].contiguous()
    bt = torch.from_numpy(np.ascontiguousarray(wb.block_table[resident])).to(dev)
    cl = torch.from_numpy(np.ascontiguousarray(wb.context_lens[resident])).to(dev)
    max_len = int(wb.context_lens[resident].max())
    kv = int(wb.context_lens[resident].astype("int64").sum()) * wb.kv_bytes_per_token
    desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads)
    out = torch.empty_like(q)
    ws = ta.alloc_workspace(desc, len(resident), 1, max_len, dev)
    side = torch.cuda.Stream(device=dev)

    def decode(stream=None):
        ta.ta_paged_decode(desc, q, wb.k_pool, wb.v_pool, bt, cl, max_len, out, None, ws, stream)

    alone_ms = time_steps(decode, 10, 3, torch)
    res = {"resident_programs": int(len(resident)), "decode_ms_alone": round(alone_ms, 4),
           "decode_kv_gbps_alone": round(kv / alone_ms / 1e6, 1)}
    for what in ("restore", "evict"):
        for mode, nbytes in (("zero_copy", ta.ta_restore_staging_min_bytes(n)),
                             ("staged", ta.ta_restore_staging_min_bytes(n) + 2 * (256 << 20))):
            staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)

            def transfer(stream=None):
                if what == "restore":
                    ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, slots,
                                          wb.pool_pages, staging, stream)
                else:
                    ta.ta_kv_page_evict(wb.k_pool, wb.v_pool, page_bytes, back_k, back_v, slots, wb.pool_pages,
                                        staging, stream)

            transfer_alone_ms = time_steps(transfer, 2, 1, torch)
            torch.cuda.synchronize()
            r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            steps = []
            with torch.cuda.stream(side):
                r0.record(side)
                transfer(side)
                r1.record(side)
            while not r1.query() and len(steps) < 2000:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                decode()
                e1.record()
                e1.synchronize()
                steps.append((e0, e1))
            torch.cuda.synchronize()
            inside = [a.elapsed_time(b) for a, b in steps if r0.elapsed_time(a) >= 0.0 and b.elapsed_time(r1) >= 0.0]
            both_ms = r0.elapsed_time(r1)
            res[f"{what}_{mode}"] = {
                "ms_alone": round(transfer_alone_ms, 2), "ms_while_decoding": round(both_ms, 2),
                "decode_steps_inside": len(inside),
                "decode_ms_meanwhile": round(float(np.mean(inside)), 4) if inside else None,
                "decode_slowdown": round(float(np.mean(inside)) / alone_ms, 3) if inside else None,
                "transfer_slowdown": round(both_ms / transfer_alone_ms, 3)}
            del staging
    return res


def schedule_demo(torch, ta, wl, dev, decay_base: float, time_per_tick: float = 1.0, ticks: int = 48,
                  n_programs: int = 64, n_backends: int = 2, seed: int = 77, pool_tokens: int = 320 * 1024):
    """The policy simulator (ta_sim_*, host code) driving the kernels on a synthetic agent trace.

    Programs alternate reasoning turns (16 decode steps per tick, the context grows) and tool calls of
    heavy-tailed latency whose output is then appended and prefilled.  Every tick the simulator decides
    who keeps its pages on which backend; a paused program's pages go to pinned host memory
    (ta_kv_page_evict) and come back on restore (ta_kv_page_restore).  GPU time is split into
    productive (append, decode, prefill) and overhead (evict, restore), events around each call.
    """
    from paper_2602_13692_amd import sim_driver

    Hq, Hkv = 32, 8
    max_context = 32768 + 2048
    capacity = 0.85 * pool_tokens                      # C_total: the rest absorbs growth within a tick
    tr = wl.agent_trace(wl.SEED_BASE + seed, n_programs, n_turns=8, context_lo=4096, context_hi=20480, turn_lo=64,
                        turn_hi=256, tool_median_ticks=3.0, tool_sigma=1.0, out_lo=128, out_hi=1024)
    sim = ta.Sim(n_backends, pool_tokens // 16, 16, max_context, time_per_tick, capacity, 1.0, 1.0, decay_base,
                 tr.initial_context, tr.turn_tokens, tr.tool_ticks, tr.tool_tokens)

    def source(p, first, n):                           # values do not matter here, only shapes
        k = torch.empty((n, Hkv, 128), dtype=torch.bfloat16, device=dev).normal_()
        return k, torch.empty_like(k).normal_(), torch.empty((n, Hq, 128), dtype=torch.bfloat16, device=dev).normal_()

    drv = sim_driver.Backends(sim, n_backends, pool_tokens // 16, Hq, Hkv, max_context, tr.initial_context, source, dev)
    for _ in range(ticks):
        drv.run_tick()
    torch.cuda.synchronize()
    productive = drv.gpu_ms["append"] + drv.gpu_ms["decode"] + drv.gpu_ms["prefill"]
    overhead = drv.gpu_ms["evict"] + drv.gpu_ms["restore"]
    sim.close()
    return {"decay_base": decay_base, "time_per_tick": time_per_tick, "ticks": ticks, "programs": n_programs,
            "backends": n_backends, "capacity_tokens_per_backend": capacity, "events": drv.counts,
            "gpu_ms": {k: round(v, 2) for k, v in drv.gpu_ms.items()},
            "moved_gb": {k: round(v / 1e9, 2) for k, v in drv.moved_bytes.items()},
            "overhead_fraction_of_gpu_time": round(overhead / max(productive + overhead, 1e-9), 4),
            "decode_tokens_per_gpu_s": round(drv.counts["decode_tokens"] / max(productive + overhead, 1e-9) * 1e3, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--only", choices=["decode", "prefill", "all"], default="all")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--crossover", action="store_true",
                    help="print the restore-versus-recompute table (one JSON line) instead of the benchmark")
    ap.add_argument("--decode-sweep", action="store_true",
                    help="time ta_paged_decode on 4 to 128 programs with the library's own choice of kernel and chunk "
                         "and with every forced chunk length (one JSON line)")
    ap.add_argument("--prefill-sweep", action="store_true",
                    help="time ta_append_prefill of few programs with the library's number of key chunks and every forced one")
    ap.add_argument("--schedule-demo", action="store_true",
                    help="drive the kernels with the scheduling tick on a synthetic agent trace (one JSON line)")
    ap.add_argument("--kernels-only", action="store_true",
                    help="leave out the legs that run many small calls (restore-versus-recompute sweep, simulator) "
                         "and the append-prefill launch on all-zero operands: what a kernel trace of the five "
                         "workloads needs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (reference for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    from paper_2602_13692_amd import binding as ta
    from paper_2602_13692_amd import workloads as wl

    if not os.path.exists(ta.LIB_PATH):
        import __graft_entry__

        __graft_entry__.build()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.schedule_demo:
        print(json.dumps({"metric": "schedule_demo_one_backend_one_layer", "data": "synthetic",
                          "runs": [schedule_demo(torch, ta, wl, dev, base, dt)
                                   for base, dt in ((2.0, 1.0), (2.0, 0.25), (1.0, 1.0))]}), flush=True)
        return
    if args.decode_sweep:
        print(json.dumps({"metric": "paged_decode_route_and_chunk_sweep", "data": "synthetic",
                          "rows": decode_sweep(torch, ta, wl, dev)}), flush=True)
        return
    if args.prefill_sweep:
        print(json.dumps({"metric": "append_prefill_key_chunk_sweep", "data": "synthetic",
                          "rows": prefill_sweep(torch, ta, wl, dev)}), flush=True)
        return
    if args.crossover:
        print(json.dumps({"metric": "restore_vs_recompute_one_layer", "data": "synthetic",
                          "rows": crossover(torch, ta, wl, dev)}), flush=True)
        return

    # ---------------- headline: decode on the Llama-3-8B-shaped batch ----------------
    wb = wl.llama8b_decode(dev)
    kv_bytes = int(wb.context_lens.astype("int64").sum()) * wb.kv_bytes_per_token
    ms, kernel_ms, out, lse = run_decode(wb, args.steps, args.warmup, torch, ta)
    ktimes = run_decode.last_kernel_times
    stream_gbps = stream_read_gbps(torch, ta, wb.k_pool)
    value = kv_bytes / ms / 1e6
    achieved = kv_bytes / kernel_ms / 1e6
    traffic = TRAFFIC_BYTES.get(source_hash("ta_prefill.hip"))
    result = {
        "metric": "paged_decode_kv_gbps", "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "config 2: Llama-3-8B-shaped decode layer, 64 programs, 32 q / 8 kv heads, "
                        "d=128, page 16, context lengths uniform 4k-32k, seeded page permutation",
            "batch": wb.batch, "cached_tokens": int(wb.context_lens.sum()),
            "kv_bytes_per_step": kv_bytes, "layer_tokens_per_s": round(wb.batch / ms * 1e3, 1),
        },
        "roofline": {
            "bound": "hbm", "kernel": "attention_tile_kernel<4, true>", "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "kernel_ms": round(kernel_ms, 4), "kernel_ms_median": round(ktimes[len(ktimes) // 2], 4),
            "kernel_ms_min": round(ktimes[0], 4), "traffic": traffic,
            # what a kernel with the same load shape and no arithmetic reads per second in this run
            "stream_read_same_run_gbps": round(stream_gbps, 1),
            "frac_of_stream_read": round(achieved / stream_gbps, 4),
        },
    }
    if not args.no_cpu_baseline:
        base, ref_out, ref_lse = oracle_baseline(wb, wl)
        base["value"] = round(base["value"], 3)
        result["cpu_baseline"] = base
        result["config"]["parity_vs_oracle"] = spot_check(out, lse, ref_out, ref_lse, torch)
        del ref_out, ref_lse
    fp8_leg = None
    vector_leg = None
    if args.only in ("all", "decode"):
        # ---------------- the same batch on the vector-ALU kernel (a chunk size given by the caller keeps it there) ----
        v_ms, v_kernel_ms, _, _ = run_decode(wb, args.steps, args.warmup, torch, ta, chunk_pages=128)
        vector_leg = {
            "what": "config 2 streamed by decode_chunk_kernel<4, false> (decode_chunk_pages = 128): what the "
                    "library picks for batches too small to fill the tile kernel",
            "ms_per_step": round(v_ms, 4), "kv_gbps": round(kv_bytes / v_ms / 1e6, 1),
            "kernel_ms": round(v_kernel_ms, 4), "kernel_frac_of_hbm_peak": round(kv_bytes / v_kernel_ms / 1e6 / HBM_PEAK_GBPS, 4),
            "traffic": VECTOR_TRAFFIC_BYTES.get(source_hash("ta_decode.hip")),
        }
        # ---------------- the same batch with its cache as FP8 (E4M3) codes: half the bytes per token ----------------
        import oracle

        fc = wl.to_fp8_cache(wb)
        f_ms, f_kernel_ms, f_out, f_lse = run_decode(wb, args.steps, args.warmup, torch, ta, fp8_cache=fc)
        fp8_bytes = kv_bytes // 2
        fp8_leg = {
            "workload": "config 2 with the KV cache as E4M3 codes (2048 B per cached token and layer), scales "
                        f"k {fc.k_scale:.4g} / v {fc.v_scale:.4g}",
            "metric": "paged_decode_fp8_kv_gbps", "value": round(fp8_bytes / f_ms / 1e6, 1), "unit": "GB/s",
            "ms_per_step": round(f_ms, 4), "kv_bytes_per_step": fp8_bytes, "dtype": "fp8 e4m3 cache, bf16 q/out, f32 accumulate",
            "layer_tokens_per_s": round(wb.batch / f_ms * 1e3, 1),
            "roofline": {"bound": "hbm", "kernel": "decode_fp8_kernel<false, false>",
                         "achieved": round(fp8_bytes / f_kernel_ms / 1e6, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(fp8_bytes / f_kernel_ms / 1e6 / HBM_PEAK_GBPS, 4),
                         "kernel_ms": round(f_kernel_ms, 4),
                         "traffic": FP8_TRAFFIC_BYTES.get(source_hash("ta_decode_fp8.hip"))},
        }
        if not args.no_cpu_baseline:
            t0 = time.perf_counter()
            r_out, r_lse = oracle.paged_decode_fp8(oracle.Geometry(wb.num_q_heads, wb.num_kv_heads), wl.as_u16(wb.q),
                                                   wl.as_u8(fc.k_codes), wl.as_u8(fc.v_codes), fc.k_scale, fc.v_scale,
                                                   wb.block_table, wb.context_lens)
            dt = time.perf_counter() - t0
            fp8_leg["parity_vs_oracle"] = spot_check(f_out, f_lse, r_out, r_lse, torch)
            fp8_leg["cpu_baseline"] = {"value": round(fp8_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(),
                                       "cpu": cpu_model(), "kind": "oracle",
                                       "sample": f"all {wb.batch} programs x {wb.num_q_heads} query heads, {dt:.2f} s wall"}
            del r_out, r_lse
        del fc, f_out, f_lse
    if args.calibrate_copy:
        x = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        y = torch.empty_like(x)
        y.copy_(x)
        torch.cuda.synchronize()
        del x, y
    del wb, out, lse
    torch.cuda.empty_cache()

    extra = {}
    if vector_leg is not None:
        extra["decode_on_vector_alu_kernel"] = vector_leg
    if fp8_leg is not None:
        extra["fp8_decode"] = fp8_leg
    if args.only in ("all", "prefill"):
        # ---------------- append-prefill (MFMA) ----------------
        wb = wl.append_prefill(dev)
        flops = 4.0 * wb.head_dim * wb.num_q_heads * wb.unmasked_pairs()
        p_steps = max(2, min(args.steps, 5))
        ms, kernel_ms, out, lse = run_prefill(wb, p_steps, 1, torch, ta)
        extra["append_prefill"] = {
            "workload": "config 3: 64 programs append 256-2048 new tokens onto 8k-32k prefixes",
            "metric": "append_prefill_tflops", "value": round(flops / ms / 1e9, 1), "unit": "TFLOP/s",
            "ms_per_step": round(ms, 3), "steps": p_steps, "new_tokens": wb.total_q,
            "new_tokens_per_s": round(wb.total_q / ms * 1e3, 1), "flops_per_step": flops,
            "roofline": {"bound": "mfma", "kernel": "attention_tile_kernel<4, false>",
                         "achieved": round(flops / kernel_ms / 1e9, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": round(flops / kernel_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                         "kernel_ms": round(kernel_ms, 3),
                         "traffic": PREFILL_TRAFFIC_BYTES.get(source_hash("ta_prefill.hip"))},
        }
        if not args.no_cpu_baseline:
            check, base = prefill_sample_check(wb, wl, out, lse, torch)
            extra["append_prefill"]["parity_vs_oracle"] = check
            extra["append_prefill"]["cpu_baseline"] = base
        # writing the new tokens' K/V into their pages first (what a serving step does before this call)
        new_k = torch.empty((wb.total_q, wb.num_kv_heads, wb.head_dim), dtype=torch.bfloat16, device=dev).normal_()
        new_v = torch.empty_like(new_k).normal_()
        a_bt = torch.from_numpy(wb.block_table).to(dev)
        a_cl = torch.from_numpy(wb.context_lens).to(dev)
        a_cu = torch.from_numpy(wb.cu_q_lens).to(dev)
        a_desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads)
        a_ms = time_steps(lambda: ta.ta_kv_append(a_desc, new_k, new_v, a_cu, wb.k_pool, wb.v_pool, a_bt, a_cl,
                                                  wb.total_q), 5, 1, torch)
        moved = 2.0 * 2.0 * new_k.numel() * 2      # K and V, read once and written once
        extra["append_prefill"]["kv_append"] = {"ms": round(a_ms, 4), "bytes_read_plus_written": moved,
                                                "gbps": round(moved / a_ms / 1e6, 1)}
        # append-prefill over the same cache as E4M3 codes: one widening pass into the workspace (a bf16
        # copy of the batch's pages), then the same tile kernel
        fc3 = wl.to_fp8_cache(wb)
        f_ms, f_kernel_ms, f_out, _ = run_prefill(wb, 3, 1, torch, ta, fp8_cache=fc3)
        extra["append_prefill"]["fp8_cache"] = {
            "ms_per_step": round(f_ms, 3), "tflops": round(flops / f_ms / 1e9, 1), "tile_kernel_ms": round(f_kernel_ms, 3),
            "widening_pass_and_plan_ms": round(f_ms - f_kernel_ms, 3),
            "workspace_gb": round(ta.ta_workspace_bytes(ta.Desc(wb.num_q_heads, wb.num_kv_heads, kv_format=ta.KV_FP8_E4M3,
                                                                 k_scale=fc3.k_scale, v_scale=fc3.v_scale), wb.batch,
                                                        wb.max_q_len, wb.max_context_len) / 1e9, 2),
            "max_abs_diff_to_the_bf16_cache_result": round(float((f_out.float() - out.float()).abs().max()), 4),
        }
        del fc3, f_out
        torch.cuda.empty_cache()
        # the same tokens quantised into an FP8 cache of the same shape (bf16 rows in, E4M3 codes out)
        f_desc = ta.Desc(wb.num_q_heads, wb.num_kv_heads, kv_format=ta.KV_FP8_E4M3, k_scale=0.021, v_scale=0.017)
        k8 = torch.zeros(wb.k_pool.shape, dtype=torch.uint8, device=dev)
        v8 = torch.zeros_like(k8)
        f_ms = time_steps(lambda: ta.ta_kv_append(f_desc, new_k, new_v, a_cu, k8, v8, a_bt, a_cl, wb.total_q), 5, 1, torch)
        moved8 = 2.0 * new_k.numel() * (2 + 1)      # K and V: two bytes read, one written per element
        extra["append_prefill"]["kv_append_fp8"] = {"ms": round(f_ms, 4), "bytes_read_plus_written": moved8,
                                                    "gbps": round(moved8 / f_ms / 1e6, 1)}
        del new_k, new_v, k8, v8
        # What the matrix cores sustain on operands of the same kind (N(0,1) in bf16) when they do
        # nothing else: under such a load the power management, not the nominal clock, sets the rate.
        sustained = matrix_core_sustained_tflops(torch, ta, dev)
        extra["append_prefill"]["matrix_cores_alone_same_operand_kind_tflops"] = round(sustained, 1)
        extra["append_prefill"]["frac_of_matrix_cores_alone"] = round(flops / kernel_ms / 1e9 / sustained, 4)
        # the same probe on operands that toggle no bits: the gap to the N(0,1) rate is the power management's
        extra["append_prefill"]["matrix_cores_alone_tflops_by_operand_kind"] = {
            "normal": round(sustained, 1),
            "zero": round(matrix_core_sustained_tflops(torch, ta, dev, operands="zero"), 1),
            "one": round(matrix_core_sustained_tflops(torch, ta, dev, operands="one"), 1)}
        # do matrix and vector instructions of two waves overlap on a SIMD?
        extra["append_prefill"]["issue_port_probe_ns_per_iteration"] = issue_port_ns(torch, ta, dev)
        # the same batch with every block table folded onto 64 pages: K and V never leave the L2
        import numpy as np

        folded = wb.block_table.copy()
        folded[folded >= 0] %= 64
        keep = wb.block_table
        wb.block_table = folded
        _, hot_ms, _, _ = run_prefill(wb, 3, 1, torch, ta)
        wb.block_table = keep
        extra["append_prefill"]["kernel_ms_with_kv_always_in_l2"] = round(hot_ms, 3)
        # the same launch on operands that toggle no bits (Q, K and V all zero): the instruction stream is
        # the same, so what separates the two times is the clock that the power management allows
        # (left out of a kernel trace, where it would be averaged with the launches on the real batch)
        if not args.kernels_only:
            wb.q.zero_()
            wb.k_pool.zero_()
            wb.v_pool.zero_()
            _, zero_ms, _, _ = run_prefill(wb, 3, 2, torch, ta)
            extra["append_prefill"]["kernel_ms_on_all_zero_operands"] = round(zero_ms, 3)
            extra["append_prefill"]["frac_of_peak_on_all_zero_operands"] = round(
                flops / zero_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)
        del wb, out, lse
        torch.cuda.empty_cache()

    if args.only == "all":
        # ---------------- the tiny configuration: latency of one call, eager and from a HIP graph ----------------
        extra["tiny_decode"] = tiny_decode_latency(torch, ta, wl, dev)

        # ---------------- forked programs with shared prefixes ----------------
        wb = wl.forked_decode(dev)
        logical = int(wb.context_lens.astype("int64").sum()) * wb.kv_bytes_per_token
        unique = wb.unique_tokens() * wb.kv_bytes_per_token
        f_steps = max(2, min(args.steps, 50))
        # (the legs before this one leave the GPU in a low-power state: a longer warm-up than elsewhere)
        ms, kernel_ms, out, lse = run_decode(wb, f_steps, 60, torch, ta, events_in_timed_steps=False)
        ms_ev, _, out, lse = run_decode(wb, f_steps, 5, torch, ta)
        extra["forked_decode"] = {
            "workload": "config 4: 256 programs, 64 q / 8 kv heads, groups of 16 share a 16k prefix",
            "ms_per_step": round(ms, 4), "logical_kv_gbps": round(logical / ms / 1e6, 1),
            "unique_kv_gbps": round(unique / ms / 1e6, 1),
            "frac_of_unique_bytes_roofline": round(unique / ms / 1e6 / HBM_PEAK_GBPS, 4),
            "dominant_kernel_ms": round(kernel_ms, 4),
            "ms_per_step_with_event_records_inside_the_call": round(ms_ev, 4),
        }
        # the same batch over an FP8 cache: shared chunks go through the FP8 kernel, four programs (32
        # query heads) per workgroup
        fc4 = wl.to_fp8_cache(wb)
        f8_ms, f8_kernel_ms, _, _ = run_decode(wb, f_steps, 5, torch, ta, fp8_cache=fc4, events_in_timed_steps=False)
        extra["forked_decode"]["fp8_cache"] = {
            "ms_per_step": round(f8_ms, 4), "unique_kv_gbps_of_2048_B_per_token": round(unique / 2 / f8_ms / 1e6, 1),
            "private_chunks_kernel_ms": round(f8_kernel_ms, 4)}
        del fc4
        torch.cuda.empty_cache()
        # the same batch with its programs in shuffled order: the groups are found all the same
        import numpy as np

        perm = np.random.default_rng(wl.SEED_BASE + 44).permutation(wb.batch)
        wb.q = wb.q[torch.from_numpy(perm).to(dev)].contiguous()
        wb.block_table = np.ascontiguousarray(wb.block_table[perm])
        wb.context_lens = np.ascontiguousarray(wb.context_lens[perm])
        ms_shuffled, _, out, lse = run_decode(wb, f_steps, 5, torch, ta, events_in_timed_steps=False)
        extra["forked_decode"]["ms_per_step_shuffled_batch_order"] = round(ms_shuffled, 4)
        del wb, out, lse
        torch.cuda.empty_cache()

        # ---------------- restore from pinned host memory, then decode ----------------
        wb = wl.long_horizon_restore(dev)
        rs = wb.restore
        page_bytes = wb.num_kv_heads * wb.page_size * wb.head_dim * 2
        n = int(rs.dst_slots.shape[0])
        slots = torch.from_numpy(rs.dst_slots.copy())
        res = {}
        for mode, nbytes in (("zero_copy", ta.ta_restore_staging_min_bytes(n)),
                             ("staged", ta.ta_restore_staging_min_bytes(n) + 2 * (256 << 20))):
            staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)

            def step():
                ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, slots,
                                      wb.pool_pages, staging)

            r_ms = time_steps(step, 3, 1, torch)
            res[mode] = {"ms": round(r_ms, 2), "gbps": round(2.0 * n * page_bytes / r_ms / 1e6, 2)}
            del staging
        # the link roofline: one large pinned host-to-device copy of the same bytes
        big = torch.empty_like(rs.host_k, device=dev)
        link_ms = time_steps(lambda: big.copy_(rs.host_k, non_blocking=True), 3, 1, torch)
        link_gbps = n * page_bytes / link_ms / 1e6
        # the Pause side: the same pages leave the pool for pinned host memory
        back_k, back_v = torch.empty_like(rs.host_k).pin_memory(), torch.empty_like(rs.host_v).pin_memory()
        ev = {}
        for mode, nbytes in (("zero_copy", ta.ta_restore_staging_min_bytes(n)),
                             ("staged", ta.ta_restore_staging_min_bytes(n) + 2 * (256 << 20))):
            staging = torch.empty(nbytes, dtype=torch.uint8, device=dev)

            def evict_step():
                ta.ta_kv_page_evict(wb.k_pool, wb.v_pool, page_bytes, back_k, back_v, slots,
                                    wb.pool_pages, staging)

            e_ms = time_steps(evict_step, 3, 1, torch)
            ev[mode] = {"ms": round(e_ms, 2), "gbps": round(2.0 * n * page_bytes / e_ms / 1e6, 2)}
            del staging
        d2h_ms = time_steps(lambda: back_k.copy_(big, non_blocking=True), 3, 1, torch)
        d2h_gbps = n * page_bytes / d2h_ms / 1e6
        overlapped = (None if args.kernels_only
                      else restore_while_decoding(wb, torch, ta, page_bytes, slots, back_k, back_v))
        del big, back_k, back_v
        kv5 = int(wb.context_lens.astype("int64").sum()) * wb.kv_bytes_per_token
        ms, kernel_ms, out, lse = run_decode(wb, max(2, min(args.steps, 10)), 2, torch, ta)
        best = min(res.values(), key=lambda r: r["ms"])
        extra["restore_then_decode"] = {
            "workload": "config 5: 128 programs, lognormal lengths (median 24k, cap 128k), 30% restored "
                        "from pinned host memory into random free slots, then one decode",
            "restored_pages": n, "restored_bytes": 2 * n * page_bytes, "restore": res,
            "host_link_h2d_gbps": round(link_gbps, 2),
            "restore_frac_of_link": round(best["gbps"] / link_gbps, 3),
            "evict": ev, "host_link_d2h_gbps": round(d2h_gbps, 2),
            "evict_frac_of_link": round(max(r["gbps"] for r in ev.values()) / d2h_gbps, 3),
            "decode_ms": round(ms, 4), "decode_kv_gbps": round(kv5 / ms / 1e6, 1),
            "decode_kernel_frac_of_hbm_peak": round(kv5 / kernel_ms / 1e6 / HBM_PEAK_GBPS, 4),
            "restore_to_decode_time_ratio": round(best["ms"] / ms, 1),
            "transfers_while_resident_programs_decode": overlapped,
        }
        del wb, out, lse
        torch.cuda.empty_cache()
    if args.only == "all" and not args.kernels_only:
        # ---------------- restore against recompute (short sweep; --crossover runs 1k .. 128k) ----------------
        extra["restore_vs_recompute"] = {
            "what": "one program, one layer: ta_append_prefill with an empty prefix (attention part of a re-prefill, "
                    "quadratic in the context) against ta_kv_page_restore of the same context (linear)",
            "rows": crossover(torch, ta, wl, dev, contexts=(2048, 8192, 32768))}
        # ---------------- the policy simulator driving the kernels (short run; --schedule-demo compares decays) ------
        extra["scheduler_sim"] = schedule_demo(torch, ta, wl, dev, 2.0, 0.25, ticks=24, n_programs=32, n_backends=2,
                                               pool_tokens=128 * 1024)
    result["extra"] = extra
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
