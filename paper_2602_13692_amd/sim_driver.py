"""Carries out the simulator's events on real page pools with the library's device calls.

The decisions (who is paused, restored, which pages) are the library's (ta_sim_*, host code);
this module only turns each event into the call it stands for:

    EVICT / EVICT_FORCED  ta_kv_page_evict    pool pages -> the program's pinned host store
    RESTORE               ta_kv_page_restore  host store -> the pages named by the event
    PREFILL               ta_kv_append + ta_append_prefill of the tool output's tokens
    DECODE                ta_kv_append + ta_paged_decode, one batch per (decode step, backend)
    RELEASE               nothing on the device: the pages are simply free again

Every backend has its own K and V pool on the one GPU.  Token values (keys, values, queries) come
from a caller-supplied source, so that a test can keep its own record of what every program's
cache must hold.
"""
from __future__ import annotations

from typing import Callable, Dict, List

import numpy as np
import torch

from . import binding as ta

PAGE = 16
HEAD_DIM = 128


class Backends:
    def __init__(self, sim: ta.Sim, n_backends: int, pool_pages: int, num_q_heads: int, num_kv_heads: int,
                 max_context: int, initial_context, token_source: Callable, device="cuda:0",
                 kv_format: int = ta.KV_BF16, k_scale: float = 1.0, v_scale: float = 1.0):
        """token_source(program, first_token, n) -> (k, v, q): bf16 device tensors [n, Hkv, 128],
        [n, Hkv, 128], [n, Hq, 128] for the program's tokens first_token .. first_token + n - 1.
        With kv_format = KV_FP8_E4M3 the pools and the host stores hold E4M3 codes (one byte per
        element), written by the library's quantising append."""
        self.sim, self.dev = sim, device
        self.nb, self.P, self.Hq, self.Hkv = n_backends, pool_pages, num_q_heads, num_kv_heads
        self.max_pages = (max_context + PAGE - 1) // PAGE
        self.fp8 = kv_format == ta.KV_FP8_E4M3
        fmt = dict(kv_format=kv_format, k_scale=k_scale, v_scale=v_scale) if self.fp8 else {}
        pool_dtype = torch.uint8 if self.fp8 else torch.bfloat16
        self.page_bytes = num_kv_heads * PAGE * HEAD_DIM * (1 if self.fp8 else 2)
        self.desc = ta.Desc(num_q_heads, num_kv_heads, pool_pages=pool_pages, **fmt)
        self.source = token_source
        self.k_pool = [torch.zeros((pool_pages, num_kv_heads, PAGE, HEAD_DIM), dtype=pool_dtype, device=device)
                       for _ in range(n_backends)]
        self.v_pool = [torch.zeros_like(k) for k in self.k_pool]
        # a pool of one program's size: where an initial context is laid out before it goes to the host
        self._first_desc = ta.Desc(num_q_heads, num_kv_heads, pool_pages=self.max_pages, **fmt)
        self._first_k = torch.zeros((self.max_pages, num_kv_heads, PAGE, HEAD_DIM), dtype=pool_dtype, device=device)
        self._first_v = torch.zeros_like(self._first_k)
        n = len(initial_context)
        self.context = [int(c) for c in initial_context]
        self.table: List[List[int]] = [[] for _ in range(n)]       # pool pages of each program (empty while paused)
        self.backend = [-1] * n
        # the host side of Pause / Restore: one pinned store per program, page-major like the pool
        self.host_k = [torch.zeros((self.max_pages, self.page_bytes), dtype=torch.uint8).pin_memory() for _ in range(n)]
        self.host_v = [torch.zeros((self.max_pages, self.page_bytes), dtype=torch.uint8).pin_memory() for _ in range(n)]
        self.staging = torch.empty(2 * (16 << 20), dtype=torch.uint8, device=device)
        self.workspace = torch.empty(1 << 20, dtype=torch.uint8, device=device)
        self.gpu_ms: Dict[str, float] = {k: 0.0 for k in ("evict", "restore", "append", "prefill", "decode")}
        self.moved_bytes = {"evict": 0, "restore": 0}
        self.counts = {k: 0 for k in ("evict", "evict_forced", "restore", "prefill_tokens", "decode_tokens", "release")}
        self.last_decode = None     # (programs, out, lse) of the most recent decode batch, for checks
        self.last_prefill = None    # (programs, q_lens, out, lse) of the most recent prefill batch
        for p, c in enumerate(self.context):            # every program starts paused, its context on the host
            k, v, _ = self.source(p, 0, c)
            self._tokens_to_host(p, k, v, c)

    # ---- helpers ----
    def _tokens_to_host(self, p, k, v, c):
        """A program's first c tokens into its host store, the way they would have got there:
        appended to pages (quantised on the way into an FP8 cache), then evicted."""
        pages = (c + PAGE - 1) // PAGE
        if pages == 0:
            return
        self._first_k.zero_()
        self._first_v.zero_()
        table = torch.arange(pages, dtype=torch.int32, device=self.dev).view(1, pages)
        lens = torch.tensor([c], dtype=torch.int32, device=self.dev)
        cu = torch.tensor([0, c], dtype=torch.int32, device=self.dev)
        ta.ta_kv_append(self._first_desc, k.contiguous(), v.contiguous(), cu, self._first_k, self._first_v, table, lens, c)
        ta.ta_kv_page_evict(self._first_k, self._first_v, self.page_bytes, self.host_k[p][:pages], self.host_v[p][:pages],
                            torch.arange(pages, dtype=torch.int32), self.max_pages, self.staging)
        torch.cuda.synchronize()

    def _timed(self, kind, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        self.gpu_ms[kind] += e0.elapsed_time(e1)

    def _workspace(self, batch, max_q_len, longest):
        """The split-K plan depends on the batch and its longest context: size the buffer per call."""
        need = ta.ta_workspace_bytes(self.desc, batch, max_q_len, longest)
        if need > self.workspace.numel():
            self.workspace = torch.empty(2 * need, dtype=torch.uint8, device=self.dev)
        return self.workspace

    def _batch_tables(self, programs):
        width = max(len(self.table[p]) for p in programs)
        bt = np.full((len(programs), width), -1, np.int32)
        for i, p in enumerate(programs):
            bt[i, : len(self.table[p])] = self.table[p]
        lens = np.array([self.context[p] for p in programs], np.int32)
        return torch.from_numpy(bt).to(self.dev), torch.from_numpy(lens).to(self.dev), int(lens.max())

    def _grow_and_attend(self, b, programs, new_lens):
        """The programs (all on backend b) have grown by new_lens tokens: write the new tokens' K/V
        to the tail of their pages, then attend from them (decode if every growth is one token)."""
        ks, vs, qs = [], [], []
        for p, n in zip(programs, new_lens):
            k, v, q = self.source(p, self.context[p] - n, n)
            ks.append(k); vs.append(v); qs.append(q)
        new_k, new_v, q = torch.cat(ks), torch.cat(vs), torch.cat(qs)
        cu_np = np.zeros(len(programs) + 1, np.int32)
        np.cumsum(new_lens, out=cu_np[1:])
        cu = torch.from_numpy(cu_np).to(self.dev)
        total = int(cu_np[-1])
        bt, cl, longest = self._batch_tables(programs)
        out = torch.empty_like(q)
        lse = torch.empty((total, self.Hq), dtype=torch.float32, device=self.dev)
        kp, vp = self.k_pool[b], self.v_pool[b]
        self._timed("append", lambda: ta.ta_kv_append(self.desc, new_k, new_v, cu, kp, vp, bt, cl, total))
        if max(new_lens) == 1:
            ws = self._workspace(len(programs), 1, longest)
            self._timed("decode", lambda: ta.ta_paged_decode(self.desc, q, kp, vp, bt, cl, longest, out, lse, ws))
            self.counts["decode_tokens"] += total
            self.last_decode = (list(programs), out, lse)
        else:
            ws = self._workspace(len(programs), max(int(max(new_lens)), 2), longest)
            self._timed("prefill", lambda: ta.ta_append_prefill(self.desc, q, cu, kp, vp, bt, cl, total, int(max(new_lens)),
                                                                longest, out, lse, ws))
            self.counts["prefill_tokens"] += total
            self.last_prefill = (list(programs), list(new_lens), out, lse)

    # ---- one tick ----
    def run_tick(self):
        events, slots = self.sim.tick()
        self.sim_events = events
        i, n = 0, len(events)
        while i < n:
            e = events[i]
            kind, p, b = int(e["kind"]), int(e["program"]), int(e["backend"])
            mine = slots[int(e["first_slot"]): int(e["first_slot"]) + int(e["n_slots"])]
            if kind in (ta.SIM_EVICT, ta.SIM_EVICT_FORCED):
                src = torch.from_numpy(np.ascontiguousarray(mine))
                assert [int(s) for s in mine] == self.table[p]
                m = len(mine)
                self._timed("evict", lambda: ta.ta_kv_page_evict(self.k_pool[b], self.v_pool[b], self.page_bytes,
                                                                 self.host_k[p][:m], self.host_v[p][:m], src, self.P,
                                                                 self.staging))
                self.moved_bytes["evict"] += 2 * m * self.page_bytes
                self.counts["evict" if kind == ta.SIM_EVICT else "evict_forced"] += 1
                self.table[p], self.backend[p] = [], -1
                i += 1
            elif kind == ta.SIM_RESTORE:
                dst = torch.from_numpy(np.ascontiguousarray(mine))
                m = len(mine)
                self._timed("restore", lambda: ta.ta_kv_page_restore(self.k_pool[b], self.v_pool[b], self.page_bytes,
                                                                     self.host_k[p][:m], self.host_v[p][:m], dst, self.P,
                                                                     self.staging))
                self.moved_bytes["restore"] += 2 * m * self.page_bytes
                self.counts["restore"] += 1
                self.table[p], self.backend[p] = [int(s) for s in mine], b
                i += 1
            elif kind == ta.SIM_RELEASE:
                self.table[p], self.backend[p] = [], -1
                self.counts["release"] += 1
                i += 1
            else:
                # a run of PREFILL events, or of DECODE events of one step, on one backend: one batch
                step = int(e["tokens"]) if kind == ta.SIM_DECODE else -1
                programs, new_lens = [], []
                while i < n:
                    f = events[i]
                    same = int(f["kind"]) == kind and int(f["backend"]) == b and \
                        (kind == ta.SIM_PREFILL or int(f["tokens"]) == step)
                    if not same:
                        break
                    q = int(f["program"])
                    self.table[q] += [int(s) for s in slots[int(f["first_slot"]): int(f["first_slot"]) + int(f["n_slots"])]]
                    grown = int(f["context"]) - self.context[q]
                    self.context[q] = int(f["context"])
                    programs.append(q); new_lens.append(grown)
                    i += 1
                self._grow_and_attend(b, programs, new_lens)
        return events
