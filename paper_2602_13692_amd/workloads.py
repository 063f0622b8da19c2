"""Seeded synthetic inputs shaped like agentic serving workloads.

The paper (ThunderAgent, Sec. 5.1) measures on agent traces with 48-192
concurrent long-lived programs whose contexts only grow (Sec. 2.1), that share
a system prompt (Sec. 4.3) and that are restored from host memory under
offloading (App. A.4).  Those traces are not available; the batches built here
stand in for the shapes they induce: many programs, ragged context lengths of
thousands to tens of thousands of tokens, 16-token pages scattered over a pool
in random order, shared prefix pages, and a restore set held in pinned host
memory.

This module holds NO attention arithmetic.  It draws integers (lengths, page
permutations, restore sets) from numpy's PCG64 and values from torch's seeded
normal generator, and is the only module used both by the GPU path's callers
and by the oracle's callers.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

SEED_BASE = 260213692
HEAD_DIM = 128
PAGE_SIZE = 16


@dataclass
class RestoreSet:
    """Pages that start in pinned host memory and must be scattered into the pool."""

    programs: np.ndarray            # int32 [n_prog] programs whose pages are on the host
    dst_slots: np.ndarray           # int32 [n] destination pool slots, distinct
    host_k: torch.Tensor            # bf16 [n, Hkv, page, d], pinned when a GPU is used
    host_v: torch.Tensor


@dataclass
class PagedBatch:
    """One batch of programs over a shared page pool.

    q is packed [total_q, Hq, d]; for decode total_q == batch and q_lens is all
    ones.  block_table entries beyond ceil(context_len / page) are -1.
    """

    name: str
    num_q_heads: int
    num_kv_heads: int
    context_lens: np.ndarray        # int32 [B]
    q_lens: np.ndarray              # int32 [B]
    block_table: np.ndarray         # int32 [B, stride]
    pool_pages: int
    unique_pages: int               # distinct pages the block tables name
    q: torch.Tensor                 # bf16 [total_q, Hq, d]
    k_pool: torch.Tensor            # bf16 [P, Hkv, page, d]
    v_pool: torch.Tensor
    head_dim: int = HEAD_DIM
    page_size: int = PAGE_SIZE
    restore: Optional[RestoreSet] = None
    notes: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return int(self.context_lens.shape[0])

    @property
    def cu_q_lens(self) -> np.ndarray:
        cu = np.zeros(self.batch + 1, dtype=np.int32)
        np.cumsum(self.q_lens, out=cu[1:])
        return cu

    @property
    def total_q(self) -> int:
        return int(self.q_lens.sum())

    @property
    def max_context_len(self) -> int:
        return int(self.context_lens.max()) if self.batch else 0

    @property
    def max_q_len(self) -> int:
        return int(self.q_lens.max()) if self.batch else 0

    @property
    def kv_bytes_per_token(self) -> int:
        """K plus V bytes of one cached token over all kv heads (bf16)."""
        return 2 * self.num_kv_heads * self.head_dim * 2

    def unique_tokens(self) -> int:
        """Cached tokens counted once even when several block tables name their page."""
        seen = {}
        total = 0
        ps = self.page_size
        for b in range(self.batch):
            L = int(self.context_lens[b])
            npages = (L + ps - 1) // ps
            for i in range(npages):
                page = int(self.block_table[b, i])
                rows = min(ps, L - i * ps)
                if seen.get(page, 0) < rows:
                    total += rows - seen.get(page, 0)
                    seen[page] = rows
        return total

    def unmasked_pairs(self) -> int:
        """(query token, key) pairs that attention evaluates, per query head."""
        total = 0
        for b in range(self.batch):
            L, n = int(self.context_lens[b]), int(self.q_lens[b])
            p = L - n
            total += n * p + n * (n + 1) // 2
        return total


# --------------------------------------------------------------------------
# value and structure generators
# --------------------------------------------------------------------------

def normal_bf16(shape, seed: int, device, pin: bool = False, chunk_elems: int = 1 << 28) -> torch.Tensor:
    """i.i.d. N(0,1) rounded to bf16, drawn on `device` from a seeded generator.

    With pin=True the result is a pinned host tensor filled through the device.
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    numel = int(np.prod(shape)) if len(shape) else 1
    if pin and device.type == "cuda":
        host = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
        flat = host.view(-1)
        for lo in range(0, numel, chunk_elems):
            hi = min(numel, lo + chunk_elems)
            tmp = torch.empty(hi - lo, dtype=torch.bfloat16, device=device)
            tmp.normal_(generator=gen)
            flat[lo:hi].copy_(tmp)
        torch.cuda.synchronize(device)
        return host
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    for lo in range(0, numel, chunk_elems):
        hi = min(numel, lo + chunk_elems)
        flat[lo:hi].normal_(generator=gen)
    return out


def pages_of(lengths: np.ndarray, page_size: int = PAGE_SIZE) -> np.ndarray:
    return (np.asarray(lengths, dtype=np.int64) + page_size - 1) // page_size


def scatter_tables(rng: np.random.Generator, n_pages: np.ndarray, slots: np.ndarray,
                   stride: Optional[int] = None) -> np.ndarray:
    """Give program b its n_pages[b] pages from `slots` (already in random order)."""
    B = int(n_pages.shape[0])
    width = int(n_pages.max()) if B else 0
    stride = max(width, 1) if stride is None else stride
    table = np.full((B, stride), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        k = int(n_pages[b])
        table[b, :k] = slots[off:off + k]
        off += k
    return table


def _finish(name, Hq, Hkv, context_lens, q_lens, table, pool_pages, seed, device,
            restore=None, notes=None) -> PagedBatch:
    context_lens = np.asarray(context_lens, dtype=np.int32)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    total_q = int(q_lens.sum())
    q = normal_bf16((total_q, Hq, HEAD_DIM), seed * 16 + 1, device)
    k_pool = normal_bf16((pool_pages, Hkv, PAGE_SIZE, HEAD_DIM), seed * 16 + 2, device)
    v_pool = normal_bf16((pool_pages, Hkv, PAGE_SIZE, HEAD_DIM), seed * 16 + 3, device)
    used = table[table >= 0]
    return PagedBatch(
        name=name, num_q_heads=Hq, num_kv_heads=Hkv, context_lens=context_lens, q_lens=q_lens,
        block_table=table, pool_pages=int(pool_pages), unique_pages=int(np.unique(used).size),
        q=q, k_pool=k_pool, v_pool=v_pool, restore=restore, notes=notes or {},
    )


# --------------------------------------------------------------------------
# the five configurations; every size is a parameter so tests can shrink them
# --------------------------------------------------------------------------

def tiny_decode(device="cpu", seed: int = SEED_BASE + 1) -> PagedBatch:
    """4 programs, 8 q / 2 kv heads, lengths 64..512, 60 pages shuffled into a 64-page pool."""
    rng = np.random.default_rng(seed)
    lens = np.array([64, 128, 256, 512], dtype=np.int32)
    pool_pages = 64
    slots = rng.permutation(pool_pages).astype(np.int32)
    table = scatter_tables(rng, pages_of(lens), slots)
    return _finish("tiny_decode", 8, 2, lens, np.ones(4, np.int32), table, pool_pages, seed, device)


def llama8b_decode(device="cpu", seed: int = SEED_BASE + 2, batch: int = 64,
                   len_lo: int = 4096, len_hi: int = 32768,
                   num_q_heads: int = 32, num_kv_heads: int = 8, first_lens=()) -> PagedBatch:
    """Decode layer, lengths uniform in [len_lo, len_hi], pool sized to fit all pages.

    first_lens overrides the lengths of the first programs (edge cases in tests).
    """
    rng = np.random.default_rng(seed)
    lens = rng.integers(len_lo, len_hi + 1, size=batch).astype(np.int32)
    lens[:len(first_lens)] = np.asarray(first_lens, dtype=np.int32)
    n_pages = pages_of(lens)
    pool_pages = int(n_pages.sum())
    slots = rng.permutation(pool_pages).astype(np.int32)
    table = scatter_tables(rng, n_pages, slots)
    return _finish("llama8b_decode", num_q_heads, num_kv_heads, lens, np.ones(batch, np.int32),
                   table, pool_pages, seed, device)


def append_prefill(device="cpu", seed: int = SEED_BASE + 3, batch: int = 64,
                   new_lo: int = 256, new_hi: int = 2048,
                   prefix_lo: int = 8192, prefix_hi: int = 32768,
                   num_q_heads: int = 32, num_kv_heads: int = 8) -> PagedBatch:
    """Each program appends n new tokens causally onto a retained prefix."""
    rng = np.random.default_rng(seed)
    n_new = rng.integers(new_lo, new_hi + 1, size=batch).astype(np.int32)
    prefix = rng.integers(prefix_lo, prefix_hi + 1, size=batch).astype(np.int32)
    lens = (prefix + n_new).astype(np.int32)
    n_pages = pages_of(lens)
    pool_pages = int(n_pages.sum())
    slots = rng.permutation(pool_pages).astype(np.int32)
    table = scatter_tables(rng, n_pages, slots)
    return _finish("append_prefill", num_q_heads, num_kv_heads, lens, n_new, table, pool_pages,
                   seed, device)


def forked_decode(device="cpu", seed: int = SEED_BASE + 4, batch: int = 256, group: int = 16,
                  prefix_len: int = 16384, suffix_lo: int = 1024, suffix_hi: int = 4096,
                  num_q_heads: int = 64, num_kv_heads: int = 8) -> PagedBatch:
    """Groups of programs whose block tables begin with the same prefix pages."""
    assert batch % group == 0 and prefix_len % PAGE_SIZE == 0
    rng = np.random.default_rng(seed)
    n_groups = batch // group
    suffix = rng.integers(suffix_lo, suffix_hi + 1, size=batch).astype(np.int32)
    lens = (prefix_len + suffix).astype(np.int32)
    prefix_pages = prefix_len // PAGE_SIZE
    suffix_pages = pages_of(suffix)
    pool_pages = int(n_groups * prefix_pages + suffix_pages.sum())
    slots = rng.permutation(pool_pages).astype(np.int32)
    stride = int(prefix_pages + suffix_pages.max())
    table = np.full((batch, stride), -1, dtype=np.int32)
    off = 0
    for g in range(n_groups):
        shared = slots[off:off + prefix_pages]
        off += prefix_pages
        for m in range(group):
            b = g * group + m
            table[b, :prefix_pages] = shared
            k = int(suffix_pages[b])
            table[b, prefix_pages:prefix_pages + k] = slots[off:off + k]
            off += k
    return _finish("forked_decode", num_q_heads, num_kv_heads, lens, np.ones(batch, np.int32),
                   table, pool_pages, seed, device,
                   notes={"group": group, "prefix_len": prefix_len})


def long_horizon_restore(device="cpu", seed: int = SEED_BASE + 5, batch: int = 128,
                         median: int = 24576, sigma: float = 0.75, len_lo: int = 1024,
                         len_cap: int = 131072, restore_frac: float = 0.3, slack: float = 0.10,
                         num_q_heads: int = 32, num_kv_heads: int = 8) -> PagedBatch:
    """Lognormal context lengths; a fraction of programs starts in pinned host memory.

    The block tables already point at the destination slots of the programs to
    be restored; until the restore runs those slots hold unrelated values.
    """
    rng = np.random.default_rng(seed)
    raw = np.exp(rng.normal(math.log(median), sigma, size=batch))
    lens = np.clip(np.rint(raw), len_lo, len_cap).astype(np.int32)
    n_pages = pages_of(lens)
    pool_pages = int(math.ceil(n_pages.sum() * (1.0 + slack)))
    n_restore = int(round(restore_frac * batch))
    evicted = np.sort(rng.choice(batch, size=n_restore, replace=False)).astype(np.int32)
    is_evicted = np.zeros(batch, dtype=bool)
    is_evicted[evicted] = True
    slots = rng.permutation(pool_pages).astype(np.int32)
    # resident programs take slots first; the restored ones draw from what is left free
    table = np.full((batch, int(n_pages.max())), -1, dtype=np.int32)
    off = 0
    for b in np.flatnonzero(~is_evicted):
        k = int(n_pages[b])
        table[b, :k] = slots[off:off + k]
        off += k
    free = slots[off:]
    n_dst = int(n_pages[evicted].sum())
    dst = rng.choice(free, size=n_dst, replace=False).astype(np.int32)
    off = 0
    for b in evicted:
        k = int(n_pages[b])
        table[b, :k] = dst[off:off + k]
        off += k
    pin = torch.device(device).type == "cuda"
    host_k = normal_bf16((n_dst, num_kv_heads, PAGE_SIZE, HEAD_DIM), seed * 16 + 4, device, pin=pin)
    host_v = normal_bf16((n_dst, num_kv_heads, PAGE_SIZE, HEAD_DIM), seed * 16 + 5, device, pin=pin)
    if not pin:
        host_k, host_v = host_k.cpu(), host_v.cpu()
    restore = RestoreSet(programs=evicted, dst_slots=dst, host_k=host_k, host_v=host_v)
    return _finish("long_horizon_restore", num_q_heads, num_kv_heads, lens,
                   np.ones(batch, np.int32), table, pool_pages, seed, device, restore=restore)


# --------------------------------------------------------------------------
# adversarial edits of a batch (inputs only)
# --------------------------------------------------------------------------

def poison_padding(wb: PagedBatch) -> None:
    """NaN in every pool row no block table can legally read.

    That is: rows of a program's last page beyond its context length (unless
    another program reads them) and pages no block table names.
    """
    ps = wb.page_size
    readable = np.zeros((wb.pool_pages,), dtype=np.int32)  # rows legally read per page
    for b in range(wb.batch):
        L = int(wb.context_lens[b])
        npages = (L + ps - 1) // ps
        for i in range(npages):
            page = int(wb.block_table[b, i])
            readable[page] = max(readable[page], min(ps, L - i * ps))
    rows = torch.arange(ps).view(1, ps)
    mask = rows >= torch.from_numpy(readable).view(-1, 1)            # [P, ps] True = poison
    mask = mask.to(wb.k_pool.device).view(wb.pool_pages, 1, ps, 1)
    nan = torch.tensor(float("nan"), dtype=torch.bfloat16, device=wb.k_pool.device)
    wb.k_pool.copy_(torch.where(mask, nan, wb.k_pool))
    wb.v_pool.copy_(torch.where(mask, nan, wb.v_pool))


def plant_needles(wb: PagedBatch, seed: int, strength: float = 30.0) -> np.ndarray:
    """Make one key per (program, kv head) dominate the softmax of one query head.

    For the first query head of every kv-head group (decode batches only) one
    cached key at a random position is overwritten with strength*sqrt(d)*q/|q|^2,
    so its score is about `strength` and the output is close to that token's value
    row, of magnitude O(1).  Returns int64 [B, Hkv] positions.  Pages shared
    between programs are skipped (position -1).
    """
    assert wb.total_q == wb.batch
    rng = np.random.default_rng(seed)
    group = wb.num_q_heads // wb.num_kv_heads
    ps = wb.page_size
    counts = np.bincount(wb.block_table[wb.block_table >= 0], minlength=wb.pool_pages)
    pos = np.full((wb.batch, wb.num_kv_heads), -1, dtype=np.int64)
    qf = wb.q.float()
    for b in range(wb.batch):
        L = int(wb.context_lens[b])
        if L == 0:
            continue
        for g in range(wb.num_kv_heads):
            j = int(rng.integers(0, L))
            page = int(wb.block_table[b, j // ps])
            if counts[page] > 1:
                continue
            qv = qf[b, g * group]
            key = qv * (strength * math.sqrt(wb.head_dim) / float((qv * qv).sum()))
            wb.k_pool[page, g, j % ps] = key.to(torch.bfloat16)
            pos[b, g] = j
    return pos


def plant_needles_prefill(wb: PagedBatch, seed: int, programs, strength: float = 30.0):
    """Append-prefill batches: for each given program and every kv head, one new token's first query
    head of the group gets a dominating key at a random visible position (as plant_needles).
    Returns the (program, new token, query head) rows whose softmax is dominated."""
    rng = np.random.default_rng(seed)
    group = wb.num_q_heads // wb.num_kv_heads
    ps = wb.page_size
    cu = wb.cu_q_lens
    qf = wb.q
    rows = []
    for b in programs:
        n, L = int(wb.q_lens[b]), int(wb.context_lens[b])
        for g in range(wb.num_kv_heads):
            i = int(rng.integers(0, n))
            j = int(rng.integers(0, L - n + i + 1))
            qv = qf[int(cu[b]) + i, g * group].float()
            key = qv * (strength * math.sqrt(wb.head_dim) / float((qv * qv).sum()))
            wb.k_pool[int(wb.block_table[b, j // ps]), g, j % ps] = key.to(torch.bfloat16)
            rows.append((int(b), i, g * group))
    return rows


def sharpen(wb: PagedBatch, factor: float = 4.0) -> None:
    """Scale the queries so that the softmax concentrates on few keys."""
    wb.q.copy_((wb.q.float() * factor).to(torch.bfloat16))


@dataclass
class AgentTrace:
    """Workflows of multi-turn agent programs: reasoning turns separated by tool calls."""

    initial_context: np.ndarray     # int32 [n] tokens each program starts with (system prompt + task)
    turn_tokens: np.ndarray         # int32 [n, turns] tokens decoded in each reasoning turn
    tool_ticks: np.ndarray          # int32 [n, turns] latency of the tool call after each turn, in ticks
    tool_tokens: np.ndarray         # int32 [n, turns] tokens of that tool's output


def agent_trace(seed: int, n_programs: int, n_turns: int, context_lo: int = 4096, context_hi: int = 20480,
                turn_lo: int = 64, turn_hi: int = 256, tool_median_ticks: float = 3.0, tool_sigma: float = 1.0,
                out_lo: int = 128, out_hi: int = 1024) -> AgentTrace:
    """A seeded trace: uniform contexts, turn lengths and tool-output sizes, and lognormal tool
    latencies (a heavy tail: most tools return within a few ticks, a few take ten times longer, the
    shape the paper reports for its agent workloads in App. B).  Integers only, no arithmetic of
    the method."""
    rng = np.random.default_rng(seed)
    shape = (n_programs, n_turns)
    ticks = np.maximum(1, np.rint(np.exp(rng.normal(math.log(tool_median_ticks), tool_sigma, size=shape))))
    return AgentTrace(
        initial_context=rng.integers(context_lo, context_hi + 1, size=n_programs).astype(np.int32),
        turn_tokens=rng.integers(turn_lo, turn_hi + 1, size=shape).astype(np.int32),
        tool_ticks=ticks.astype(np.int32),
        tool_tokens=rng.integers(out_lo, out_hi + 1, size=shape).astype(np.int32))


@dataclass
class Fp8Cache:
    """The K and V pools of a batch as 8-bit E4M3 codes plus the two scales of the call."""

    k_codes: torch.Tensor           # uint8 [P, Hkv, page, d]
    v_codes: torch.Tensor
    k_scale: float                  # value of a cached key element = code value * k_scale
    v_scale: float


def to_fp8_cache(wb: PagedBatch, k_scale: float = 0.021, v_scale: float = 0.017) -> Fp8Cache:
    """Quantise the bf16 pools of a batch to E4M3 codes with torch's own conversion
    (x / scale -> float8_e4m3fn, round to nearest even).  With N(0,1) values and these scales the
    codes stay far below the format's largest value (448).  NaN rows stay NaN (code 0x7f / 0xff).
    Input preparation only: what the codes mean is each side's own business."""
    k = (wb.k_pool.float() / float(np.float32(k_scale))).to(torch.float8_e4m3fn).view(torch.uint8)
    v = (wb.v_pool.float() / float(np.float32(v_scale))).to(torch.float8_e4m3fn).view(torch.uint8)
    return Fp8Cache(k.contiguous(), v.contiguous(), float(np.float32(k_scale)), float(np.float32(v_scale)))


def as_u8(t: torch.Tensor) -> np.ndarray:
    """uint8 tensor -> numpy on the host."""
    return t.detach().contiguous().cpu().numpy()


def as_u16(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns on the host."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
