"""Shared helpers of the GPU parity tests: call the C ABI, call the oracle, compare."""
import numpy as np
import torch

import oracle
from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

ABS_TOL = 2e-2      # contract: |gpu - oracle| <= 2e-2 + 1e-2 * |oracle| (bf16 in, fp32 accumulate)
REL_TOL = 1e-2
ROW_L2_TOL = 1e-2   # tighter gates of our own: relative L2 error per output row ...
# ... and the log-sum-exp, which a zero output could not fake.  With a bf16 cache both kernels add up
# the weights in fp32 before any rounding: summing n of them one after another is off by about
# sqrt(n) * 2^-24 relative (2e-5 at 128k keys; at most n * 2^-24 if every rounding went the same way),
# the exponentials and the logarithm by a few units in the last place.  Observed: 8e-6 at most, with
# planted needles; the bound in the tests is 2e-4.
LSE_TOL = 2e-4
# The kernel for FP8 caches sums the bf16-ROUNDED weights (the ones the matrix core multiplies): a
# bf16 has 8 significant bits, so each weight is off by at most 2^-8 relative (half a step of
# 2^-7 just above a power of two), hence so is the sum, and |lse error| <= ln(1 + 2^-8) = 3.9e-3
# whatever the input; the bound is approached when one key dominates a row.  fp32 rounding comes on top.
LSE_TOL_FP8 = 4.5e-3
# With many keys of comparable weight (N(0,1) inputs at long context) the rounding errors average
# out; observed 1.0e-4 on the full-size workload.
LSE_TOL_FP8_DIFFUSE = 5e-4


def widen_bf16(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def desc_of(wb, **kw) -> ta.Desc:
    return ta.Desc(wb.num_q_heads, wb.num_kv_heads, **kw)


def geom_of(wb) -> oracle.Geometry:
    return oracle.Geometry(wb.num_q_heads, wb.num_kv_heads)


def gpu_decode(wb, stream=None, chunk_pages=0):
    dev = wb.q.device
    desc = desc_of(wb, decode_chunk_pages=chunk_pages)
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    out = torch.full_like(wb.q, float("nan"))
    lse = torch.full((wb.batch, wb.num_q_heads), float("nan"), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, dev)
    ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, wb.max_context_len, out, lse, ws, stream)
    torch.cuda.synchronize()
    return out, lse


def gpu_decode_fp8(wb, fc, stream=None, chunk_pages=0):
    """Decode over the batch's cache as E4M3 codes (fc: workloads.Fp8Cache)."""
    dev = wb.q.device
    desc = desc_of(wb, decode_chunk_pages=chunk_pages, kv_format=ta.KV_FP8_E4M3, k_scale=fc.k_scale,
                   v_scale=fc.v_scale)
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    out = torch.full_like(wb.q, float("nan"))
    lse = torch.full((wb.batch, wb.num_q_heads), float("nan"), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, dev)
    ta.ta_paged_decode(desc, wb.q, fc.k_codes, fc.v_codes, bt, cl, wb.max_context_len, out, lse, ws, stream)
    torch.cuda.synchronize()
    return out, lse


def gpu_decode_bound(wb, max_context_len):
    """ta_paged_decode with a context-length bound (and block-table width) far above the batch's own
    lengths, as a serving loop sizes them once for its longest admissible program.  With up to four
    query heads per kv head a large batch x bound sends the private chunks to the matrix-core tile
    kernel instead of the vector-ALU kernel."""
    dev = wb.q.device
    width = (max_context_len + 15) // 16
    assert width >= wb.block_table.shape[1]
    table = np.full((wb.batch, width), -1, np.int32)
    table[:, : wb.block_table.shape[1]] = wb.block_table
    desc = desc_of(wb)
    bt = torch.from_numpy(table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    out = torch.full_like(wb.q, float("nan"))
    lse = torch.full((wb.batch, wb.num_q_heads), float("nan"), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, 1, max_context_len, dev)
    ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, max_context_len, out, lse, ws)
    torch.cuda.synchronize()
    return out, lse


def oracle_decode_fp8(wb, fc):
    return oracle.paged_decode_fp8(geom_of(wb), wl.as_u16(wb.q), wl.as_u8(fc.k_codes), wl.as_u8(fc.v_codes),
                                   fc.k_scale, fc.v_scale, wb.block_table, wb.context_lens)


def gpu_prefill(wb, stream=None, key_chunks=0):
    dev = wb.q.device
    desc = desc_of(wb, prefill_key_chunks=key_chunks)
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    cu = torch.from_numpy(wb.cu_q_lens).to(dev)
    out = torch.full_like(wb.q, float("nan"))
    lse = torch.full((wb.total_q, wb.num_q_heads), float("nan"), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, max(wb.max_q_len, 2), wb.max_context_len, dev)
    ta.ta_append_prefill(desc, wb.q, cu, wb.k_pool, wb.v_pool, bt, cl, wb.total_q, wb.max_q_len,
                         wb.max_context_len, out, lse, ws, stream)
    torch.cuda.synchronize()
    return out, lse


def gpu_prefill_fp8(wb, fc, stream=None):
    """Append-prefill over the batch's cache as E4M3 codes (fc: workloads.Fp8Cache)."""
    dev = wb.q.device
    desc = desc_of(wb, kv_format=ta.KV_FP8_E4M3, k_scale=fc.k_scale, v_scale=fc.v_scale)
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    cu = torch.from_numpy(wb.cu_q_lens).to(dev)
    out = torch.full_like(wb.q, float("nan"))
    lse = torch.full((wb.total_q, wb.num_q_heads), float("nan"), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, max(wb.max_q_len, 2), wb.max_context_len, dev)
    ta.ta_append_prefill(desc, wb.q, cu, fc.k_codes, fc.v_codes, bt, cl, wb.total_q, wb.max_q_len,
                         wb.max_context_len, out, lse, ws, stream)
    torch.cuda.synchronize()
    return out, lse


def oracle_prefill_fp8(wb, fc):
    return oracle.append_prefill_fp8(geom_of(wb), wl.as_u16(wb.q), wb.cu_q_lens, wl.as_u8(fc.k_codes),
                                     wl.as_u8(fc.v_codes), fc.k_scale, fc.v_scale, wb.block_table, wb.context_lens)


def oracle_decode(wb):
    return oracle.paged_decode(geom_of(wb), wl.as_u16(wb.q), wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool),
                               wb.block_table, wb.context_lens)


def oracle_prefill(wb):
    return oracle.append_prefill(geom_of(wb), wl.as_u16(wb.q), wb.cu_q_lens, wl.as_u16(wb.k_pool),
                                 wl.as_u16(wb.v_pool), wb.block_table, wb.context_lens)


def assert_close(gpu_out, gpu_lse, ref_out, ref_lse, what="", lse_tol=LSE_TOL):
    """Element-wise contract tolerance plus the tighter per-row gates."""
    got = widen_bf16(gpu_out).reshape(ref_out.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref_out)
    bound = ABS_TOL + REL_TOL * np.abs(ref_out)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), f"{what}: |err|={err[worst]:.4g} at {worst}, ref={ref_out[worst]:.4g}"
    num = np.sqrt((err ** 2).sum(axis=-1))
    den = np.sqrt((ref_out ** 2).sum(axis=-1))
    ok_rows = den > 0
    rel = np.where(ok_rows, num / np.where(ok_rows, den, 1.0), num)
    assert rel.max() <= ROW_L2_TOL, f"{what}: row relative L2 error {rel.max():.4g}"
    if gpu_lse is not None:
        gl = gpu_lse.detach().cpu().numpy().astype(np.float64).reshape(ref_lse.shape)
        finite = np.isfinite(ref_lse)
        assert np.array_equal(np.isneginf(gl), np.isneginf(ref_lse)), f"{what}: -inf lse mismatch"
        assert np.max(np.abs(gl[finite] - ref_lse[finite]), initial=0.0) <= lse_tol, \
            f"{what}: lse error {np.max(np.abs(gl[finite] - ref_lse[finite])):.4g}"
    return float(err.max()), float(rel.max())


def compact_programs(wb, programs):
    """Host copy of just the pages the given programs name, with block tables remapped.

    Input plumbing only: lets the oracle check sampled rows of a workload whose whole
    pool would be many GiB.  Returns (k_pool_u16, v_pool_u16, table[int32, len(programs) x stride]).
    """
    ps = wb.page_size
    remap = {}
    rows = []
    for b in programs:
        npg = (int(wb.context_lens[b]) + ps - 1) // ps
        row = np.full(wb.block_table.shape[1], -1, dtype=np.int32)
        for i in range(npg):
            page = int(wb.block_table[b, i])
            row[i] = remap.setdefault(page, len(remap))
        rows.append(row)
    order = np.array(list(remap.keys()), dtype=np.int64)     # insertion order == new index
    idx = torch.from_numpy(order).to(wb.k_pool.device)
    k_small = wl.as_u16(wb.k_pool.index_select(0, idx))
    v_small = wl.as_u16(wb.v_pool.index_select(0, idx))
    return k_small, v_small, np.stack(rows)


def check_sampled_rows(wb, gpu_out, gpu_lse, rng, n_programs=6, rows_per_program=8, what="",
                       lse_tol=LSE_TOL, dense_programs=0, dense_tokens=64, extra_rows=()):
    """Compare sampled (program, new token, head) rows of a full-size run with the oracle.

    n_programs programs contribute rows_per_program random rows each plus their first and last new
    token; the first dense_programs of them contribute ALL heads of dense_tokens consecutive new
    tokens (a whole tile of rows, across a tile boundary); extra_rows are (program, token, head)
    triples that must be among the rows (planted needles).
    """
    programs = sorted(rng.choice(wb.batch, size=min(n_programs, wb.batch), replace=False).tolist())
    # always include the longest context: it crosses the most chunks / tiles
    longest = int(np.argmax(wb.context_lens))
    if longest not in programs:
        programs[0] = longest
        programs.sort()
    for b, _, _ in extra_rows:
        if b not in programs:
            programs.append(int(b))
    local_of = {b: i for i, b in enumerate(programs)}
    k_small, v_small, table = compact_programs(wb, programs)
    cu = wb.cu_q_lens
    row_b, row_t, row_h, row_vis = [], [], [], []

    def add(b, i, h):
        n, L = int(wb.q_lens[b]), int(wb.context_lens[b])
        row_b.append(local_of[b]); row_t.append(int(cu[b]) + i); row_h.append(h); row_vis.append(L - n + i + 1)

    for b, i, h in extra_rows:
        add(int(b), int(i), int(h))
    for rank, b in enumerate(programs[: n_programs]):
        n = int(wb.q_lens[b])
        for _ in range(rows_per_program):
            add(b, int(rng.integers(0, n)), int(rng.integers(0, wb.num_q_heads)))
        # the last new token sees everything, the first sees only the prefix and itself
        for i in (0, n - 1):
            add(b, i, 0)
        if rank < dense_programs:
            first = int(rng.integers(0, max(n - dense_tokens, 0) + 1))
            for i in range(first, min(n, first + dense_tokens)):
                for h in range(wb.num_q_heads):
                    add(b, i, h)
    ref, ref_lse = oracle.attend_rows(geom_of(wb), wl.as_u16(wb.q), k_small, v_small, table,
                                      row_b, row_t, row_h, row_vis)
    t = torch.tensor(row_t, device=gpu_out.device)
    h = torch.tensor(row_h, device=gpu_out.device)
    got = gpu_out[t, h]
    got_lse = gpu_lse[t, h]
    return assert_close(got, got_lse, ref, ref_lse, what, lse_tol=lse_tol)
