"""GPU: in debug mode bad device-resident metadata is turned into an error by a checking
kernel before any other kernel runs (the attention and append kernels never see it)."""
import numpy as np
import pytest
import torch

from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture
def debug_mode():
    before = ta.ta_set_debug_checks(True)
    yield
    ta.ta_set_debug_checks(before)


def _decode_rc(wb, table, lens, pool_pages=0):
    desc = gu.desc_of(wb, pool_pages=pool_pages)
    bt = torch.from_numpy(np.ascontiguousarray(table)).to(DEV)
    cl = torch.from_numpy(np.ascontiguousarray(lens)).to(DEV)
    out = torch.zeros_like(wb.q)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, DEV)
    rc = ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, wb.max_context_len, out, None, ws, check=False)
    torch.cuda.synchronize()
    return rc


def test_decode_metadata_is_checked_in_debug_mode(debug_mode):
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 1400, batch=7, len_lo=20, len_hi=900)
    assert _decode_rc(wb, wb.block_table, wb.context_lens) == ta.TA_OK
    lens = wb.context_lens.copy()
    lens[3] = wb.max_context_len + 1                   # longer than the bound the launch was sized for
    assert _decode_rc(wb, wb.block_table, lens) == ta.TA_ERR_INVALID_ARG
    lens = wb.context_lens.copy()
    lens[0] = -5
    assert _decode_rc(wb, wb.block_table, lens) == ta.TA_ERR_INVALID_ARG
    table = wb.block_table.copy()
    table[5, 0] = -1                                   # a page the program uses is missing
    assert _decode_rc(wb, table, wb.context_lens) == ta.TA_ERR_INVALID_ARG
    # an entry at or beyond the pool end is caught when the descriptor states the pool size
    assert _decode_rc(wb, wb.block_table, wb.context_lens, pool_pages=wb.pool_pages) == ta.TA_OK
    used = int(wb.block_table[2, 0])
    assert _decode_rc(wb, wb.block_table, wb.context_lens, pool_pages=used) == ta.TA_ERR_INVALID_ARG
    table = wb.block_table.copy()
    table[4, 0] = wb.pool_pages
    assert _decode_rc(wb, table, wb.context_lens, pool_pages=wb.pool_pages) == ta.TA_ERR_INVALID_ARG


def test_checks_are_off_by_default_and_switchable():
    before = ta.ta_set_debug_checks(False)
    try:
        assert ta.ta_set_debug_checks(True) is False
        assert ta.ta_set_debug_checks(False) is True
    finally:
        ta.ta_set_debug_checks(before)


def test_append_metadata_is_checked_in_debug_mode(debug_mode):
    """ta_kv_append writes the pools through device-resident metadata: a stale table entry or more
    new tokens than the context holds is rejected before any byte is written."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 1402, batch=4, new_lo=5, new_hi=60, prefix_lo=30, prefix_hi=500)
    desc = gu.desc_of(wb, pool_pages=wb.pool_pages)
    new_k = torch.randn(wb.total_q, wb.num_kv_heads, 128, device=DEV).to(torch.bfloat16)
    new_v = torch.randn_like(new_k)
    k_before, v_before = wb.k_pool.clone(), wb.v_pool.clone()

    def rc_with(table, lens, cu, total=wb.total_q):
        bt = torch.from_numpy(np.ascontiguousarray(table)).to(DEV)
        cl = torch.from_numpy(np.ascontiguousarray(lens)).to(DEV)
        cu_t = torch.from_numpy(np.ascontiguousarray(cu, dtype=np.int32)).to(DEV)
        rc = ta.ta_kv_append(desc, new_k, new_v, cu_t, wb.k_pool, wb.v_pool, bt, cl, total, check=False)
        torch.cuda.synchronize()
        return rc

    table = wb.block_table.copy(); table[1, 0] = wb.pool_pages          # beyond the pool
    assert rc_with(table, wb.context_lens, wb.cu_q_lens) == ta.TA_ERR_INVALID_ARG
    table = wb.block_table.copy(); table[2, 1] = -1
    assert rc_with(table, wb.context_lens, wb.cu_q_lens) == ta.TA_ERR_INVALID_ARG
    lens = wb.context_lens.copy(); lens[0] = int(wb.q_lens[0]) - 1      # more new tokens than the context holds
    assert rc_with(wb.block_table, lens, wb.cu_q_lens) == ta.TA_ERR_INVALID_ARG
    cu = wb.cu_q_lens.copy(); cu[2] = cu[1] - 1
    assert rc_with(wb.block_table, wb.context_lens, cu) == ta.TA_ERR_INVALID_ARG
    cu = wb.cu_q_lens.copy(); cu[-1] -= 1                                # does not end at total_new
    assert rc_with(wb.block_table, wb.context_lens, cu) == ta.TA_ERR_INVALID_ARG
    assert torch.equal(wb.k_pool.view(torch.int16), k_before.view(torch.int16))
    assert torch.equal(wb.v_pool.view(torch.int16), v_before.view(torch.int16))
    assert rc_with(wb.block_table, wb.context_lens, wb.cu_q_lens) == ta.TA_OK


def test_prefill_metadata_is_checked_in_debug_mode(debug_mode):
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 1401, batch=4, new_lo=5, new_hi=60, prefix_lo=30, prefix_hi=500)
    desc = gu.desc_of(wb)
    bt = torch.from_numpy(wb.block_table).to(DEV)
    cl = torch.from_numpy(wb.context_lens).to(DEV)
    out = torch.zeros_like(wb.q)
    ws = ta.alloc_workspace(desc, wb.batch, wb.max_q_len, wb.max_context_len, DEV)

    def rc_with(cu_np, max_q_len=wb.max_q_len):
        cu = torch.from_numpy(np.ascontiguousarray(cu_np, dtype=np.int32)).to(DEV)
        rc = ta.ta_append_prefill(desc, wb.q, cu, wb.k_pool, wb.v_pool, bt, cl, wb.total_q, max_q_len,
                                  wb.max_context_len, out, None, ws, check=False)
        torch.cuda.synchronize()
        return rc

    good = wb.cu_q_lens
    assert rc_with(good) == ta.TA_OK
    bad = good.copy(); bad[0] = 1
    assert rc_with(bad) == ta.TA_ERR_INVALID_ARG       # does not start at zero
    bad = good.copy(); bad[2] = bad[1] - 1
    assert rc_with(bad) == ta.TA_ERR_INVALID_ARG       # decreases
    bad = good.copy(); bad[-1] += 3
    assert rc_with(bad) == ta.TA_ERR_INVALID_ARG       # does not end at total_q
    assert rc_with(good, max_q_len=int(wb.q_lens.max()) - 1) == ta.TA_ERR_INVALID_ARG
