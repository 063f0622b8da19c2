"""GPU parity at the full sizes of the five workload configurations, in the launch
configuration the benchmark times.  Where the oracle finishes the whole batch in seconds
(decode: configurations 2, 4 and 5) every output row is compared; append-prefill
(configuration 3, minutes for the oracle) is compared on whole tiles of rows of some programs
plus rows of every program.  Needle and sharpened variants make outputs of magnitude O(1), where
the relative term of the tolerance bites, on every kernel path."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _free():
    torch.cuda.empty_cache()


def test_config2_llama8b_decode_full_size_every_row():
    wb = wl.llama8b_decode(DEV)
    assert wb.batch == 64 and 4096 <= wb.context_lens.min() and wb.context_lens.max() <= 32768
    # a batch of this size streams on the matrix-core tile kernel
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "config 2", lse_tol=gu.LSE_TOL)
    # the same batch on the vector-ALU kernel (a chunk size given by the caller keeps it there)
    out, lse = gu.gpu_decode(wb, chunk_pages=128)
    gu.assert_close(out, lse, ref, ref_lse, "config 2, vector-ALU kernel")
    # needle variant on the same batch: outputs of magnitude O(1)
    pos = wl.plant_needles(wb, seed=22)
    ref, ref_lse = gu.oracle_decode(wb)
    out, lse = gu.gpu_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "config 2 + needles", lse_tol=gu.LSE_TOL)
    out, lse = gu.gpu_decode(wb, chunk_pages=128)
    gu.assert_close(out, lse, ref, ref_lse, "config 2 + needles, vector-ALU kernel")
    assert (pos >= 0).all() and np.abs(ref[:, ::4]).max() > 0.5
    del wb, out, lse
    _free()


def test_config2_fp8_cache_full_size_every_row():
    wb = wl.llama8b_decode(DEV)
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "config 2, fp8 cache", lse_tol=gu.LSE_TOL_FP8_DIFFUSE)
    wl.sharpen(wb, 4.0)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "config 2, fp8 cache, sharpened", lse_tol=gu.LSE_TOL_FP8)
    assert np.abs(ref).max() > 0.3
    del wb, fc, out, lse
    _free()


def test_config3_append_prefill_full_size():
    wb = wl.append_prefill(DEV)
    assert wb.batch == 64 and wb.q_lens.min() >= 256 and wb.q_lens.max() <= 2048
    out, lse = gu.gpu_prefill(wb)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    # every program contributes rows; four of them whole tiles of rows (all 32 heads of 96 tokens)
    gu.check_sampled_rows(wb, out, lse, np.random.default_rng(4), n_programs=wb.batch, rows_per_program=14,
                          dense_programs=4, dense_tokens=96, what="config 3",
                          lse_tol=gu.LSE_TOL)
    # needles: one dominated row per kv head in twelve programs; and sharpened queries
    needle_rows = wl.plant_needles_prefill(wb, seed=33, programs=list(range(0, wb.batch, 6)))
    out, lse = gu.gpu_prefill(wb)
    gu.check_sampled_rows(wb, out, lse, np.random.default_rng(41), n_programs=4, rows_per_program=6,
                          extra_rows=needle_rows, what="config 3 + needles", lse_tol=gu.LSE_TOL)
    wl.sharpen(wb, 4.0)
    out, lse = gu.gpu_prefill(wb)
    gu.check_sampled_rows(wb, out, lse, np.random.default_rng(42), n_programs=12, rows_per_program=10,
                          what="config 3 sharpened", lse_tol=gu.LSE_TOL)
    del wb, out, lse
    _free()


def test_config4_forked_decode_full_size_every_row():
    wb = wl.forked_decode(DEV)
    assert wb.batch == 256 and wb.num_q_heads == 64
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "config 4", lse_tol=gu.LSE_TOL)
    # needles sit in the private suffixes (shared pages are skipped): the matrix-core decode path
    # with eight heads per kv head gets outputs of magnitude O(1)
    pos = wl.plant_needles(wb, seed=44)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "config 4 + needles", lse_tol=gu.LSE_TOL)
    assert (pos >= 0).sum() > 0.05 * pos.size and np.abs(ref).max() > 0.5
    # property: two members of a group given the same query and truncated to the shared prefix agree
    wb.q[1] = wb.q[0]
    wb.context_lens[:2] = wb.notes["prefix_len"]
    out2, lse2 = gu.gpu_decode(wb)
    assert torch.equal(out2[0].view(torch.int16), out2[1].view(torch.int16))
    assert torch.equal(lse2[0], lse2[1])
    del wb, out, lse, out2, lse2
    _free()


def test_config4_in_shuffled_batch_order_every_row():
    """The 256 programs of configuration 4 in shuffled order: same results as the oracle, and the
    groups are still found (the benchmark shows the same step time for both orders)."""
    wb = wl.forked_decode(DEV)
    perm = np.random.default_rng(wl.SEED_BASE + 44).permutation(wb.batch)
    wb.q = wb.q[torch.from_numpy(perm).to(DEV)].contiguous()
    wb.block_table = np.ascontiguousarray(wb.block_table[perm])
    wb.context_lens = np.ascontiguousarray(wb.context_lens[perm])
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "config 4 shuffled", lse_tol=gu.LSE_TOL)
    del wb, out, lse
    _free()


def test_config5_restore_then_decode_full_size_every_row():
    wb = wl.long_horizon_restore(DEV)
    assert wb.batch == 128 and wb.context_lens.max() <= 131072
    rs = wb.restore
    page_bytes = wb.num_kv_heads * 16 * 128 * 2
    n = int(rs.dst_slots.shape[0])
    # checksum of the pages that must stay untouched (sampled: every 97th page not in dst)
    keep = np.setdiff1d(np.arange(0, wb.pool_pages, 97), rs.dst_slots)
    keep_t = torch.from_numpy(keep).to(DEV)
    before_k = wb.k_pool.index_select(0, keep_t).clone()
    before_v = wb.v_pool.index_select(0, keep_t).clone()
    staging = torch.empty(ta.ta_restore_staging_min_bytes(n) + (64 << 20), dtype=torch.uint8, device=DEV)
    ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v,
                          torch.from_numpy(rs.dst_slots.copy()), wb.pool_pages, staging)
    torch.cuda.synchronize()
    # bit-exact: every restored page equals its host source, the sampled others are unchanged
    dst = torch.from_numpy(rs.dst_slots.astype(np.int64)).to(DEV)
    step = 4096
    for lo in range(0, n, step):
        sl = slice(lo, min(n, lo + step))
        assert torch.equal(wb.k_pool.index_select(0, dst[sl]).cpu().view(torch.int16), rs.host_k[sl].view(torch.int16))
        assert torch.equal(wb.v_pool.index_select(0, dst[sl]).cpu().view(torch.int16), rs.host_v[sl].view(torch.int16))
    assert torch.equal(wb.k_pool.index_select(0, keep_t).view(torch.int16), before_k.view(torch.int16))
    assert torch.equal(wb.v_pool.index_select(0, keep_t).view(torch.int16), before_v.view(torch.int16))
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)            # every row, restored programs included
    gu.assert_close(out, lse, ref, ref_lse, "config 5 after the restore", lse_tol=gu.LSE_TOL)
    del wb, out, lse
    _free()
