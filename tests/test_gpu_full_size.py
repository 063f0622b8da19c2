"""GPU parity at the full sizes of the five workload configurations, in the launch
configuration the benchmark times: sampled output rows against the oracle, plus
properties that hold at any size."""
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


def test_config2_llama8b_decode_full_size():
    wb = wl.llama8b_decode(DEV)
    assert wb.batch == 64 and 4096 <= wb.context_lens.min() and wb.context_lens.max() <= 32768
    out, lse = gu.gpu_decode(wb)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    err, rel = gu.check_sampled_rows(wb, out, lse, np.random.default_rng(2), what="config 2")
    # needle variant on the same batch: outputs of magnitude O(1), where the relative term bites
    wl.plant_needles(wb, seed=22)
    out, lse = gu.gpu_decode(wb)
    gu.check_sampled_rows(wb, out, lse, np.random.default_rng(3), what="config 2 + needles")
    del wb, out, lse
    _free()


def test_config3_append_prefill_full_size():
    wb = wl.append_prefill(DEV)
    assert wb.batch == 64 and wb.q_lens.min() >= 256 and wb.q_lens.max() <= 2048
    out, lse = gu.gpu_prefill(wb)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    gu.check_sampled_rows(wb, out, lse, np.random.default_rng(4), n_programs=5, rows_per_program=10,
                          what="config 3", lse_tol=gu.LSE_TOL_PREFILL)
    del wb, out, lse
    _free()


def test_config4_forked_decode_full_size():
    wb = wl.forked_decode(DEV)
    assert wb.batch == 256 and wb.num_q_heads == 64
    out, lse = gu.gpu_decode(wb)
    assert torch.isfinite(out.float()).all()
    gu.check_sampled_rows(wb, out, lse, np.random.default_rng(5), what="config 4")
    # property: two members of a group given the same query and truncated to the shared prefix agree
    wb.q[1] = wb.q[0]
    wb.context_lens[:2] = wb.notes["prefix_len"]
    out2, lse2 = gu.gpu_decode(wb)
    assert torch.equal(out2[0].view(torch.int16), out2[1].view(torch.int16))
    assert torch.equal(lse2[0], lse2[1])
    del wb, out, lse, out2, lse2
    _free()


def test_config5_restore_then_decode_full_size():
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
    assert torch.isfinite(out.float()).all()
    rng = np.random.default_rng(6)
    gu.check_sampled_rows(wb, out, lse, rng, what="config 5 (all programs)")
    # and specifically rows of restored programs
    restored = rs.programs[:4].tolist()
    k_small, v_small, table = gu.compact_programs(wb, restored)
    rows_b = list(range(len(restored))) * 2
    rows_t = restored * 2
    rows_h = [0] * len(restored) + [31] * len(restored)
    vis = [int(wb.context_lens[b]) for b in restored] * 2
    ref, ref_lse = oracle.attend_rows(gu.geom_of(wb), wl.as_u16(wb.q), k_small, v_small, table,
                                      rows_b, rows_t, rows_h, vis)
    t = torch.tensor(rows_t, device=DEV); h = torch.tensor(rows_h, device=DEV)
    gu.assert_close(out[t, h], lse[t, h], ref, ref_lse, "config 5 (restored programs)")
    del wb, out, lse
    _free()
