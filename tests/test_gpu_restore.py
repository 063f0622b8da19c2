"""GPU parity: ta_kv_page_restore through the C ABI, bit-exact against the oracle's memcpy scatter."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _restore_case(batch=24, median=900, cap=5000, seed=wl.SEED_BASE + 1000):
    return wl.long_horizon_restore(DEV, seed=seed, batch=batch, median=median, sigma=0.75, len_lo=16,
                                   len_cap=cap)


def _expected_pools(wb):
    page_bytes = wb.num_kv_heads * 16 * 128 * 2
    kp = wl.as_u16(wb.k_pool).copy().view(np.uint8).reshape(wb.pool_pages, page_bytes)
    vp = wl.as_u16(wb.v_pool).copy().view(np.uint8).reshape(wb.pool_pages, page_bytes)
    rs = wb.restore
    hk = wl.as_u16(rs.host_k).view(np.uint8).reshape(-1, page_bytes)
    hv = wl.as_u16(rs.host_v).view(np.uint8).reshape(-1, page_bytes)
    assert oracle.kv_page_restore(kp, vp, page_bytes, hk, hv, rs.dst_slots, wb.pool_pages) == 0
    return kp, vp, page_bytes


@pytest.mark.parametrize("batch,median", [(24, 900), (48, 3000)])   # about 400 and 2700 pages: the second needs
@pytest.mark.parametrize("mode", ["zero_copy", "staged_small", "staged_all", "staged_rounds"])   # several launches per slot list
def test_restore_is_bit_exact_and_touches_nothing_else(mode, batch, median):
    wb = _restore_case(batch=batch, median=median, cap=6 * median)
    kp, vp, page_bytes = _expected_pools(wb)
    rs = wb.restore
    n = int(rs.dst_slots.shape[0])
    if mode == "zero_copy":
        nbytes = ta.ta_restore_staging_min_bytes(n)
    elif mode == "staged_small":
        nbytes = ta.ta_restore_staging_full_bytes(n, page_bytes) + 7 * 2 * page_bytes
    elif mode == "staged_rounds":      # two buffers of 260 pages: copies on the side stream, many rounds with a ragged last one
        nbytes = ta.ta_restore_staging_min_bytes(n) + 4 * 260 * page_bytes
    else:
        nbytes = ta.ta_restore_staging_min_bytes(n) + 2 * n * page_bytes + 512
    staging = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    slots = torch.from_numpy(rs.dst_slots.copy())
    ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, slots, wb.pool_pages, staging)
    slots.fill_(-7)            # the list was read before the call returned: the caller may reuse it at once
    torch.cuda.synchronize()
    got_k = wl.as_u16(wb.k_pool).view(np.uint8).reshape(wb.pool_pages, page_bytes)
    got_v = wl.as_u16(wb.v_pool).view(np.uint8).reshape(wb.pool_pages, page_bytes)
    assert np.array_equal(got_k, kp) and np.array_equal(got_v, vp)


def test_restore_then_decode_matches_oracle_config5_shape():
    wb = _restore_case(batch=32, median=1500, cap=9000, seed=wl.SEED_BASE + 1001)
    kp, vp, page_bytes = _expected_pools(wb)
    rs = wb.restore
    n = int(rs.dst_slots.shape[0])
    staging = torch.empty(ta.ta_restore_staging_min_bytes(n) + 64 * 2 * page_bytes, dtype=torch.uint8, device=DEV)
    ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v,
                          torch.from_numpy(rs.dst_slots.copy()), wb.pool_pages, staging)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = oracle.paged_decode(gu.geom_of(wb), wl.as_u16(wb.q), kp.view(np.uint16), vp.view(np.uint16),
                                       wb.block_table, wb.context_lens)
    gu.assert_close(out, lse, ref, ref_lse, "restore+decode")


def test_restore_rejects_bad_arguments_on_the_host():
    wb = _restore_case(batch=6, median=200, cap=600)
    rs = wb.restore
    page_bytes = wb.num_kv_heads * 16 * 128 * 2
    n = int(rs.dst_slots.shape[0])
    staging = torch.empty(ta.ta_restore_staging_min_bytes(n), dtype=torch.uint8, device=DEV)
    before = wb.k_pool.clone()
    dup = torch.from_numpy(rs.dst_slots.copy()); dup[1] = dup[0]
    oob = torch.from_numpy(rs.dst_slots.copy()); oob[0] = wb.pool_pages
    for bad in (dup, oob):
        rc = ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, bad,
                                   wb.pool_pages, staging, check=False)
        assert rc == ta.TA_ERR_INVALID_ARG
    misaligned = torch.empty(4096, dtype=torch.uint8, device=DEV)[16:]      # staging must be 256-byte aligned
    good = torch.from_numpy(rs.dst_slots.copy())
    assert ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, good, wb.pool_pages,
                                 misaligned, check=False) == ta.TA_ERR_INVALID_ARG
    assert ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, 100, rs.host_k, rs.host_v, good, wb.pool_pages,
                                 staging, check=False) == ta.TA_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), wb.k_pool.view(torch.int16))
    assert ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v,
                                 torch.empty(0, dtype=torch.int32), wb.pool_pages, staging, check=False) == ta.TA_OK


@pytest.mark.parametrize("mode", ["zero_copy", "staged"])
def test_restore_on_a_second_stream_while_resident_programs_decode(mode):
    """A paused program comes back while the others keep decoding (Sec. 4.3): the restore runs on a
    stream of its own, decode steps of the resident programs on another.  The restored pages are
    bit-exact, nothing else in the pools moved, and every decode step gives what it gives alone."""
    wb = _restore_case(batch=40, median=2500, cap=12000, seed=wl.SEED_BASE + 1002)
    kp, vp, page_bytes = _expected_pools(wb)
    rs = wb.restore
    n = int(rs.dst_slots.shape[0])
    resident = np.setdiff1d(np.arange(wb.batch), rs.programs)
    idx = torch.from_numpy(resident).to(DEV)
    q = wb.q[idx].contiguous()
    bt = torch.from_numpy(np.ascontiguousarray(wb.block_table[resident])).to(DEV)
    cl = torch.from_numpy(np.ascontiguousarray(wb.context_lens[resident])).to(DEV)
    max_len = int(wb.context_lens[resident].max())
    desc = gu.desc_of(wb)
    ws = ta.alloc_workspace(desc, len(resident), 1, max_len, DEV)

    def decode():
        out = torch.full_like(q, float("nan"))
        lse = torch.full((len(resident), wb.num_q_heads), float("nan"), dtype=torch.float32, device=DEV)
        ta.ta_paged_decode(desc, q, wb.k_pool, wb.v_pool, bt, cl, max_len, out, lse, ws)
        return out, lse

    alone_out, alone_lse = decode()
    torch.cuda.synchronize()
    # staged: room for two rounds of 300 pages, so the copies run on the library's side stream
    extra = 0 if mode == "zero_copy" else 4 * 300 * page_bytes
    assert n > 1200
    staging = torch.empty(ta.ta_restore_staging_min_bytes(n) + extra, dtype=torch.uint8, device=DEV)
    slots = torch.from_numpy(rs.dst_slots.copy())
    side = torch.cuda.Stream(device=DEV)
    done = torch.cuda.Event()
    ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, slots, wb.pool_pages, staging, side)
    done.record(side)
    results = [decode() for _ in range(6)]
    torch.cuda.synchronize()
    for out, lse in results:
        assert torch.equal(out.view(torch.int16), alone_out.view(torch.int16)) and torch.equal(lse, alone_lse)
    got_k = wl.as_u16(wb.k_pool).view(np.uint8).reshape(wb.pool_pages, page_bytes)
    got_v = wl.as_u16(wb.v_pool).view(np.uint8).reshape(wb.pool_pages, page_bytes)
    assert np.array_equal(got_k, kp) and np.array_equal(got_v, vp)
