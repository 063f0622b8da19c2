"""GPU: the attention calls are plain kernel launches on the caller's stream, so they can be
captured in a HIP graph; every replay must reproduce the eager result bit for bit."""
import pytest
import torch

from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("Hq", [32, 64])
def test_decode_replays_from_a_graph(Hq):
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 1300, batch=12, len_lo=50, len_hi=4000, num_q_heads=Hq)
    desc = gu.desc_of(wb)
    bt = torch.from_numpy(wb.block_table).to(DEV)
    cl = torch.from_numpy(wb.context_lens).to(DEV)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, DEV)
    eager, eager_lse = gu.gpu_decode(wb)                       # also the warm-up: one-time attributes are set
    out = torch.zeros_like(wb.q)
    lse = torch.zeros((wb.batch, wb.num_q_heads), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, wb.max_context_len, out, lse, ws, side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            ta.ta_paged_decode(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, wb.max_context_len, out, lse, ws, side)
    torch.cuda.synchronize()
    for replay in range(3):
        out.zero_()
        lse.zero_()
        ws.zero_()                                             # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager) and torch.equal(lse, eager_lse), f"replay {replay}"
    # new queries through the same graph: the captured pointers are read afresh at every replay
    wb.q.copy_(torch.randn(wb.q.shape, device=DEV).to(torch.bfloat16))
    fresh, fresh_lse = gu.gpu_decode(wb)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, fresh) and torch.equal(lse, fresh_lse)


@pytest.mark.parametrize("prefix_lo,prefix_hi", [(100, 1500), (3000, 9000)])   # the second: keys cut into chunks, merged
def test_append_prefill_replays_from_a_graph(prefix_lo, prefix_hi):
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 1301, batch=5, new_lo=10, new_hi=300, prefix_lo=prefix_lo,
                           prefix_hi=prefix_hi)
    desc = gu.desc_of(wb)
    bt = torch.from_numpy(wb.block_table).to(DEV)
    cl = torch.from_numpy(wb.context_lens).to(DEV)
    cu = torch.from_numpy(wb.cu_q_lens).to(DEV)
    ws = ta.alloc_workspace(desc, wb.batch, wb.max_q_len, wb.max_context_len, DEV)
    eager, eager_lse = gu.gpu_prefill(wb)
    out = torch.zeros_like(wb.q)
    lse = torch.zeros((wb.total_q, wb.num_q_heads), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()

    def call():
        ta.ta_append_prefill(desc, wb.q, cu, wb.k_pool, wb.v_pool, bt, cl, wb.total_q, wb.max_q_len,
                             wb.max_context_len, out, lse, ws, side)

    with torch.cuda.stream(side):
        call()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    for replay in range(3):
        out.zero_()
        lse.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager) and torch.equal(lse, eager_lse), f"replay {replay}"


def test_staged_restore_replays_from_a_graph():
    """With staging for two rounds the library would put the scatter kernels on a stream of its own; a
    stream under capture keeps everything on the one stream, and the graph replays bit-exactly."""
    import numpy as np
    import oracle

    wb = wl.long_horizon_restore(DEV, seed=wl.SEED_BASE + 1310, batch=24, median=2000, sigma=0.75, len_lo=16, len_cap=9000)
    rs = wb.restore
    page_bytes = wb.num_kv_heads * 16 * 128 * 2
    n = int(rs.dst_slots.shape[0])
    assert n > 600
    kp = wl.as_u16(wb.k_pool).copy().view(np.uint8).reshape(wb.pool_pages, page_bytes)
    vp = wl.as_u16(wb.v_pool).copy().view(np.uint8).reshape(wb.pool_pages, page_bytes)
    hk = wl.as_u16(rs.host_k).view(np.uint8).reshape(-1, page_bytes)
    hv = wl.as_u16(rs.host_v).view(np.uint8).reshape(-1, page_bytes)
    assert oracle.kv_page_restore(kp, vp, page_bytes, hk, hv, rs.dst_slots, wb.pool_pages) == 0
    staging = torch.empty(4 * 260 * page_bytes, dtype=torch.uint8, device=DEV)
    slots = torch.from_numpy(rs.dst_slots.copy())
    k0, v0 = wb.k_pool.clone(), wb.v_pool.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()

    def call():
        ta.ta_kv_page_restore(wb.k_pool, wb.v_pool, page_bytes, rs.host_k, rs.host_v, slots, wb.pool_pages, staging, side)

    with torch.cuda.stream(side):
        call()                       # eager: kernels on the library's side stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()                   # captured: one stream
    torch.cuda.synchronize()
    for replay in range(2):
        wb.k_pool.copy_(k0)
        wb.v_pool.copy_(v0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_k = wl.as_u16(wb.k_pool).view(np.uint8).reshape(wb.pool_pages, page_bytes)
        got_v = wl.as_u16(wb.v_pool).view(np.uint8).reshape(wb.pool_pages, page_bytes)
        assert np.array_equal(got_k, kp) and np.array_equal(got_v, vp), f"replay {replay}"
