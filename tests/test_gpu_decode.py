"""GPU parity: ta_paged_decode through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_config1_tiny_decode():
    wb = wl.tiny_decode(DEV)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "config 1")


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (8, 2), (8, 1), (32, 8), (64, 8)])
def test_ragged_lengths_all_group_sizes(Hq, Hkv):
    """Lengths that end inside a page, span several chunks and leave some waves without pages."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 100 + Hq + Hkv, batch=13, len_lo=1, len_hi=2500,
                           num_q_heads=Hq, num_kv_heads=Hkv, first_lens=[1, 15, 16, 17, 1024, 1025])
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"ragged Hq={Hq} Hkv={Hkv}")


@pytest.mark.parametrize("Hq,chunk_pages", [(32, 8), (32, 16), (32, 32), (32, 64), (32, 128), (32, 256), (32, 512),
                                             (64, 8), (64, 16), (64, 32), (64, 64), (64, 128), (64, 256), (64, 512)])
def test_every_chunk_length(chunk_pages, Hq):
    """Four heads per kv head run on the vector-ALU kernel with chunks of up to 128 pages (the leftover
    of a program in quarter-chunk pieces) and on the matrix-core tile kernel with 256 or 512; eight
    heads per kv head always on the tile kernel."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 200, batch=9, len_lo=100, len_hi=9000, num_q_heads=Hq)
    out, lse = gu.gpu_decode(wb, chunk_pages=chunk_pages)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"chunk_pages={chunk_pages} Hq={Hq}")


def test_padding_poison_is_never_read():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 300, batch=16, len_lo=1, len_hi=700)
    ref, ref_lse = gu.oracle_decode(wb)
    wl.poison_padding(wb)
    out, lse = gu.gpu_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "poisoned padding")


def test_needle_key_dominates():
    """One key per (program, kv head) gets weight ~1: outputs are O(1) and the relative term bites."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 400, batch=8, len_lo=3000, len_hi=9000)
    pos = wl.plant_needles(wb, seed=7)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "needle")
    G = wb.num_q_heads // wb.num_kv_heads
    assert np.abs(ref[:, ::G]).max() > 0.5 and (pos >= 0).all()


def test_sharpened_queries():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 500, batch=8, len_lo=500, len_hi=6000)
    wl.sharpen(wb, 4.0)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "sharp")


def test_empty_program_and_empty_batch():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 600, batch=4, len_lo=20, len_hi=90)
    wb.context_lens[2] = 0
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "empty program")
    assert torch.all(out[2] == 0) and torch.all(torch.isneginf(lse[2]))
    desc = gu.desc_of(wb)
    assert ta.ta_paged_decode(desc, None, None, None, None, torch.empty(0, dtype=torch.int32, device=DEV),
                              0, None, None, None, check=False) == ta.TA_OK


def test_forked_programs_shared_prefix_config4_shape():
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 700, batch=32, group=16, prefix_len=2048,
                          suffix_lo=100, suffix_hi=600)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "forked")


def test_runs_are_deterministic():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 800, batch=12, len_lo=100, len_hi=4000)
    a, la = gu.gpu_decode(wb)
    b, lb = gu.gpu_decode(wb)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)


def test_runs_on_the_tile_kernel_route_are_deterministic():
    """There the workgroups take items from a counter in whatever order they finish: every item writes
    its own partial slots, so the result must not depend on who ran what."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 801, batch=40, len_lo=100, len_hi=12000)
    runs = [gu.gpu_decode_bound(wb, 16 * 1100) for _ in range(4)]          # 40 x 1100 pages, 320 pairs: tile route
    for out, lse in runs[1:]:
        assert torch.equal(out.view(torch.int16), runs[0][0].view(torch.int16)) and torch.equal(lse, runs[0][1])
    wf = wl.forked_decode(DEV, seed=wl.SEED_BASE + 802, batch=48, group=16, prefix_len=4096, suffix_lo=10,
                          suffix_hi=3000)
    runs = [gu.gpu_decode(wf) for _ in range(4)]
    for out, lse in runs[1:]:
        assert torch.equal(out.view(torch.int16), runs[0][0].view(torch.int16)) and torch.equal(lse, runs[0][1])


def test_scale_override_and_strided_pool():
    """A non-default scale, and a pool whose page stride is larger than the packed tile size."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 900, batch=5, len_lo=50, len_hi=900,
                           num_q_heads=8, num_kv_heads=2)
    import oracle
    dev = wb.q.device
    pad = 256
    tile = 2 * 16 * 128
    k_wide = torch.randn(wb.pool_pages, tile + pad, device=dev).to(torch.bfloat16)
    v_wide = torch.randn(wb.pool_pages, tile + pad, device=dev).to(torch.bfloat16)
    k_wide[:, :tile] = wb.k_pool.view(wb.pool_pages, tile)
    v_wide[:, :tile] = wb.v_pool.view(wb.pool_pages, tile)
    desc = ta.Desc(8, 2, scale=0.05, pool_stride_page=tile + pad)
    bt = torch.from_numpy(wb.block_table).to(dev)
    cl = torch.from_numpy(wb.context_lens).to(dev)
    out = torch.empty_like(wb.q)
    lse = torch.empty((wb.batch, 8), dtype=torch.float32, device=dev)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, dev)
    ta.ta_paged_decode(desc, wb.q, k_wide, v_wide, bt, cl, wb.max_context_len, out, lse, ws)
    torch.cuda.synchronize()
    geom = oracle.Geometry(8, 2, scale=float(np.float32(0.05)))
    ref, ref_lse = oracle.paged_decode(geom, wl.as_u16(wb.q), wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool),
                                       wb.block_table, wb.context_lens)
    gu.assert_close(out, lse, ref, ref_lse, "scale/stride")


@pytest.mark.parametrize("chunk_pages", [8, 64, 128])
@pytest.mark.parametrize("Hq,Hkv,group", [(64, 8, 16), (32, 8, 5), (8, 8, 40), (16, 2, 40)])
def test_shared_prefix_groups_take_the_matrix_core_path(Hq, Hkv, group, chunk_pages):
    """Forked programs: whole shared chunks are computed once per group by the tile kernel.

    Groups larger than one tile of rows are split, the shared length is not a multiple of the
    chunk, and one member is cut short inside the shared region.
    """
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 710 + group, batch=2 * group, group=group,
                          prefix_len=2048 + 16 * 37, suffix_lo=1, suffix_hi=700, num_q_heads=Hq,
                          num_kv_heads=Hkv)
    wb.context_lens[3] = 1500          # ends inside the shared prefix
    wb.context_lens[group + 1] = 16    # shares a single page
    wl.poison_padding(wb)
    out, lse = gu.gpu_decode(wb, chunk_pages=chunk_pages)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"shared prefix Hq={Hq} Hkv={Hkv} group={group}",
                    lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("Hq,Hkv", [(64, 8), (32, 8)])
def test_forked_programs_in_shuffled_batch_order(Hq, Hkv):
    """Members of a group need not be neighbours in the batch: the groups are found by what the
    block tables name, and the result is the oracle's whatever the order."""
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 730, batch=48, group=8, prefix_len=4096, suffix_lo=10,
                          suffix_hi=900, num_q_heads=Hq, num_kv_heads=Hkv)
    perm = np.random.default_rng(wl.SEED_BASE + 731).permutation(wb.batch)
    wb.q = wb.q[torch.from_numpy(perm).to(wb.q.device)].contiguous()
    wb.block_table = np.ascontiguousarray(wb.block_table[perm])
    wb.context_lens = np.ascontiguousarray(wb.context_lens[perm])
    out, lse = gu.gpu_decode(wb, chunk_pages=64)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "shuffled forked batch", lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("batch,group,Hq,Hkv,chunk_pages", [(600, 20, 32, 8, 16), (1000, 50, 32, 8, 8), (330, 33, 64, 8, 32),
                                                          (130, 5, 8, 2, 0), (1024, 16, 16, 4, 16)])
def test_many_forked_programs_in_shuffled_order(batch, group, Hq, Hkv, chunk_pages):
    """Hundreds of programs in groups of irregular size (larger than one tile of rows too), shuffled:
    the plan sorts them with several waves and cuts the groups into sub-groups; the result is the
    oracle's."""
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 760 + group, batch=batch // group * group, group=group,
                          prefix_len=1024, suffix_lo=1, suffix_hi=200, num_q_heads=Hq, num_kv_heads=Hkv)
    perm = np.random.default_rng(wl.SEED_BASE + 761).permutation(wb.batch)
    wb.q = wb.q[torch.from_numpy(perm).to(wb.q.device)].contiguous()
    wb.block_table = np.ascontiguousarray(wb.block_table[perm])
    wb.context_lens = np.ascontiguousarray(wb.context_lens[perm])
    out, lse = gu.gpu_decode(wb, chunk_pages=chunk_pages)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"{wb.batch} forked programs, groups of {group}")


def test_short_contexts_take_the_single_launch_path():
    """Contexts of at most one bulk chunk: the chunk kernel writes the output itself (no partials)."""
    for Hq, Hkv in ((32, 8), (8, 8), (4, 2)):
        wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 740 + Hq, batch=11, len_lo=1, len_hi=2048, num_q_heads=Hq,
                               num_kv_heads=Hkv, first_lens=[1, 16, 17, 2048, 2047, 1025])
        wb.context_lens[7] = 0
        wl.poison_padding(wb)
        out, lse = gu.gpu_decode(wb)
        ref, ref_lse = gu.oracle_decode(wb)
        gu.assert_close(out, lse, ref, ref_lse, f"single launch Hq={Hq} Hkv={Hkv}")
        assert torch.all(out[7] == 0) and torch.all(torch.isneginf(lse[7]))


def test_tables_that_only_start_alike_are_not_grouped():
    """Two programs whose tables agree on the first page only: nothing may be shared."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 720, batch=6, len_lo=1200, len_hi=3000,
                           num_q_heads=8, num_kv_heads=2)
    wb.block_table[1, 0] = wb.block_table[0, 0]
    wb.block_table[3, :5] = wb.block_table[2, :5]
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, "partly aliased tables")


@pytest.mark.parametrize("poison", [False, True])
def test_large_bounds_send_four_heads_per_kv_head_to_the_tile_kernel(poison):
    """With up to four query heads per kv head the library streams the private chunks on the
    vector-ALU kernel for small batches and on the matrix-core tile kernel once batch x bound is
    large.  A small ragged batch under a large bound takes the second route: same results."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 260, batch=36, len_lo=1, len_hi=5000,
                           first_lens=[1, 16, 17, 2047, 2048, 2049, 4096])
    wb.context_lens[11] = 0
    if poison:
        wl.poison_padding(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    out_v, lse_v = gu.gpu_decode(wb)                          # 36 x 313 pages: vector-ALU kernel
    gu.assert_close(out_v, lse_v, ref, ref_lse, "small bound")
    out_t, lse_t = gu.gpu_decode_bound(wb, 32000)              # 36 x 2000 pages, 288 (program, kv head) pairs: tile kernel
    gu.assert_close(out_t, lse_t, ref, ref_lse, "large bound", lse_tol=gu.LSE_TOL)
    assert ta.ta_workspace_bytes(gu.desc_of(wb), wb.batch, 1, 32000) > 0


def test_more_than_1024_programs_on_every_route():
    """Above 1024 programs the plan kernel walks the batch in passes and does not look for shared
    prefixes; both routes, and a forked batch (whose groups then simply are not shared), stay exact."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 270, batch=1100, len_lo=1, len_hi=3000, num_q_heads=8,
                           num_kv_heads=2, first_lens=[0, 1, 2047, 2048, 2049])
    ref, ref_lse = gu.oracle_decode(wb)
    out, lse = gu.gpu_decode(wb)                       # 1100 x 188 pages, 2200 pairs: tile route
    gu.assert_close(out, lse, ref, ref_lse, "1100 programs, tile route", lse_tol=gu.LSE_TOL)
    out, lse = gu.gpu_decode(wb, chunk_pages=64)       # vector-ALU route
    gu.assert_close(out, lse, ref, ref_lse, "1100 programs, vector-ALU route")
    del wb
    torch.cuda.empty_cache()
    wf = wl.forked_decode(DEV, seed=wl.SEED_BASE + 271, batch=1040, group=16, prefix_len=2048, suffix_lo=1,
                          suffix_hi=300, num_q_heads=8, num_kv_heads=2)
    out, lse = gu.gpu_decode(wf, chunk_pages=64)
    ref, ref_lse = gu.oracle_decode(wf)
    gu.assert_close(out, lse, ref, ref_lse, "1040 forked programs")


@pytest.mark.parametrize("Hq", [32, 64])
def test_a_loose_context_bound_changes_nothing_but_the_plan(Hq):
    """Under a bound far above the real lengths the host sizes the workspace for long chunks and the
    plan kernel, which sees the lengths, settles on shorter ones (and recognises shared prefixes at that
    finer grain): same results as under a tight bound, on both routes."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 280 + Hq, batch=8, len_lo=1, len_hi=3000, num_q_heads=Hq,
                           first_lens=[0, 1, 127, 128, 129])
    ref, ref_lse = gu.oracle_decode(wb)
    for bound in (wb.max_context_len, 32768, 131072):
        out, lse = gu.gpu_decode_bound(wb, bound)
        gu.assert_close(out, lse, ref, ref_lse, f"bound {bound} Hq={Hq}", lse_tol=gu.LSE_TOL)
    wf = wl.forked_decode(DEV, seed=wl.SEED_BASE + 290 + Hq, batch=12, group=6, prefix_len=1024, suffix_lo=1,
                          suffix_hi=300, num_q_heads=Hq, num_kv_heads=8)
    ref, ref_lse = gu.oracle_decode(wf)
    for bound in (wf.max_context_len, 131072):
        out, lse = gu.gpu_decode_bound(wf, bound)
        gu.assert_close(out, lse, ref, ref_lse, f"forked, bound {bound} Hq={Hq}", lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 8), (32, 8)])
def test_thousands_of_short_programs_under_a_bound_one_of_them_sets(Hq, Hkv):
    """2200 programs of 16 to 700 tokens and one of 3000: the host's product of batch and bound asks
    for the tile kernel, the plan kernel sees the real lengths and hands the batch to the vector-ALU
    kernel, whose (item, kv head) pairs here outnumber the workgroups of one launch, so that the
    second, looping launch has work too."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 990 + Hq, batch=2200, len_lo=16, len_hi=700, num_q_heads=Hq,
                           num_kv_heads=Hkv, first_lens=[3000, 1, 0, 2049])
    out, lse = gu.gpu_decode(wb)
    assert torch.isfinite(out.float()).all()
    rng = np.random.default_rng(wl.SEED_BASE + 991)
    gu.check_sampled_rows(wb, out, lse, rng, n_programs=60, rows_per_program=4, extra_rows=[(0, 0, 0), (3, 0, Hq - 1)],
                          what=f"many short programs Hq={Hq}", lse_tol=gu.LSE_TOL)
    # every program's row is written (a program without context: zeros and -inf)
    assert torch.all(out[2] == 0) and torch.all(torch.isinf(lse[2]))
    assert torch.isfinite(lse[torch.arange(wb.batch, device=DEV) != 2]).all()
