"""GPU parity on many small seeded batches of random shape: head counts, group sizes, context and
query lengths, forked groups, padding poison.  Every case is valid input; each is compared with the
oracle element by element."""
import numpy as np
import pytest
import torch

from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HEADS = [(1, 1), (2, 1), (4, 1), (8, 1), (4, 2), (8, 2), (16, 2), (8, 8), (32, 8), (64, 8), (12, 3), (24, 3)]


@pytest.mark.parametrize("seed", range(24))
def test_decode_random_shapes(seed):
    rng = np.random.default_rng(wl.SEED_BASE + 5000 + seed)
    Hq, Hkv = HEADS[seed % len(HEADS)]
    batch = int(rng.integers(1, 40))
    hi = int(rng.choice([40, 300, 1500, 6000]))
    firsts = [int(x) for x in rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 1023, 1024, 1025], size=min(batch, 3))]
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 5100 + seed, batch=batch, len_lo=1, len_hi=hi,
                           num_q_heads=Hq, num_kv_heads=Hkv, first_lens=firsts)
    if seed % 2:
        wl.poison_padding(wb)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"decode seed={seed} Hq={Hq} Hkv={Hkv} B={batch}",
                    lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("seed", range(16))
def test_forked_decode_random_shapes(seed):
    rng = np.random.default_rng(wl.SEED_BASE + 5200 + seed)
    Hq, Hkv = HEADS[(seed * 5 + 3) % len(HEADS)]
    group = int(rng.integers(2, 20))
    n_groups = int(rng.integers(1, 4))
    prefix = 16 * int(rng.integers(1, 300))
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 5300 + seed, batch=group * n_groups, group=group,
                          prefix_len=prefix, suffix_lo=1, suffix_hi=int(rng.choice([5, 200, 900])),
                          num_q_heads=Hq, num_kv_heads=Hkv)
    out, lse = gu.gpu_decode(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"forked seed={seed} Hq={Hq} Hkv={Hkv} group={group} prefix={prefix}",
                    lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("seed", range(16))
def test_tile_kernel_route_random_shapes_up_to_four_heads_per_kv_head(seed):
    """One, two or four query heads per kv head on the tile-kernel route (asked for by its chunk
    lengths): private chunks, leftovers and chunks shared by forked groups (cut into sub-groups of
    128 rows) all run on the matrix-core tile kernel, where the two waves of a row block split the
    keys and meet in LDS."""
    rng = np.random.default_rng(wl.SEED_BASE + 5600 + seed)
    Hq, Hkv = [(32, 8), (16, 4), (8, 2), (4, 1), (16, 8), (8, 8), (2, 1), (1, 1)][seed % 8]
    if seed % 3 == 0:
        batch = int(rng.integers(1, 30))
        firsts = [int(x) for x in rng.choice([0, 1, 16, 17, 2047, 2048, 2049, 4095, 4097], size=min(batch, 4))]
        wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 5700 + seed, batch=batch, len_lo=1,
                               len_hi=int(rng.choice([100, 3000, 7000])), num_q_heads=Hq, num_kv_heads=Hkv,
                               first_lens=firsts)
    else:
        group = int(rng.choice([2, 3, 16, 33, 40]))
        n_groups = int(rng.integers(1, 3))
        wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 5700 + seed, batch=group * n_groups, group=group,
                              prefix_len=int(rng.choice([4096, 8192, 9000 // 16 * 16, 16384])), suffix_lo=1,
                              suffix_hi=int(rng.choice([5, 900, 3000])), num_q_heads=Hq, num_kv_heads=Hkv)
    if seed % 2:
        wl.poison_padding(wb)
    out, lse = gu.gpu_decode(wb, chunk_pages=256 if seed % 4 < 2 else 512)     # chunks of this length run on the tile kernel
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"tile route seed={seed} Hq={Hq} Hkv={Hkv} B={wb.batch}",
                    lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("seed", range(24))
def test_prefill_random_shapes(seed):
    rng = np.random.default_rng(wl.SEED_BASE + 5400 + seed)
    Hq, Hkv = HEADS[(seed * 7 + 1) % len(HEADS)]
    if Hq // Hkv not in (1, 2, 4, 8):
        Hq, Hkv = 8, 2
    batch = int(rng.integers(1, 9))
    new_hi = int(rng.choice([3, 70, 300, 700]))
    prefix_hi = int(rng.choice([0, 50, 700, 2500]))
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 5500 + seed, batch=batch, new_lo=1, new_hi=new_hi,
                           prefix_lo=0, prefix_hi=prefix_hi, num_q_heads=Hq, num_kv_heads=Hkv)
    if seed % 2:
        wl.poison_padding(wb)
    out, lse = gu.gpu_prefill(wb)
    ref, ref_lse = gu.oracle_prefill(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"prefill seed={seed} Hq={Hq} Hkv={Hkv} B={batch}",
                    lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("seed", range(20))
def test_prefill_random_shapes_with_cut_keys(seed):
    """Few programs with the keys of every query tile cut into chunks (the library's count or a forced
    one): ragged lengths, so that tiles end inside, at and before chunk boundaries, every group size."""
    rng = np.random.default_rng(wl.SEED_BASE + 6000 + seed)
    Hq, Hkv = [(32, 8), (8, 8), (64, 8), (16, 8), (8, 2), (4, 1), (2, 2), (16, 2), (8, 1), (12, 3)][seed % 10]
    batch = int(rng.integers(1, 7))
    new_hi = int(rng.choice([1, 20, 150, 400]))
    prefix_hi = int(rng.choice([300, 2500, 6000, 12000]))
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 6100 + seed, batch=batch, new_lo=1, new_hi=new_hi,
                           prefix_lo=0, prefix_hi=prefix_hi, num_q_heads=Hq, num_kv_heads=Hkv)
    if seed % 2:
        wl.poison_padding(wb)
    chunks = int(rng.choice([0, 0, 2, 3, 5, 8, 13, 32]))
    out, lse = gu.gpu_prefill(wb, key_chunks=chunks)
    if batch * new_hi * prefix_hi * Hq <= 40_000_000:
        ref, ref_lse = gu.oracle_prefill(wb)
        gu.assert_close(out, lse, ref, ref_lse, f"cut keys seed={seed} Hq={Hq} Hkv={Hkv} B={batch} chunks={chunks}",
                        lse_tol=gu.LSE_TOL)
    else:
        assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
        gu.check_sampled_rows(wb, out, lse, rng, n_programs=batch, rows_per_program=16, dense_programs=1,
                              dense_tokens=8, what=f"cut keys seed={seed} Hq={Hq} Hkv={Hkv} B={batch} chunks={chunks}",
                              lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("seed", range(16))
def test_fp8_cache_random_shapes(seed):
    """The same over an FP8 cache: ragged batches and forked groups (whose shared chunks one workgroup
    computes for up to 32 / (heads per kv head) members at once), any supported head shape."""
    rng = np.random.default_rng(wl.SEED_BASE + 5800 + seed)
    Hq, Hkv = [(32, 8), (8, 8), (64, 8), (16, 8), (8, 2), (4, 1), (2, 2), (16, 2)][seed % 8]
    if seed % 2 == 0:
        group = int(rng.choice([2, 3, 5, 16, 33, 40]))
        n_groups = int(rng.integers(1, 4))
        wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 5900 + seed, batch=group * n_groups, group=group,
                              prefix_len=16 * int(rng.integers(8, 400)), suffix_lo=1,
                              suffix_hi=int(rng.choice([5, 300, 2000])), num_q_heads=Hq, num_kv_heads=Hkv)
        perm = rng.permutation(wb.batch)
        wb.q = wb.q[torch.from_numpy(perm).to(wb.q.device)].contiguous()
        wb.block_table = np.ascontiguousarray(wb.block_table[perm])
        wb.context_lens = np.ascontiguousarray(wb.context_lens[perm])
    else:
        batch = int(rng.integers(1, 40))
        firsts = [int(x) for x in rng.choice([0, 1, 15, 16, 17, 31, 32, 33, 2047, 2048, 2049, 8191, 8193], size=min(batch, 4))]
        wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 5900 + seed, batch=batch, len_lo=1,
                               len_hi=int(rng.choice([40, 1500, 9000])), num_q_heads=Hq, num_kv_heads=Hkv,
                               first_lens=firsts)
    if seed % 3 == 0:
        wl.poison_padding(wb)
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc, chunk_pages=int(rng.choice([0, 0, 8, 32, 128, 512])))
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, f"fp8 seed={seed} Hq={Hq} Hkv={Hkv} B={wb.batch}", lse_tol=gu.LSE_TOL_FP8)
