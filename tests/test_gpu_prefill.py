"""GPU parity: ta_append_prefill through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check(wb, what):
    out, lse = gu.gpu_prefill(wb)
    ref, ref_lse = gu.oracle_prefill(wb)
    return gu.assert_close(out, lse, ref, ref_lse, what, lse_tol=gu.LSE_TOL)


def test_config3_shape_small():
    """Same structure as the append-prefill configuration, shrunk so the oracle takes seconds."""
    wb = wl.append_prefill(DEV, batch=6, new_lo=16, new_hi=300, prefix_lo=500, prefix_hi=2500)
    _check(wb, "config 3 (small)")


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (8, 2), (8, 1)])
def test_all_group_sizes(Hq, Hkv):
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 30 + Hkv, batch=4, new_lo=1, new_hi=150,
                           prefix_lo=0, prefix_hi=700, num_q_heads=Hq, num_kv_heads=Hkv)
    _check(wb, f"groups Hq={Hq} Hkv={Hkv}")


@pytest.mark.parametrize("n,prefix", [(1, 0), (1, 77), (63, 1), (64, 0), (65, 63), (128, 64), (200, 0),
                                      (17, 1000), (257, 31)])
def test_tile_and_page_boundaries(n, prefix):
    """Query-tile (64 tokens), key-tile (64 keys) and page (16) boundaries, empty prefixes."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 31, batch=3, new_lo=n, new_hi=n, prefix_lo=prefix,
                           prefix_hi=prefix, num_q_heads=8, num_kv_heads=2)
    _check(wb, f"n={n} prefix={prefix}")


def test_padding_poison_is_never_read():
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 32, batch=5, new_lo=3, new_hi=120, prefix_lo=5,
                           prefix_hi=900, num_q_heads=8, num_kv_heads=2)
    ref, ref_lse = gu.oracle_prefill(wb)
    wl.poison_padding(wb)
    out, lse = gu.gpu_prefill(wb)
    gu.assert_close(out, lse, ref, ref_lse, "poisoned padding", lse_tol=gu.LSE_TOL)


def test_sharpened_queries():
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 33, batch=3, new_lo=40, new_hi=200, prefix_lo=300,
                           prefix_hi=1500, num_q_heads=8, num_kv_heads=2)
    wl.sharpen(wb, 4.0)
    _check(wb, "sharp")


def test_program_without_new_tokens_and_empty_call():
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 34, batch=4, new_lo=5, new_hi=90, prefix_lo=20,
                           prefix_hi=400, num_q_heads=8, num_kv_heads=2)
    # program 1 contributes no rows: drop its queries from the packed array
    cu = wb.cu_q_lens
    keep = np.ones(wb.total_q, dtype=bool)
    keep[cu[1]:cu[2]] = False
    wb.context_lens[1] -= wb.q_lens[1]
    wb.q_lens[1] = 0
    wb.q = wb.q[torch.from_numpy(keep).to(DEV)].contiguous()
    _check(wb, "n_b = 0")
    desc = gu.desc_of(wb)
    assert ta.ta_append_prefill(desc, None, None, None, None, None,
                                torch.empty(0, dtype=torch.int32, device=DEV), 0, 0, 0, None, None, None,
                                check=False) == ta.TA_OK


def test_single_new_token_agrees_with_decode():
    """Append-prefill with one new token per program is the decode step."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 35, batch=7, len_lo=1, len_hi=1500, num_q_heads=8,
                           num_kv_heads=2)
    out_p, lse_p = gu.gpu_prefill(wb)
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(out_p, lse_p, ref, ref_lse, "prefill n=1", lse_tol=gu.LSE_TOL)


def test_runs_are_deterministic():
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 36, batch=4, new_lo=30, new_hi=200, prefix_lo=100,
                           prefix_hi=1200)
    a, la = gu.gpu_prefill(wb)
    b, lb = gu.gpu_prefill(wb)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)


def test_long_causal_sequences_without_a_prefix():
    """Whole-context re-prefill (the recompute side of the paper's trade-off): every query tile walks a
    different number of key tiles, most of the work lies near the diagonal."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 950, batch=3, new_lo=3000, new_hi=9000, prefix_lo=0,
                           prefix_hi=0)
    out, lse = gu.gpu_prefill(wb)
    assert torch.isfinite(out.float()).all()
    rng = np.random.default_rng(wl.SEED_BASE + 951)
    gu.check_sampled_rows(wb, out, lse, rng, n_programs=3, rows_per_program=24, what="long causal",
                          lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("batch,n_lo,n_hi,p_lo,p_hi,Hq,Hkv", [
    (1, 1, 1, 20000, 20000, 32, 8),          # one token onto a long context
    (1, 64, 64, 32768, 32768, 32, 8),        # a tool result coming back for one program
    (1, 256, 256, 9000, 9000, 8, 8),
    (2, 100, 300, 3000, 12000, 8, 2),
    (3, 1, 40, 2000, 70000, 64, 8),          # one long context among short ones
    (4, 200, 256, 16000, 16400, 8, 1),
    (1, 1500, 1500, 900, 900, 32, 8),        # the new tokens themselves span several chunks of keys
])
def test_few_programs_whose_keys_are_cut_into_chunks(batch, n_lo, n_hi, p_lo, p_hi, Hq, Hkv):
    """With few query tiles the keys of every tile are cut into chunks of whole kilotokens, one
    workgroup each, and the chunks' partials merged: rows whose visible keys end inside a chunk, or
    before it begins, and programs too short to reach the later chunks are all among these."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 960 + batch + Hq, batch=batch, new_lo=n_lo, new_hi=n_hi,
                           prefix_lo=p_lo, prefix_hi=p_hi, num_q_heads=Hq, num_kv_heads=Hkv)
    wl.poison_padding(wb)
    out, lse = gu.gpu_prefill(wb)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    rng = np.random.default_rng(wl.SEED_BASE + 961)
    gu.check_sampled_rows(wb, out, lse, rng, n_programs=batch, rows_per_program=12, dense_programs=1,
                          dense_tokens=20, what=f"chunked keys B={batch} n<={n_hi} prefix<={p_hi}", lse_tol=gu.LSE_TOL)


def test_chunked_keys_over_an_fp8_cache():
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 970, batch=2, new_lo=30, new_hi=90, prefix_lo=2500,
                           prefix_hi=6000, num_q_heads=16, num_kv_heads=4)
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_prefill_fp8(wb, fc)
    ref, ref_lse = gu.oracle_prefill_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "chunked keys, fp8 cache", lse_tol=gu.LSE_TOL_FP8)


@pytest.mark.parametrize("key_chunks", [1, 2, 3, 7, 40, 1024])
def test_any_number_of_key_chunks_gives_the_same_result(key_chunks):
    """The caller's number of chunks (1 = never cut; more than the keys allow is reduced): every choice
    agrees with the oracle, on a ragged batch whose short programs do not reach the later chunks."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 980, batch=5, new_lo=1, new_hi=200, prefix_lo=0,
                           prefix_hi=3000, num_q_heads=16, num_kv_heads=2)
    out, lse = gu.gpu_prefill(wb, key_chunks=key_chunks)
    ref, ref_lse = gu.oracle_prefill(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"key chunks {key_chunks}", lse_tol=gu.LSE_TOL)


@pytest.mark.parametrize("Hq,Hkv,chunks", [(8, 1, 0), (4, 2, 4)])
def test_cut_keys_with_more_programs_than_a_wave_has_lanes(Hq, Hkv, chunks):
    """Eighty programs of a few tokens each with one or two kv heads: few enough (tile, kv head) pairs
    for the keys to be cut (the library's own choice with one kv head, asked for with two), too many
    programs for the tile kernel to work the tile list out in one wave, so the plan kernel's list is
    used together with the chunks."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 985, batch=80, new_lo=1, new_hi=20, prefix_lo=2500,
                           prefix_hi=6000, num_q_heads=Hq, num_kv_heads=Hkv)
    assert ta.ta_workspace_bytes(gu.desc_of(wb, prefill_key_chunks=chunks), wb.batch, wb.max_q_len, wb.max_context_len) > \
        ta.ta_workspace_bytes(gu.desc_of(wb, prefill_key_chunks=1), wb.batch, wb.max_q_len, wb.max_context_len)
    out, lse = gu.gpu_prefill(wb, key_chunks=chunks)
    ref, ref_lse = gu.oracle_prefill(wb)
    gu.assert_close(out, lse, ref, ref_lse, f"cut keys, 80 programs, Hq={Hq} Hkv={Hkv}", lse_tol=gu.LSE_TOL)
