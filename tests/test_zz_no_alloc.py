"""GPU: ta_paged_decode_static (the entry point that allocates nothing and brings its own scratch)
gives exactly what ta_paged_decode gives with a caller's workspace, call after call."""
import pytest
import torch

from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _static_decode(wb):
    desc = gu.desc_of(wb)
    bt = torch.from_numpy(wb.block_table).to(DEV)
    cl = torch.from_numpy(wb.context_lens).to(DEV)
    out = torch.full_like(wb.q, float("nan"))
    lse = torch.full((wb.batch, wb.num_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    ta.ta_paged_decode_static(desc, wb.q, wb.k_pool, wb.v_pool, bt, cl, wb.max_context_len, out, lse)
    torch.cuda.synchronize()
    return out, lse


def _same(a, b):
    return torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1], b[1])


def test_two_calls_in_a_row_the_second_smaller_match_the_workspace_entry_point():
    big = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 1500, batch=24, len_lo=500, len_hi=9000)
    small = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 1501, batch=5, len_lo=1, len_hi=700)
    want_big, want_small = gu.gpu_decode(big), gu.gpu_decode(small)
    got_big = _static_decode(big)          # fills the library's array with a long plan and many partials
    got_small = _static_decode(small)      # must not see any of it
    assert _same(got_big, want_big) and _same(got_small, want_small)
    # and against the oracle, to the same bar as the entry point it mirrors
    ref, ref_lse = gu.oracle_decode(small)
    gu.assert_close(got_small[0], got_small[1], ref, ref_lse, "static scratch, small after big")
    ref, ref_lse = gu.oracle_decode(big)
    gu.assert_close(got_big[0], got_big[1], ref, ref_lse, "static scratch, big")


def test_forked_programs_and_eight_heads_per_kv_head_use_the_same_array():
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 1502, batch=32, group=16, prefix_len=2048, suffix_lo=100,
                          suffix_hi=600)
    assert _same(_static_decode(wb), gu.gpu_decode(wb))


def test_a_batch_large_enough_for_the_tile_kernel_route_uses_the_same_array():
    """72 programs x a bound of 10,000 tokens: the private chunks stream on the matrix-core kernel,
    whose items, work counter and partials live in the library's array as well."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 1503, batch=72, len_lo=2000, len_hi=10000)
    got, want = _static_decode(wb), gu.gpu_decode(wb)
    assert _same(got, want)
    small = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 1504, batch=3, len_lo=1, len_hi=300)
    assert _same(_static_decode(small), gu.gpu_decode(small))
    ref, ref_lse = gu.oracle_decode(wb)
    gu.assert_close(got[0], got[1], ref, ref_lse, "static scratch, tile route", lse_tol=gu.LSE_TOL)


def test_a_call_beyond_the_array_is_refused_and_writes_nothing():
    desc = ta.Desc(32, 8)
    batch, max_len = 512, 131072
    assert ta.ta_workspace_bytes(desc, batch, 1, max_len) > ta.STATIC_SCRATCH_BYTES
    q = torch.zeros((batch, 32, 128), dtype=torch.bfloat16, device=DEV)
    out = torch.full_like(q, 3.0)
    pool = torch.zeros((1, 8, 16, 128), dtype=torch.bfloat16, device=DEV)
    bt = torch.zeros((batch, max_len // 16), dtype=torch.int32, device=DEV)
    cl = torch.ones(batch, dtype=torch.int32, device=DEV)
    rc = ta.ta_paged_decode_static(desc, q, pool, pool, bt, cl, max_len, out, None, check=False)
    torch.cuda.synchronize()
    assert rc == ta.TA_ERR_TOO_LARGE and "scratch" in ta.ta_strerror(rc)
    assert torch.all(out == 3.0)
