"""GPU parity: ta_paged_decode over an FP8 (E4M3) KV cache through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_every_code_is_widened_exactly():
    """One cached token per program: the output is that token's value row times v_scale, the lse is
    scale * k_scale * <q, key>.  The value rows run through all 254 finite codes (v_scale = 1, so the
    bf16 output must equal the code's value bit for bit); the keys do too, one at a time against a
    one-hot query."""
    Hq = Hkv = 2
    codes = np.array([c for c in range(256) if (c & 0x7f) != 0x7f], np.uint8)       # 254 finite codes
    B = 128                                                                          # programs = dims probed on the key side
    k = np.zeros((B, Hkv, 16, 128), np.uint8)
    v = np.zeros((B, Hkv, 16, 128), np.uint8)
    q = torch.zeros((B, Hq, 128), dtype=torch.bfloat16)
    for b in range(B):
        for g in range(Hkv):
            v[b, g, 0] = codes[(np.arange(128) + 128 * g + b) % 254]                 # every code in many positions
            k[b, g, 0, b] = codes[(2 * b + g) % 254]                                 # a single non-zero key coordinate
        q[b, :, b] = 1.0
    table = np.arange(B, dtype=np.int32).reshape(B, 1)
    lens = np.ones(B, np.int32)
    desc = ta.Desc(Hq, Hkv, kv_format=ta.KV_FP8_E4M3, k_scale=0.5, v_scale=1.0)
    qd = q.to(DEV)
    out = torch.empty_like(qd)
    lse = torch.empty((B, Hq), dtype=torch.float32, device=DEV)
    ws = ta.alloc_workspace(desc, B, 1, 16, DEV)
    ta.ta_paged_decode(desc, qd, torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV),
                       torch.from_numpy(table).to(DEV), torch.from_numpy(lens).to(DEV), 16, out, lse, ws)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.paged_decode_fp8(oracle.Geometry(Hq, Hkv), wl.as_u16(q), k, v, 0.5, 1.0, table, lens)
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)                                                  # exact: every value is a bf16 value
    assert np.max(np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse)) <= 1e-5


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (8, 2), (8, 1), (32, 8), (64, 8)])
def test_ragged_lengths_all_group_sizes(Hq, Hkv):
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3100 + Hq + Hkv, batch=13, len_lo=1, len_hi=5000,
                           num_q_heads=Hq, num_kv_heads=Hkv, first_lens=[1, 15, 16, 17, 31, 32, 33, 2048, 2049])
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, f"fp8 ragged Hq={Hq} Hkv={Hkv}", lse_tol=gu.LSE_TOL_FP8)


@pytest.mark.parametrize("Hq", [32, 64])
@pytest.mark.parametrize("chunk_pages", [8, 16, 32, 64, 128, 256, 512])
def test_every_chunk_length(chunk_pages, Hq):
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3200, batch=9, len_lo=100, len_hi=9000, num_q_heads=Hq)
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc, chunk_pages=chunk_pages)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, f"fp8 chunk_pages={chunk_pages} Hq={Hq}", lse_tol=gu.LSE_TOL_FP8)


def test_short_contexts_single_launch_and_empty_program():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3300, batch=11, len_lo=1, len_hi=2048,
                           first_lens=[1, 16, 17, 2048, 2047, 1025, 48, 47])
    wb.context_lens[9] = 0
    wl.poison_padding(wb)                       # NaN rows become NaN codes
    fc = wl.to_fp8_cache(wb)
    assert bool(((fc.k_codes & 0x7f) == 0x7f).any())
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 short", lse_tol=gu.LSE_TOL_FP8)
    assert torch.all(out[9] == 0) and torch.all(torch.isneginf(lse[9]))


def test_nan_codes_in_unreadable_rows_are_never_read():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3400, batch=16, len_lo=1, len_hi=4000)
    ref, ref_lse = gu.oracle_decode_fp8(wb, wl.to_fp8_cache(wb))
    wl.poison_padding(wb)
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc, chunk_pages=16)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 poisoned padding", lse_tol=gu.LSE_TOL_FP8)


def test_sharpened_queries_and_other_scales():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3500, batch=8, len_lo=500, len_hi=6000)
    wl.sharpen(wb, 4.0)
    fc = wl.to_fp8_cache(wb, k_scale=0.0125, v_scale=0.03)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 sharp", lse_tol=gu.LSE_TOL_FP8)
    assert np.abs(ref).max() > 0.3              # outputs large enough for the relative term to bite


def test_runs_are_deterministic_and_the_static_scratch_variant_agrees():
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3600, batch=12, len_lo=100, len_hi=7000)
    fc = wl.to_fp8_cache(wb)
    a, la = gu.gpu_decode_fp8(wb, fc)
    b, lb = gu.gpu_decode_fp8(wb, fc)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)
    desc = gu.desc_of(wb, kv_format=ta.KV_FP8_E4M3, k_scale=fc.k_scale, v_scale=fc.v_scale)
    out = torch.empty_like(wb.q)
    lse = torch.empty_like(la)
    ta.ta_paged_decode_static(desc, wb.q, fc.k_codes, fc.v_codes, torch.from_numpy(wb.block_table).to(DEV),
                              torch.from_numpy(wb.context_lens).to(DEV), wb.max_context_len, out, lse)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), out.view(torch.int16)) and torch.equal(la, lse)


def test_forked_programs_read_aliased_pages():
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 3700, batch=16, group=8, prefix_len=2048, suffix_lo=10,
                          suffix_hi=500, num_q_heads=64, num_kv_heads=8)
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 forked", lse_tol=gu.LSE_TOL_FP8)


@pytest.mark.parametrize("Hq,Hkv,group,batch,chunk_pages", [(32, 8, 16, 48, 0), (8, 8, 20, 60, 16), (64, 8, 6, 30, 64),
                                                             (16, 8, 3, 33, 8), (32, 8, 5, 300, 32), (64, 8, 16, 64, 128)])
def test_shared_chunks_of_forked_programs_in_shuffled_order(Hq, Hkv, group, batch, chunk_pages):
    """Programs whose block tables start with the same pages share the chunks there: one workgroup
    computes the partials of up to 32 / (heads per kv head) of them at once (groups larger than that
    are cut), wherever the members sit in the batch."""
    wb = wl.forked_decode(DEV, seed=wl.SEED_BASE + 3720 + group, batch=batch, group=group, prefix_len=3072, suffix_lo=1,
                          suffix_hi=700, num_q_heads=Hq, num_kv_heads=Hkv)
    perm = np.random.default_rng(wl.SEED_BASE + 3721).permutation(wb.batch)
    wb.q = wb.q[torch.from_numpy(perm).to(wb.q.device)].contiguous()
    wb.block_table = np.ascontiguousarray(wb.block_table[perm])
    wb.context_lens = np.ascontiguousarray(wb.context_lens[perm])
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc, chunk_pages=chunk_pages)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, f"fp8 shared chunks Hq={Hq} group={group}", lse_tol=gu.LSE_TOL_FP8)


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (8, 8), (16, 2), (8, 1)])
def test_append_prefill_over_an_fp8_cache(Hq, Hkv):
    """Ragged new-token counts on prefixes from zero to a few thousand tokens: the tile kernel runs on
    the widened copy of the batch's pages; the scales enter as in the decode kernel."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 3900 + Hq + Hkv, batch=6, new_lo=1, new_hi=300, prefix_lo=0,
                           prefix_hi=2500, num_q_heads=Hq, num_kv_heads=Hkv)
    fc = wl.to_fp8_cache(wb, k_scale=0.03, v_scale=0.019)
    out, lse = gu.gpu_prefill_fp8(wb, fc)
    ref, ref_lse = gu.oracle_prefill_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, f"fp8 prefill Hq={Hq} Hkv={Hkv}", lse_tol=gu.LSE_TOL)


def test_append_prefill_over_an_fp8_cache_ignores_unreadable_codes():
    """NaN codes in every row no block table can legally read (the tails of last pages, unused pool
    pages) reach the widened copy as NaN and must never reach a result."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 3950, batch=5, new_lo=3, new_hi=90, prefix_lo=0, prefix_hi=700)
    wl.poison_padding(wb)
    fc = wl.to_fp8_cache(wb)
    assert int((wl.as_u8(fc.k_codes) & 0x7f == 0x7f).sum()) > 0
    out, lse = gu.gpu_prefill_fp8(wb, fc)
    ref, ref_lse = gu.oracle_prefill_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 prefill, poisoned padding", lse_tol=gu.LSE_TOL)


def test_append_then_prefill_then_decode_on_one_fp8_cache():
    """The serving sequence on an FP8 cache: quantise the tool output's tokens into the tail pages,
    attend from them (append-prefill), then decode one more step over the same cache."""
    wb = wl.append_prefill(DEV, seed=wl.SEED_BASE + 3960, batch=4, new_lo=10, new_hi=200, prefix_lo=50, prefix_hi=1500)
    fc = wl.to_fp8_cache(wb)
    new_k = torch.randn(wb.total_q, wb.num_kv_heads, 128, device=DEV).to(torch.bfloat16)
    new_v = torch.randn(wb.total_q, wb.num_kv_heads, 128, device=DEV).to(torch.bfloat16)
    want_k, want_v = wl.as_u8(fc.k_codes).copy(), wl.as_u8(fc.v_codes).copy()
    oracle.kv_append_fp8(gu.geom_of(wb), wl.as_u16(new_k), wl.as_u16(new_v), wb.cu_q_lens, want_k, want_v, fc.k_scale,
                         fc.v_scale, wb.block_table, wb.context_lens)
    desc = gu.desc_of(wb, kv_format=ta.KV_FP8_E4M3, k_scale=fc.k_scale, v_scale=fc.v_scale)
    _append_fp8(desc, new_k, new_v, wb.cu_q_lens, fc.k_codes, fc.v_codes, wb.block_table, wb.context_lens)
    assert np.array_equal(wl.as_u8(fc.k_codes), want_k) and np.array_equal(wl.as_u8(fc.v_codes), want_v)
    out, lse = gu.gpu_prefill_fp8(wb, fc)
    ref, ref_lse = gu.oracle_prefill_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 prefill after append", lse_tol=gu.LSE_TOL)
    # the decode step: one query per program over the same cache
    q1 = torch.randn(wb.batch, wb.num_q_heads, 128, device=DEV).to(torch.bfloat16)
    bt = torch.from_numpy(wb.block_table).to(DEV)
    cl = torch.from_numpy(wb.context_lens).to(DEV)
    out1 = torch.empty_like(q1)
    lse1 = torch.empty((wb.batch, wb.num_q_heads), dtype=torch.float32, device=DEV)
    ws = ta.alloc_workspace(desc, wb.batch, 1, wb.max_context_len, DEV)
    ta.ta_paged_decode(desc, q1, fc.k_codes, fc.v_codes, bt, cl, wb.max_context_len, out1, lse1, ws)
    torch.cuda.synchronize()
    ref1, ref1_lse = oracle.paged_decode_fp8(gu.geom_of(wb), wl.as_u16(q1), want_k, want_v, fc.k_scale, fc.v_scale,
                                             wb.block_table, wb.context_lens)
    gu.assert_close(out1, lse1, ref1, ref1_lse, "fp8 decode after append and prefill", lse_tol=gu.LSE_TOL_FP8)


def _append_fp8(desc, new_k, new_v, cu, k_codes, v_codes, table, lens):
    ta.ta_kv_append(desc, new_k, new_v, torch.from_numpy(cu).to(DEV), k_codes, v_codes,
                    torch.from_numpy(table).to(DEV), torch.from_numpy(lens).to(DEV), int(cu[-1]))
    torch.cuda.synchronize()


@pytest.mark.parametrize("scale", [1.0, 0.021, 3.0, 2.0 ** -7])
def test_append_quantises_every_bf16_pattern_as_the_oracle_does(scale):
    """All 65536 bf16 bit patterns (NaN, infinities, subnormals, ties of the format at scale 1) go
    through ta_kv_append as the 512 new tokens of one program with one kv head: codes bit-exact."""
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16).view(512, 1, 128).to(DEV)
    new_k = bits.view(torch.bfloat16)
    new_v = torch.flip(bits, dims=[0]).contiguous().view(torch.bfloat16)
    lens = np.array([512 + 40], np.int32)                       # 40 tokens are cached already
    cu = np.array([0, 512], np.int32)
    pages = (int(lens[0]) + 15) // 16
    table = np.random.default_rng(wl.SEED_BASE + 3800).permutation(pages + 3)[:pages].astype(np.int32)[None, :]
    k_codes = torch.full((pages + 3, 1, 16, 128), 0x55, dtype=torch.uint8, device=DEV)
    v_codes = torch.full((pages + 3, 1, 16, 128), 0x66, dtype=torch.uint8, device=DEV)
    want_k, want_v = wl.as_u8(k_codes).copy(), wl.as_u8(v_codes).copy()
    desc = ta.Desc(4, 1, kv_format=ta.KV_FP8_E4M3, k_scale=scale, v_scale=scale * 0.5)
    oracle.kv_append_fp8(oracle.Geometry(4, 1), wl.as_u16(new_k), wl.as_u16(new_v), cu, want_k, want_v, scale,
                         scale * 0.5, table, lens)
    _append_fp8(desc, new_k, new_v, cu, k_codes, v_codes, table, lens)
    got_k, got_v = wl.as_u8(k_codes), wl.as_u8(v_codes)
    assert np.array_equal(got_k, want_k), np.argwhere(got_k != want_k)[:5]
    assert np.array_equal(got_v, want_v), np.argwhere(got_v != want_v)[:5]
    assert (want_k == 0x55).sum() >= (40 + 3 * 16) * 128        # what was cached or unused stayed as it was


def test_a_cache_grown_by_append_decodes_like_the_oracles():
    """Ragged batch, eight kv heads: append the last tokens of every program into an FP8 cache that
    holds the earlier ones, then decode over it; codes bit-exact, attention within tolerance."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 3801, batch=9, len_lo=3, len_hi=1500,
                           first_lens=[1, 16, 17, 33])
    fc = wl.to_fp8_cache(wb)
    rng = np.random.default_rng(wl.SEED_BASE + 3802)
    new = np.minimum(wb.context_lens, rng.integers(0, 70, size=wb.batch)).astype(np.int32)
    new[0] = wb.context_lens[0]                                  # a program that is all new
    cu = np.zeros(wb.batch + 1, np.int32); np.cumsum(new, out=cu[1:])
    total = int(cu[-1])
    new_k = (torch.randn(total, wb.num_kv_heads, 128, device=DEV) * 1.5).to(torch.bfloat16)
    new_v = torch.randn(total, wb.num_kv_heads, 128, device=DEV).to(torch.bfloat16)
    want_k, want_v = wl.as_u8(fc.k_codes).copy(), wl.as_u8(fc.v_codes).copy()
    oracle.kv_append_fp8(gu.geom_of(wb), wl.as_u16(new_k), wl.as_u16(new_v), cu, want_k, want_v, fc.k_scale,
                         fc.v_scale, wb.block_table, wb.context_lens)
    desc = gu.desc_of(wb, kv_format=ta.KV_FP8_E4M3, k_scale=fc.k_scale, v_scale=fc.v_scale, pool_pages=wb.pool_pages)
    _append_fp8(desc, new_k, new_v, cu, fc.k_codes, fc.v_codes, wb.block_table, wb.context_lens)
    assert np.array_equal(wl.as_u8(fc.k_codes), want_k) and np.array_equal(wl.as_u8(fc.v_codes), want_v)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "fp8 cache grown by append", lse_tol=gu.LSE_TOL_FP8)


def test_thousands_of_short_programs_over_an_fp8_cache():
    """2200 programs of 16 to 700 tokens and one of 3000 (so the call is not the single-launch form): the
    batch has more (item, kv head) pairs than one launch has workgroups, and the second, walking launch
    of the kernel has work too.  Every row against the oracle."""
    wb = wl.llama8b_decode(DEV, seed=wl.SEED_BASE + 995, batch=2200, len_lo=16, len_hi=700, num_q_heads=16,
                           num_kv_heads=8, first_lens=[3000, 1, 0, 2049])
    fc = wl.to_fp8_cache(wb)
    out, lse = gu.gpu_decode_fp8(wb, fc)
    ref, ref_lse = gu.oracle_decode_fp8(wb, fc)
    gu.assert_close(out, lse, ref, ref_lse, "many short programs, fp8 cache", lse_tol=gu.LSE_TOL_FP8)
