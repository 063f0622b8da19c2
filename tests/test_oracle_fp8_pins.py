"""CPU pins of the oracle's FP8 (E4M3) KV-cache decode.  None of them uses the oracle to check
itself: the code values are pinned to hand-typed landmarks of the format, to its structure and to
torch's own conversion; the decode is pinned to a dense numpy evaluation on dequantised arrays,
to closed forms, and to the (already pinned) bf16 decode on pools that hold the same values."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2602_13692_amd import workloads as wl

D, PS = 128, 16
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e4m3_landmarks.txt")


def widen_bf16(u16):
    return (np.asarray(u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_bits_exact(x):
    f = np.asarray(x, dtype=np.float32)
    bits = f.view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0), "value not exactly representable in bf16"
    return (bits >> 16).astype(np.uint16)


def test_code_values_match_the_hand_typed_landmarks():
    """Catches a wrong bias, a wrong subnormal rule, a flipped sign, NaN mistaken for 480."""
    seen = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = line.split()
        code = int(parts[0], 16)
        got = float(oracle.widen_e4m3(np.array([code], np.uint8))[0])
        if parts[1] == "nan":
            assert math.isnan(got), hex(code)
        else:
            want = Fraction(int(parts[1]), int(parts[2]))
            assert Fraction(got) == want, (hex(code), got, want)
            if want == 0:
                assert math.copysign(1.0, got) == (-1.0 if code & 0x80 else 1.0)
        seen += 1
    assert seen >= 30


def test_code_values_have_the_structure_of_the_format():
    """All 256 codes: symmetric in the sign bit, strictly increasing over 0x00..0x7e, eight equal
    steps per binade that double from one binade to the next, exactly two NaNs, no infinities."""
    v = oracle.widen_e4m3(np.arange(256, dtype=np.uint8))
    pos, neg = v[:128], v[128:]
    assert np.isnan(pos[127]) and np.isnan(neg[127]) and np.isnan(v).sum() == 2
    assert np.all(np.isfinite(pos[:127])) and np.array_equal(neg[:127], -pos[:127])
    assert np.all(np.diff(pos[:127]) > 0)
    steps = np.diff(pos[:127])
    assert np.all(steps[:15] == 2.0 ** -9)                     # subnormals and the first binade share a step
    for e in range(1, 15):
        binade = steps[8 * e: 8 * e + 8]
        assert np.all(binade == 2.0 ** (e - 7 - 3)), e
    assert pos[126] == 448.0 and pos[8] == 2.0 ** -6


def test_code_values_match_torchs_own_conversion():
    """An independent implementation of the same format (torch.float8_e4m3fn -> float32)."""
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    got = oracle.widen_e4m3(codes.numpy())
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def _case(rng, B, Hq, Hkv, lens):
    lens = np.asarray(lens, np.int32)
    n_pages = (lens.astype(np.int64) + PS - 1) // PS
    P = int(n_pages.sum()) + 2
    table = wl.scatter_tables(rng, n_pages, rng.permutation(P).astype(np.int32), stride=int(n_pages.max()) + 1)
    f = rng.standard_normal((B, Hq, D)).astype(np.float32)
    bits = f.view(np.uint32)
    q = (((bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000) >> 16).astype(np.uint16)
    # finite codes only: 0x7f and 0xff are NaN
    k = rng.integers(0, 127, size=(P, Hkv, PS, D)).astype(np.uint8) | (rng.integers(0, 2, size=(P, Hkv, PS, D)) << 7).astype(np.uint8)
    v = rng.integers(0, 127, size=(P, Hkv, PS, D)).astype(np.uint8) | (rng.integers(0, 2, size=(P, Hkv, PS, D)) << 7).astype(np.uint8)
    # keep the scores moderate: codes of magnitude below 2 (exponent field <= 7)
    k = (k & 0x80) | np.minimum(k & 0x7f, 0x3f).astype(np.uint8)
    return q, k, v, table, lens


def _dequant(codes, scale):
    """torch's conversion (not the oracle's) times the scale, float64."""
    t = torch.from_numpy(np.ascontiguousarray(codes)).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    return t * float(np.float32(scale))


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 2), (8, 1), (8, 8)])
def test_fp8_decode_matches_dense_numpy_on_dequantised_arrays(Hq, Hkv):
    """Catches wrong indexing into the byte pools, a scale applied twice or to the wrong operand,
    K/V swapped, a wrong GQA map; boundary lengths around the page size."""
    rng = np.random.default_rng(wl.SEED_BASE + 2000 + Hq + Hkv)
    lens = [1, 15, 16, 17, 31, 33, 100]
    q, k, v, table, lens = _case(rng, len(lens), Hq, Hkv, lens)
    ks, vs = 0.021, 0.37
    out, lse = oracle.paged_decode_fp8(oracle.Geometry(Hq, Hkv), q, k, v, ks, vs, table, lens)
    kd, vd = _dequant(k, ks), _dequant(v, vs)
    G = Hq // Hkv
    for b, L in enumerate(lens):
        pages = table[b, : (L + PS - 1) // PS].astype(np.int64)
        for h in range(Hq):
            K = kd[pages, h // G].reshape(-1, D)[:L]
            V = vd[pages, h // G].reshape(-1, D)[:L]
            s = (K @ widen_bf16(q[b, h])) / math.sqrt(D)
            e = np.exp(s - s.max())
            ref = (e / e.sum()) @ V
            assert np.max(np.abs(out[b, h] - ref)) <= 1e-12 * max(1.0, np.abs(ref).max())
            assert abs(lse[b, h] - (s.max() + math.log(e.sum()))) <= 1e-12


def test_single_key_returns_the_scaled_value_row_exactly():
    rng = np.random.default_rng(wl.SEED_BASE + 2010)
    q, k, v, table, lens = _case(rng, 2, 2, 1, [1, 1])
    vs = 0.25                                                   # a power of two: code value * scale is exact
    out, lse = oracle.paged_decode_fp8(oracle.Geometry(2, 1), q, k, v, 0.5, vs, table, lens)
    for b in range(2):
        want = _dequant(v[table[b, 0], 0, 0], vs)
        assert np.array_equal(out[b, 0], want) and np.array_equal(out[b, 1], want)


def test_key_scale_multiplies_the_scores_and_value_scale_the_output():
    """Doubling k_scale equals doubling the softmax scale; doubling v_scale doubles the output and
    leaves lse alone.  Catches scales swapped or folded into the wrong place."""
    rng = np.random.default_rng(wl.SEED_BASE + 2020)
    q, k, v, table, lens = _case(rng, 3, 4, 2, [40, 7, 64])
    base = oracle.Geometry(4, 2)
    out1, lse1 = oracle.paged_decode_fp8(base, q, k, v, 0.03, 0.5, table, lens)
    out2, lse2 = oracle.paged_decode_fp8(oracle.Geometry(4, 2, scale=2.0 / math.sqrt(D)), q, k, v, 0.015, 0.5, table, lens)
    assert np.max(np.abs(out1 - out2)) <= 1e-13 and np.max(np.abs(lse1 - lse2)) <= 1e-13
    out3, lse3 = oracle.paged_decode_fp8(base, q, k, v, 0.03, 1.0, table, lens)
    assert np.array_equal(out3, 2.0 * out1) and np.array_equal(lse3, lse1)


def test_fp8_decode_equals_the_bf16_decode_on_pools_holding_the_same_values():
    """Every E4M3 value times a power-of-two scale is exactly a bf16 value, so the FP8 decode must
    agree bit for bit with the bf16 decode (pinned elsewhere) on pools filled with those values."""
    rng = np.random.default_rng(wl.SEED_BASE + 2030)
    lens = [1, 16, 17, 200, 333]
    q, k, v, table, lens = _case(rng, len(lens), 8, 2, lens)
    ks, vs = 2.0 ** -4, 2.0 ** 3
    k16 = bf16_bits_exact(_dequant(k, ks))
    v16 = bf16_bits_exact(_dequant(v, vs))
    geom = oracle.Geometry(8, 2)
    out8, lse8 = oracle.paged_decode_fp8(geom, q, k, v, ks, vs, table, lens)
    out16, lse16 = oracle.paged_decode(geom, q, k16, v16, table, lens)
    assert np.array_equal(out8, out16) and np.array_equal(lse8, lse16)


def test_nan_codes_in_unreadable_rows_change_nothing_and_empty_context_is_zero():
    rng = np.random.default_rng(wl.SEED_BASE + 2040)
    q, k, v, table, lens = _case(rng, 3, 2, 2, [5, 0, 20])
    geom = oracle.Geometry(2, 2)
    out, lse = oracle.paged_decode_fp8(geom, q, k, v, 0.02, 0.02, table, lens)
    k2, v2 = k.copy(), v.copy()
    k2[table[0, 0], :, 5:] = 0x7f
    v2[table[0, 0], :, 5:] = 0xff
    k2[table[2, 1], :, 4:] = 0x7f
    v2[table[2, 1], :, 4:] = 0x7f
    out2, lse2 = oracle.paged_decode_fp8(geom, q, k2, v2, 0.02, 0.02, table, lens)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
    assert np.all(out[1] == 0) and np.all(np.isneginf(lse[1]))


def test_the_generator_quantises_with_torchs_conversion_and_stays_in_range():
    wb = wl.llama8b_decode("cpu", seed=wl.SEED_BASE + 2050, batch=3, len_lo=10, len_hi=100, num_q_heads=4, num_kv_heads=2)
    fc = wl.to_fp8_cache(wb)
    kc = wl.as_u8(fc.k_codes)
    assert kc.dtype == np.uint8 and kc.shape == tuple(wb.k_pool.shape)
    assert not np.any((kc & 0x7f) == 0x7f)
    deq = _dequant(kc, fc.k_scale)
    ref = wb.k_pool.float().numpy().astype(np.float64)
    assert np.max(np.abs(deq - ref)) <= np.abs(ref).max() * 2.0 ** -4 + fc.k_scale      # half a step of 3 mantissa bits
