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


# ---- writing an FP8 cache: the quantiser and the quantising append ----
# The reading (nearest E4M3 value of x / scale taken in fp32, ties to the even code, saturation at
# +-448, NaN kept) is pinned by the format's own structure -- every code maps to itself, every
# midpoint of two neighbours goes to the even one, a hair to either side of a midpoint goes to the
# nearer one -- by hand cases of the saturation rule, and by torch's own conversion on every bf16
# value in range.

def _finite_positive_values():
    """The 127 positive finite values in code order, from the landmark-pinned, torch-pinned widening."""
    return oracle.widen_e4m3(np.arange(127, dtype=np.uint8))


def test_every_code_is_the_quantisation_of_its_own_value():
    codes = np.array([c for c in range(256) if c & 0x7f != 0x7f], np.uint8)
    values = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()      # torch's widening, exact in fp32
    assert np.array_equal(oracle.quantise_e4m3(values, 1.0), codes)                  # -0 keeps its sign: 0x80
    # and with a scale that is a power of two the division is exact as well
    assert np.array_equal(oracle.quantise_e4m3(values * np.float32(0.25), 0.25), codes)


def test_midpoints_go_to_the_even_code_and_their_neighbourhood_to_the_nearer_one():
    v = _finite_positive_values()
    mid = ((v[:-1] + v[1:]) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (v[:-1] + v[1:]) / 2), "midpoints are exact in fp32"
    lower = np.arange(126, dtype=np.uint8)
    even = np.where(lower % 2 == 0, lower, lower + 1).astype(np.uint8)
    assert np.array_equal(oracle.quantise_e4m3(mid, 1.0), even)
    assert np.array_equal(oracle.quantise_e4m3(-mid, 1.0), even | 0x80)
    below = np.nextafter(mid, np.float32(0))
    above = np.nextafter(mid, np.float32(np.inf))
    assert np.array_equal(oracle.quantise_e4m3(below, 1.0), lower)
    assert np.array_equal(oracle.quantise_e4m3(above, 1.0), lower + 1)


def test_saturation_nan_and_signed_zero_by_hand():
    x = np.array([448.0, 449.0, 464.0, 465.0, 480.0, 1e30, np.inf, -448.0, -449.0, -np.inf, np.nan, 0.0, -0.0,
                  2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -11, -2.0 ** -10], np.float32)
    want = [0x7e, 0x7e, 0x7e, 0x7e, 0x7e, 0x7e, 0x7e, 0xfe, 0xfe, 0xfe, 0x7f, 0x00, 0x80,
            0x00, 0x01, 0x00, 0x80]     # half the smallest subnormal ties to the even code 0; just above it rounds up
    got = oracle.quantise_e4m3(x, 1.0)
    assert [int(g) & 0x7f if math.isnan(float(v)) else int(g) for g, v in zip(got, x)] == want


def test_quantiser_is_monotone():
    rng = np.random.default_rng(wl.SEED_BASE + 830)
    x = np.sort(np.concatenate([rng.standard_normal(20000) * 100, rng.standard_normal(20000) * 0.01]).astype(np.float32))
    codes = oracle.quantise_e4m3(x, 1.0).astype(np.int32)
    signed = np.where(codes & 0x80, -(codes & 0x7f), codes & 0x7f)
    assert np.all(np.diff(signed) >= 0)


@pytest.mark.parametrize("scale", [1.0, 0.021, 0.017, 3.0, 2.0 ** -7])
def test_quantiser_matches_torchs_conversion_on_every_bf16_value_in_range(scale):
    """All 65536 bf16 bit patterns: x / scale in fp32 (the same division on both sides), then torch's
    float8_e4m3fn conversion.  Compared where the quotient is within the format's range (beyond it
    torch makes NaN and the reading here saturates: covered by hand above)."""
    bits = np.arange(65536, dtype=np.uint32)
    x = (bits << 16).view(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        q = x / np.float32(scale)
    in_range = np.isfinite(q) & (np.abs(q) <= 448.0)
    want = (torch.from_numpy(x) / torch.tensor(scale, dtype=torch.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.quantise_e4m3(x, scale)
    assert np.array_equal(got[in_range], want[in_range])
    assert in_range.sum() > 30000


def test_fp8_append_equals_direct_indexing_of_quantised_rows():
    rng = np.random.default_rng(wl.SEED_BASE + 831)
    Hkv, B = 2, 4
    new = np.array([1, 16, 37, 0], np.int32)
    lens = np.array([1, 50, 37, 12], np.int32)                  # the first and third programs are all new
    n_pages = (lens.astype(np.int64) + PS - 1) // PS
    P = int(n_pages.sum()) + 3
    table = wl.scatter_tables(rng, n_pages, rng.permutation(P).astype(np.int32), stride=int(n_pages.max()) + 2)
    cu = np.zeros(B + 1, np.int32); np.cumsum(new, out=cu[1:])
    f = (rng.standard_normal((int(cu[-1]), Hkv, D)) * 3).astype(np.float32)
    bits = f.view(np.uint32)
    new_k = (((bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000) >> 16).astype(np.uint16)
    new_v = new_k[::-1].copy()
    k_pool = rng.integers(0, 256, size=(P, Hkv, PS, D)).astype(np.uint8)
    v_pool = rng.integers(0, 256, size=(P, Hkv, PS, D)).astype(np.uint8)
    want_k, want_v = k_pool.copy(), v_pool.copy()
    ks, vs = 0.05, 0.031
    qk = oracle.quantise_e4m3(widen_bf16(new_k).astype(np.float32), ks)       # the quantiser is pinned above
    qv = oracle.quantise_e4m3(widen_bf16(new_v).astype(np.float32), vs)
    for b in range(B):
        for i in range(int(new[b])):
            token = int(lens[b] - new[b]) + i
            page, row = int(table[b, token // PS]), token % PS
            want_k[page, :, row, :] = qk[cu[b] + i]
            want_v[page, :, row, :] = qv[cu[b] + i]
    oracle.kv_append_fp8(oracle.Geometry(8, Hkv), new_k, new_v, cu, k_pool, v_pool, ks, vs, table, lens)
    assert np.array_equal(k_pool, want_k) and np.array_equal(v_pool, want_v)
    assert not np.array_equal(want_k, want_v)


# ---- append-prefill over an FP8 cache ----

def _prefill_case(rng, Hq, Hkv, new, prefix):
    new, prefix = np.asarray(new, np.int32), np.asarray(prefix, np.int32)
    lens = (new + prefix).astype(np.int32)
    B = len(lens)
    _, k, v, table, lens = _case(rng, B, Hq, Hkv, lens)
    cu = np.zeros(B + 1, np.int32); np.cumsum(new, out=cu[1:])
    f = rng.standard_normal((int(cu[-1]), Hq, D)).astype(np.float32)
    bits = f.view(np.uint32)
    q = (((bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000) >> 16).astype(np.uint16)
    return q, cu, k, v, table, lens


@pytest.mark.parametrize("Hq,Hkv", [(2, 1), (8, 2), (4, 4)])
def test_fp8_prefill_matches_dense_numpy_with_a_causal_mask(Hq, Hkv):
    """New token i of a program sees its prefix and the new tokens 0 .. i (itself included): dense
    numpy attention over the dequantised arrays (torch's widening), one row at a time."""
    rng = np.random.default_rng(wl.SEED_BASE + 2100 + Hq)
    new, prefix = [1, 3, 17, 2, 0], [0, 14, 20, 100, 5]
    q, cu, k, v, table, lens = _prefill_case(rng, Hq, Hkv, new, prefix)
    ks, vs = 0.03, 0.4
    out, lse = oracle.append_prefill_fp8(oracle.Geometry(Hq, Hkv), q, cu, k, v, ks, vs, table, lens)
    assert out.shape == (int(cu[-1]), Hq, D)
    kd, vd = _dequant(k, ks), _dequant(v, vs)
    G = Hq // Hkv
    for b in range(len(new)):
        L = int(lens[b])
        pages = table[b, : (L + PS - 1) // PS].astype(np.int64)
        for i in range(new[b]):
            visible = prefix[b] + i + 1
            for h in range(Hq):
                K = kd[pages, h // G].reshape(-1, D)[:visible]
                V = vd[pages, h // G].reshape(-1, D)[:visible]
                s = (K @ widen_bf16(q[cu[b] + i, h])) / math.sqrt(D)
                e = np.exp(s - s.max())
                ref = (e / e.sum()) @ V
                assert np.max(np.abs(out[cu[b] + i, h] - ref)) <= 1e-12 * max(1.0, np.abs(ref).max())
                assert abs(lse[cu[b] + i, h] - (s.max() + math.log(e.sum()))) <= 1e-12


def test_fp8_prefill_rows_equal_fp8_decodes_of_the_growing_context():
    """Row i of a program is what the (separately pinned) FP8 decode gives for a context of
    prefix + i + 1 tokens and the same query: bit-identical, both walk the same steps."""
    rng = np.random.default_rng(wl.SEED_BASE + 2110)
    Hq, Hkv = 4, 2
    new, prefix = [5, 18], [30, 0]
    q, cu, k, v, table, lens = _prefill_case(rng, Hq, Hkv, new, prefix)
    ks, vs = 0.021, 0.017
    out, lse = oracle.append_prefill_fp8(oracle.Geometry(Hq, Hkv), q, cu, k, v, ks, vs, table, lens)
    for b in range(2):
        for i in range(new[b]):
            one, one_lse = oracle.paged_decode_fp8(oracle.Geometry(Hq, Hkv), q[cu[b] + i][None], k, v, ks, vs,
                                                   table[b][None], np.array([prefix[b] + i + 1], np.int32))
            assert np.array_equal(one[0], out[cu[b] + i]) and np.array_equal(one_lse[0], lse[cu[b] + i])


def test_fp8_prefill_ignores_nan_codes_behind_the_causal_boundary():
    rng = np.random.default_rng(wl.SEED_BASE + 2120)
    Hq, Hkv = 2, 1
    q, cu, k, v, table, lens = _prefill_case(rng, Hq, Hkv, [6], [10])
    want = oracle.append_prefill_fp8(oracle.Geometry(Hq, Hkv), q, cu, k, v, 0.05, 0.05, table, lens)
    # the LAST new token's key and value only matter to itself: NaN there must leave rows 0 .. 4 alone
    page, row = int(table[0, 15 // PS]), 15 % PS
    k[page, :, row, :] = 0x7f
    v[page, :, row, :] = 0xff
    got = oracle.append_prefill_fp8(oracle.Geometry(Hq, Hkv), q, cu, k, v, 0.05, 0.05, table, lens)
    assert np.array_equal(got[0][:5], want[0][:5]) and np.array_equal(got[1][:5], want[1][:5])
    assert np.all(np.isnan(got[0][5]))
