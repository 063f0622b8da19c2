"""Pins for the fp64 oracle: it is checked against things other than itself.

The paper prints no numeric example for attention, so every pin is what the
mathematics fixes: an independent numpy evaluation on contiguous arrays,
closed forms, invariants and a brute-force sweep over boundary sizes.  Each
test names the plausible mistake it is meant to catch.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2602_13692_amd import workloads as wl

D = 128
PS = 16


# ---------------------------------------------------------------------------
# helpers that do not touch the oracle's code
# ---------------------------------------------------------------------------

def widen(u16):
    """bf16 bit patterns -> float64, exactly."""
    return (np.asarray(u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_bf16_bits(x):
    """float array whose values are exactly representable in bf16 -> bit patterns."""
    f = np.asarray(x, dtype=np.float32)
    bits = f.view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0), "value not exactly representable in bf16"
    return (bits >> 16).astype(np.uint16)


def dense_reference(q_row, K, V, scale):
    """Textbook attention of one query against contiguous K, V (numpy float64)."""
    s = (K @ q_row) * scale
    e = np.exp(s - s.max())
    p = e / e.sum()
    return p @ V, s.max() + math.log(e.sum()), p


def gather_tokens(pool_u16, table_row, kv_head, n_tokens):
    """Contiguous [n_tokens, d] float64 view of one program's cached rows."""
    pages = np.asarray(table_row[: (n_tokens + PS - 1) // PS], dtype=np.int64)
    tile = widen(pool_u16[pages, kv_head])              # [pages, PS, d]
    return tile.reshape(-1, D)[:n_tokens]


def random_case(rng, B, Hq, Hkv, lens, q_lens=None, extra_pages=3, grid=None):
    """Small random batch as numpy arrays.  grid=k draws values as integers/k (exact in bf16)."""
    lens = np.asarray(lens, dtype=np.int32)
    q_lens = np.ones(B, np.int32) if q_lens is None else np.asarray(q_lens, np.int32)
    n_pages = (lens.astype(np.int64) + PS - 1) // PS
    P = int(n_pages.sum()) + extra_pages
    slots = rng.permutation(P).astype(np.int32)
    table = wl.scatter_tables(rng, n_pages, slots, stride=int(max(n_pages.max(), 1)) + 1)

    def draw(shape):
        if grid is None:
            f = rng.standard_normal(shape).astype(np.float32)
            bits = f.view(np.uint32)
            bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000   # round to nearest even
            return (bits >> 16).astype(np.uint16)
        return to_bf16_bits(rng.integers(-3 * grid, 3 * grid + 1, size=shape) / grid)

    q = draw((int(q_lens.sum()), Hq, D))
    k_pool = draw((P, Hkv, PS, D))
    v_pool = draw((P, Hkv, PS, D))
    return dict(geom=oracle.Geometry(Hq, Hkv), q=q, k_pool=k_pool, v_pool=v_pool,
                table=table, lens=lens, q_lens=q_lens, P=P)


def cu(q_lens):
    out = np.zeros(len(q_lens) + 1, dtype=np.int32)
    np.cumsum(q_lens, out=out[1:])
    return out


# ---------------------------------------------------------------------------
# P1 / P12: independent dense evaluation, boundary sizes, GQA mapping
# ---------------------------------------------------------------------------

def test_decode_matches_dense_numpy_on_tiny_config():
    """Catches wrong page/row indexing, a wrong GQA map, a missing scale, K/V swapped."""
    wb = wl.tiny_decode("cpu")
    q, kp, vp = wl.as_u16(wb.q), wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool)
    geom = oracle.Geometry(wb.num_q_heads, wb.num_kv_heads)
    out, lse = oracle.paged_decode(geom, q, kp, vp, wb.block_table, wb.context_lens)
    G = wb.num_q_heads // wb.num_kv_heads
    for b in range(wb.batch):
        L = int(wb.context_lens[b])
        for h in range(wb.num_q_heads):
            K = gather_tokens(kp, wb.block_table[b], h // G, L)
            V = gather_tokens(vp, wb.block_table[b], h // G, L)
            ref, ref_lse, _ = dense_reference(widen(q[b, h]), K, V, 1.0 / math.sqrt(D))
            assert np.max(np.abs(out[b, h] - ref)) <= 1e-12
            assert abs(lse[b, h] - ref_lse) <= 1e-12


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (2, 1), (2, 2), (8, 2)])
def test_boundary_sweep_decode_and_prefill(Hq, Hkv):
    """Brute force over lengths around page boundaries and small append sizes."""
    rng = np.random.default_rng(1234 + Hq * 10 + Hkv)
    G = Hq // Hkv
    for L in (1, 15, 16, 17, 31, 32, 33):
        for n in (1, 2, 17):
            if n > L:
                continue
            c = random_case(rng, 3, Hq, Hkv, [L, max(n, L - 1), L + 5], q_lens=[n, n, n])
            out, lse = oracle.append_prefill(c["geom"], c["q"], cu(c["q_lens"]), c["k_pool"],
                                             c["v_pool"], c["table"], c["lens"])
            t = 0
            for b in range(3):
                Lb = int(c["lens"][b])
                for i in range(n):
                    vis = Lb - n + i + 1
                    for h in range(Hq):
                        K = gather_tokens(c["k_pool"], c["table"][b], h // G, vis)
                        V = gather_tokens(c["v_pool"], c["table"][b], h // G, vis)
                        ref, ref_lse, _ = dense_reference(widen(c["q"][t, h]), K, V, 1 / math.sqrt(D))
                        assert np.max(np.abs(out[t, h] - ref)) <= 1e-12, (L, n, b, i, h)
                        assert abs(lse[t, h] - ref_lse) <= 1e-12
                    t += 1


def test_distinct_heads_read_distinct_kv_heads():
    """With Hkv = 2 the two groups must differ; with shuffled q heads outputs permute inside a group only."""
    rng = np.random.default_rng(5)
    c = random_case(rng, 1, 4, 2, [40])
    out, _ = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    q2 = c["q"].copy()
    q2[0, 2] = c["q"][0, 0]          # head 2 (group 1) gets head 0's query (group 0)
    out2, _ = oracle.paged_decode(c["geom"], q2, c["k_pool"], c["v_pool"], c["table"], c["lens"])
    assert not np.allclose(out2[0, 2], out[0, 0])     # same q, other kv head -> other result
    q3 = c["q"].copy()
    q3[0, 1] = c["q"][0, 0]          # head 1 shares group 0 with head 0
    out3, _ = oracle.paged_decode(c["geom"], q3, c["k_pool"], c["v_pool"], c["table"], c["lens"])
    assert np.array_equal(out3[0, 1], out[0, 0])


# ---------------------------------------------------------------------------
# golden: hand-computed rational case
# ---------------------------------------------------------------------------

def test_hand_computed_power_of_two_case():
    """exp/normalise and the p.v sum against exact rationals worked out by hand."""
    path = os.path.join(os.path.dirname(__file__), "golden", "power_of_two_softmax.txt")
    want = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, num, den = line.split()
        want[name] = Fraction(int(num), int(den))
    q = np.zeros((1, 1, D)); q[0, 0, 0] = 1.0
    k_pool = np.zeros((2, 1, PS, D)); v_pool = np.zeros((2, 1, PS, D))
    k_pool[1, 0, :4, 0] = [0, 1, 2, 3]
    v_pool[1, 0, 0, :4] = [1, 0, 2, -4]
    v_pool[1, 0, 1, :4] = [0, 1, 2, 8]
    v_pool[1, 0, 2, :4] = [0, 0, 2, -16]
    v_pool[1, 0, 3, :4] = [-1, 0, 2, 0.5]
    geom = oracle.Geometry(1, 1, scale=math.log(2.0))
    out, lse = oracle.paged_decode(geom, to_bf16_bits(q), to_bf16_bits(k_pool), to_bf16_bits(v_pool),
                                   np.array([[1]], np.int32), np.array([4], np.int32))
    for i in range(4):
        assert abs(out[0, 0, i] - float(want[f"out_{i}"])) <= 1e-15
    assert np.all(out[0, 0, 4:] == 0.0)
    assert abs(math.exp(lse[0, 0]) - float(want["exp_lse"])) <= 1e-13


# ---------------------------------------------------------------------------
# P2: page-pool permutation invariance (bit identical)
# ---------------------------------------------------------------------------

def test_page_permutation_is_bit_identical():
    rng = np.random.default_rng(7)
    c = random_case(rng, 3, 4, 2, [33, 100, 16], q_lens=[2, 5, 1])
    args = (c["geom"], c["q"], cu(c["q_lens"]))
    out, lse = oracle.append_prefill(*args, c["k_pool"], c["v_pool"], c["table"], c["lens"])
    perm = rng.permutation(c["P"])                      # old page p moves to slot perm[p]
    k2 = np.empty_like(c["k_pool"]); v2 = np.empty_like(c["v_pool"])
    k2[perm] = c["k_pool"]; v2[perm] = c["v_pool"]
    table2 = np.where(c["table"] >= 0, perm[np.maximum(c["table"], 0)], -1).astype(np.int32)
    out2, lse2 = oracle.append_prefill(*args, k2, v2, table2, c["lens"])
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)


# ---------------------------------------------------------------------------
# P3: single key returns V exactly; prefill token 0 with empty prefix
# ---------------------------------------------------------------------------

def test_single_key_returns_value_row_exactly():
    rng = np.random.default_rng(11)
    c = random_case(rng, 2, 4, 2, [1, 1])
    out, lse = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    for b in range(2):
        for h in range(4):
            v0 = widen(c["v_pool"][c["table"][b, 0], h // 2, 0])
            k0 = widen(c["k_pool"][c["table"][b, 0], h // 2, 0])
            assert np.array_equal(out[b, h], v0)
            s = float(np.dot(widen(c["q"][b, h]), k0)) / math.sqrt(D)
            assert abs(lse[b, h] - s) <= 1e-13


def test_prefill_first_token_with_empty_prefix_sees_only_itself():
    """Catches an off-by-one in the causal boundary (token i sees keys 0..prefix+i inclusive)."""
    rng = np.random.default_rng(12)
    c = random_case(rng, 1, 2, 1, [5], q_lens=[5])
    out, _ = oracle.append_prefill(c["geom"], c["q"], cu(c["q_lens"]), c["k_pool"], c["v_pool"],
                                   c["table"], c["lens"])
    v0 = widen(c["v_pool"][c["table"][0, 0], 0, 0])
    assert np.array_equal(out[0, 0], v0) and np.array_equal(out[0, 1], v0)
    # the second token sees exactly two keys
    K = gather_tokens(c["k_pool"], c["table"][0], 0, 2)
    V = gather_tokens(c["v_pool"], c["table"][0], 0, 2)
    ref, _, _ = dense_reference(widen(c["q"][1, 0]), K, V, 1 / math.sqrt(D))
    assert np.max(np.abs(out[1, 0] - ref)) <= 1e-14


# ---------------------------------------------------------------------------
# P4: probabilities
# ---------------------------------------------------------------------------

def test_probabilities_are_nonnegative_and_sum_to_one():
    rng = np.random.default_rng(13)
    for L in (1, 7, 100, 1000):
        c = random_case(rng, 1, 2, 1, [L])
        p, out, lse = oracle.row_probs(c["geom"], c["q"][0, 1], 1, c["k_pool"], c["v_pool"],
                                       c["table"][0], L)
        assert p.shape == (L,) and np.all(p >= 0.0)
        assert abs(p.sum() - 1.0) <= 1e-15 * max(L, 8)
        K = gather_tokens(c["k_pool"], c["table"][0], 0, L)
        V = gather_tokens(c["v_pool"], c["table"][0], 0, L)
        _, _, p_ref = dense_reference(widen(c["q"][0, 1]), K, V, 1 / math.sqrt(D))
        assert np.max(np.abs(p - p_ref)) <= 1e-14


# ---------------------------------------------------------------------------
# P5: closed forms
# ---------------------------------------------------------------------------

def test_zero_query_gives_mean_of_values():
    rng = np.random.default_rng(17)
    L = 37
    c = random_case(rng, 1, 2, 2, [L], grid=8)
    c["q"][:] = 0
    out, lse = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    for h in range(2):
        V = gather_tokens(c["v_pool"], c["table"][0], h, L)
        assert np.max(np.abs(out[0, h] - V.mean(axis=0))) <= 1e-14
        assert abs(lse[0, h] - math.log(L)) <= 1e-14


def test_identical_keys_give_mean_and_shifted_lse():
    rng = np.random.default_rng(18)
    L = 50
    c = random_case(rng, 1, 1, 1, [L])
    pages = c["table"][0, : (L + PS - 1) // PS]
    key = c["k_pool"][pages[0], 0, 0].copy()
    c["k_pool"][pages, 0, :, :] = key
    out, lse = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    V = gather_tokens(c["v_pool"], c["table"][0], 0, L)
    s = float(np.dot(widen(c["q"][0, 0]), widen(key))) / math.sqrt(D)
    assert np.max(np.abs(out[0, 0] - V.mean(axis=0))) <= 1e-13
    assert abs(lse[0, 0] - (s + math.log(L))) <= 1e-12


def test_two_keys_give_logistic_weights():
    rng = np.random.default_rng(19)
    c = random_case(rng, 1, 1, 1, [2])
    out, _ = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    K = gather_tokens(c["k_pool"], c["table"][0], 0, 2)
    V = gather_tokens(c["v_pool"], c["table"][0], 0, 2)
    s = K @ widen(c["q"][0, 0]) / math.sqrt(D)
    w0 = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
    assert np.max(np.abs(out[0, 0] - (w0 * V[0] + (1 - w0) * V[1]))) <= 1e-14


def test_scale_is_applied_once():
    """Doubling the scale equals doubling q (exact in bf16); catches a squared or missing scale."""
    rng = np.random.default_rng(20)
    c = random_case(rng, 1, 1, 1, [70], grid=8)
    g2 = oracle.Geometry(1, 1, scale=2.0 / math.sqrt(D))
    out_a, lse_a = oracle.paged_decode(g2, c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    q2 = to_bf16_bits(widen(c["q"]) * 2.0)
    out_b, lse_b = oracle.paged_decode(c["geom"], q2, c["k_pool"], c["v_pool"], c["table"], c["lens"])
    assert np.max(np.abs(out_a - out_b)) <= 1e-13 and np.max(np.abs(lse_a - lse_b)) <= 1e-12


# ---------------------------------------------------------------------------
# P6: shift invariance (max subtraction)
# ---------------------------------------------------------------------------

def test_key_shift_leaves_output_and_moves_lse():
    rng = np.random.default_rng(23)
    L = 90
    c = random_case(rng, 1, 1, 1, [L], grid=2)
    out, lse = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    shift = 32.0                                        # along coordinate 0; 32 + k/2 is exact in bf16
    k2 = widen(c["k_pool"]).copy()
    k2[..., 0] += shift
    out2, lse2 = oracle.paged_decode(c["geom"], c["q"], to_bf16_bits(k2), c["v_pool"], c["table"], c["lens"])
    q0 = float(widen(c["q"][0, 0, 0]))
    assert np.max(np.abs(out2 - out)) <= 1e-11
    assert abs((lse2[0, 0] - lse[0, 0]) - shift * q0 / math.sqrt(D)) <= 1e-11


def test_large_scores_do_not_overflow():
    """Scores of several hundred must not produce inf/nan (the max is subtracted before exp)."""
    c = random_case(np.random.default_rng(24), 1, 1, 1, [40], grid=1)
    g = oracle.Geometry(1, 1, scale=50.0)
    out, lse = oracle.paged_decode(g, c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))


# ---------------------------------------------------------------------------
# P7: split-and-merge algebra
# ---------------------------------------------------------------------------

def test_split_key_axis_and_merge_equals_whole():
    """The (max, sum, weighted output) merge identity that any split-K scheme relies on."""
    rng = np.random.default_rng(29)
    L = 300
    c = random_case(rng, 1, 2, 1, [L])
    out, lse = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    for a in (1, 16, 137, 299):
        for h in range(2):
            qv = widen(c["q"][0, h])
            K = gather_tokens(c["k_pool"], c["table"][0], 0, L)
            V = gather_tokens(c["v_pool"], c["table"][0], 0, L)
            # first part through the oracle itself (keys 0..a-1), second part dense
            o1, l1 = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"],
                                         np.array([a], np.int32))
            o1, l1 = o1[0, h], l1[0, h]
            o2, l2, _ = dense_reference(qv, K[a:], V[a:], 1 / math.sqrt(D))
            m = max(l1, l2)
            w1, w2 = math.exp(l1 - m), math.exp(l2 - m)
            merged = (w1 * o1 + w2 * o2) / (w1 + w2)
            assert np.max(np.abs(merged - out[0, h])) <= 1e-12
            assert abs(m + math.log(w1 + w2) - lse[0, h]) <= 1e-12


# ---------------------------------------------------------------------------
# P8: causal consistency between the two entry points
# ---------------------------------------------------------------------------

def test_prefill_row_equals_decode_with_truncated_context():
    rng = np.random.default_rng(31)
    n, L = 19, 83
    c = random_case(rng, 2, 4, 2, [L, L - 7], q_lens=[n, n])
    out, lse = oracle.append_prefill(c["geom"], c["q"], cu(c["q_lens"]), c["k_pool"], c["v_pool"],
                                     c["table"], c["lens"])
    for b in range(2):
        for i in (0, 1, n // 2, n - 1):
            t = b * n + i
            vis = int(c["lens"][b]) - n + i + 1
            lens = c["lens"].copy(); lens[b] = vis
            qd = np.zeros((2, 4, D), np.uint16); qd[b] = c["q"][t]
            od, ld = oracle.paged_decode(c["geom"], qd, c["k_pool"], c["v_pool"], c["table"], lens)
            assert np.array_equal(od[b], out[t]) and np.array_equal(ld[b], lse[t])


def test_attend_rows_matches_full_calls():
    rng = np.random.default_rng(32)
    c = random_case(rng, 3, 4, 2, [40, 64, 9], q_lens=[3, 10, 9])
    cuq = cu(c["q_lens"])
    out, lse = oracle.append_prefill(c["geom"], c["q"], cuq, c["k_pool"], c["v_pool"], c["table"], c["lens"])
    rows = [(0, 2, 1), (1, 0, 3), (1, 9, 0), (2, 4, 2)]
    rb = [r[0] for r in rows]
    rt = [int(cuq[r[0]]) + r[1] for r in rows]
    rh = [r[2] for r in rows]
    vis = [int(c["lens"][r[0]]) - int(c["q_lens"][r[0]]) + r[1] + 1 for r in rows]
    o2, l2 = oracle.attend_rows(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], rb, rt, rh, vis)
    for k, (b, i, h) in enumerate(rows):
        assert np.array_equal(o2[k], out[rt[k], h]) and l2[k] == lse[rt[k], h]


# ---------------------------------------------------------------------------
# P9: padding poison, C-6 empty rows
# ---------------------------------------------------------------------------

def test_nan_in_unreadable_rows_changes_nothing():
    wb = wl.llama8b_decode("cpu", batch=5, len_lo=1, len_hi=70, num_q_heads=4, num_kv_heads=2)
    geom = oracle.Geometry(4, 2)
    base = oracle.paged_decode(geom, wl.as_u16(wb.q), wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool),
                               wb.block_table, wb.context_lens)
    wl.poison_padding(wb)
    kp = wl.as_u16(wb.k_pool)
    assert np.isnan(widen(kp)).any() or np.all(wb.context_lens % PS == 0)
    again = oracle.paged_decode(geom, wl.as_u16(wb.q), kp, wl.as_u16(wb.v_pool),
                                wb.block_table, wb.context_lens)
    assert np.array_equal(base[0], again[0]) and np.array_equal(base[1], again[1])
    assert np.all(np.isfinite(again[0]))


def test_empty_context_gives_zero_row_and_minus_inf():
    rng = np.random.default_rng(37)
    c = random_case(rng, 2, 2, 1, [0, 5])
    out, lse = oracle.paged_decode(c["geom"], c["q"], c["k_pool"], c["v_pool"], c["table"], c["lens"])
    assert np.all(out[0] == 0.0) and np.all(np.isneginf(lse[0])) and np.all(np.isfinite(lse[1]))


# ---------------------------------------------------------------------------
# P10: aliased block tables (forked programs)
# ---------------------------------------------------------------------------

def test_forked_programs_share_prefix_pages():
    wb = wl.forked_decode("cpu", batch=8, group=4, prefix_len=64, suffix_lo=1, suffix_hi=40,
                          num_q_heads=4, num_kv_heads=2)
    assert np.array_equal(wb.block_table[0, :4], wb.block_table[3, :4])
    assert not np.array_equal(wb.block_table[0, :4], wb.block_table[4, :4])
    q = wl.as_u16(wb.q).copy()
    q[1] = q[0]
    table = wb.block_table.copy(); lens = wb.context_lens.copy()
    table[1] = table[0]; lens[1] = lens[0]
    geom = oracle.Geometry(4, 2)
    out, lse = oracle.paged_decode(geom, q, wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool), table, lens)
    assert np.array_equal(out[0], out[1]) and np.array_equal(lse[0], lse[1])
    # truncated to the shared prefix, members of a group differ only through q
    lens[:] = 64
    q[2] = q[0]
    out, _ = oracle.paged_decode(geom, q, wl.as_u16(wb.k_pool), wl.as_u16(wb.v_pool), wb.block_table, lens)
    assert np.array_equal(out[0], out[2]) and not np.array_equal(out[0], out[3])


# ---------------------------------------------------------------------------
# P11: restore
# ---------------------------------------------------------------------------

def test_restore_scatters_exact_bytes_and_touches_nothing_else():
    rng = np.random.default_rng(41)
    P, page_bytes, n = 23, 2 * PS * D * 2, 9
    k_pool = rng.integers(0, 256, size=(P, page_bytes), dtype=np.uint8)
    v_pool = rng.integers(0, 256, size=(P, page_bytes), dtype=np.uint8)
    k0, v0 = k_pool.copy(), v_pool.copy()
    host_k = rng.integers(0, 256, size=(n, page_bytes), dtype=np.uint8)
    host_v = rng.integers(0, 256, size=(n, page_bytes), dtype=np.uint8)
    dst = rng.choice(P, size=n, replace=False).astype(np.int32)
    assert oracle.kv_page_restore(k_pool, v_pool, page_bytes, host_k, host_v, dst, P) == 0
    untouched = np.setdiff1d(np.arange(P), dst)
    assert np.array_equal(k_pool[dst], host_k) and np.array_equal(v_pool[dst], host_v)
    assert np.array_equal(k_pool[untouched], k0[untouched]) and np.array_equal(v_pool[untouched], v0[untouched])


def test_restore_rejects_bad_slot_lists_without_writing():
    P, page_bytes = 4, 64
    k_pool = np.zeros((P, page_bytes), np.uint8); v_pool = np.zeros((P, page_bytes), np.uint8)
    host = np.ones((2, page_bytes), np.uint8)
    for bad in ([0, 0], [1, 4], [-1, 2]):
        assert oracle.kv_page_restore(k_pool, v_pool, page_bytes, host, host, np.array(bad, np.int32), P) == -1
        assert not k_pool.any() and not v_pool.any()


def test_evict_restore_round_trip_keeps_decode_result():
    """Pages moved to other slots (and block tables rewritten) give the bit-identical decode."""
    wb = wl.long_horizon_restore("cpu", batch=6, median=60, sigma=0.5, len_lo=5, len_cap=200,
                                 restore_frac=0.5, num_q_heads=4, num_kv_heads=2)
    geom = oracle.Geometry(4, 2)
    kp, vp = wl.as_u16(wb.k_pool).copy(), wl.as_u16(wb.v_pool).copy()
    page_bytes = 2 * PS * D * 2
    rs = wb.restore
    rc = oracle.kv_page_restore(kp.view(np.uint8).reshape(wb.pool_pages, page_bytes),
                                vp.view(np.uint8).reshape(wb.pool_pages, page_bytes), page_bytes,
                                wl.as_u16(rs.host_k).view(np.uint8).reshape(-1, page_bytes),
                                wl.as_u16(rs.host_v).view(np.uint8).reshape(-1, page_bytes),
                                rs.dst_slots, wb.pool_pages)
    assert rc == 0
    out, lse = oracle.paged_decode(geom, wl.as_u16(wb.q), kp, vp, wb.block_table, wb.context_lens)
    # the same programs with their restored pages laid out contiguously in a fresh pool
    hk, hv = wl.as_u16(rs.host_k), wl.as_u16(rs.host_v)
    off = 0
    for b in rs.programs:
        L = int(wb.context_lens[b]); npg = (L + PS - 1) // PS
        table = np.arange(npg, dtype=np.int32)[None, :]
        o, l = oracle.paged_decode(geom, wl.as_u16(wb.q)[b:b + 1], hk[off:off + npg], hv[off:off + npg],
                                   table, np.array([L], np.int32))
        assert np.array_equal(o[0], out[b]) and np.array_equal(l[0], lse[b])
        off += npg


# ---------------------------------------------------------------------------
# evict (the inverse of restore) and append (the cache grows at its tail)
# ---------------------------------------------------------------------------

def test_evict_gathers_exact_bytes_and_leaves_the_pool_alone():
    rng = np.random.default_rng(43)
    P, page_bytes, n = 19, 2 * PS * D * 2, 11
    k_pool = rng.integers(0, 256, size=(P, page_bytes), dtype=np.uint8)
    v_pool = rng.integers(0, 256, size=(P, page_bytes), dtype=np.uint8)
    k0, v0 = k_pool.copy(), v_pool.copy()
    src = rng.integers(0, P, size=n).astype(np.int32)          # repeats allowed
    host_k = np.zeros((n, page_bytes), np.uint8)
    host_v = np.zeros((n, page_bytes), np.uint8)
    assert oracle.kv_page_evict(k_pool, v_pool, page_bytes, host_k, host_v, src, P) == 0
    assert np.array_equal(host_k, k0[src]) and np.array_equal(host_v, v0[src])     # numpy fancy indexing
    assert np.array_equal(k_pool, k0) and np.array_equal(v_pool, v0)
    for bad in ([0, P], [-1, 2]):
        hk = np.zeros((2, page_bytes), np.uint8)
        assert oracle.kv_page_evict(k_pool, v_pool, page_bytes, hk, hk.copy(), np.array(bad, np.int32), P) == -1
        assert not hk.any()


def test_evict_then_restore_elsewhere_is_the_identity_on_contents():
    rng = np.random.default_rng(44)
    P, page_bytes, n = 16, 256, 6
    k_pool = rng.integers(0, 256, size=(P, page_bytes), dtype=np.uint8)
    v_pool = rng.integers(0, 256, size=(P, page_bytes), dtype=np.uint8)
    src = rng.choice(P, size=n, replace=False).astype(np.int32)
    host_k = np.zeros((n, page_bytes), np.uint8)
    host_v = np.zeros((n, page_bytes), np.uint8)
    assert oracle.kv_page_evict(k_pool, v_pool, page_bytes, host_k, host_v, src, P) == 0
    k2, v2 = np.zeros_like(k_pool), np.zeros_like(v_pool)
    dst = rng.choice(P, size=n, replace=False).astype(np.int32)
    assert oracle.kv_page_restore(k2, v2, page_bytes, host_k, host_v, dst, P) == 0
    assert np.array_equal(k2[dst], k_pool[src]) and np.array_equal(v2[dst], v_pool[src])


@pytest.mark.parametrize("Hkv", [1, 2])
def test_append_writes_the_tail_rows_and_nothing_else(Hkv):
    """Checked against direct numpy indexing of the [P][Hkv][16][d] pool."""
    rng = np.random.default_rng(45 + Hkv)
    lens = np.array([1, 16, 17, 40, 33], np.int32)            # after the append
    n_new = np.array([1, 3, 17, 0, 20], np.int32)             # one token, a page boundary, a whole context, none
    c = random_case(rng, 5, 2 * Hkv, Hkv, lens)
    total = int(n_new.sum())
    new_k = rng.integers(0, 65536, size=(total, Hkv, D)).astype(np.uint16)
    new_v = rng.integers(0, 65536, size=(total, Hkv, D)).astype(np.uint16)
    kp, vp = c["k_pool"].copy(), c["v_pool"].copy()
    oracle.kv_append(c["geom"], new_k, new_v, cu(n_new), kp, vp, c["table"], lens)
    want_k, want_v = c["k_pool"].copy(), c["v_pool"].copy()
    row = 0
    for b in range(5):
        for i in range(int(n_new[b])):
            tok = int(lens[b] - n_new[b] + i)
            page = int(c["table"][b, tok // PS])
            want_k[page, :, tok % PS, :] = new_k[row]
            want_v[page, :, tok % PS, :] = new_v[row]
            row += 1
    assert np.array_equal(kp, want_k) and np.array_equal(vp, want_v)
    assert not np.array_equal(kp, c["k_pool"])


def test_append_then_attend_equals_attending_a_pool_filled_directly():
    """The precondition of append-prefill (new K/V already in their pages) is what append produces."""
    rng = np.random.default_rng(47)
    lens = np.array([37, 20, 64], np.int32)
    n_new = np.array([5, 20, 1], np.int32)
    c = random_case(rng, 3, 4, 2, lens, q_lens=n_new)
    geom = c["geom"]
    ref_out, ref_lse = oracle.append_prefill(geom, c["q"], cu(n_new), c["k_pool"], c["v_pool"], c["table"], lens)
    # pull the new tokens' rows out of the full pool, blank them, append them again
    kp, vp = c["k_pool"].copy(), c["v_pool"].copy()
    new_k = np.zeros((int(n_new.sum()), 2, D), np.uint16)
    new_v = np.zeros_like(new_k)
    row = 0
    for b in range(3):
        for i in range(int(n_new[b])):
            tok = int(lens[b] - n_new[b] + i)
            page = int(c["table"][b, tok // PS])
            new_k[row] = kp[page, :, tok % PS, :]
            new_v[row] = vp[page, :, tok % PS, :]
            kp[page, :, tok % PS, :] = 0x7FC0     # NaN until appended
            vp[page, :, tok % PS, :] = 0x7FC0
            row += 1
    oracle.kv_append(geom, new_k, new_v, cu(n_new), kp, vp, c["table"], lens)
    assert np.array_equal(kp, c["k_pool"]) and np.array_equal(vp, c["v_pool"])
    out, lse = oracle.append_prefill(geom, c["q"], cu(n_new), kp, vp, c["table"], lens)
    assert np.array_equal(out, ref_out) and np.array_equal(lse, ref_lse)


# ---------------------------------------------------------------------------
# workload generators: structure only
# ---------------------------------------------------------------------------

def test_generators_are_seeded_and_well_formed():
    a = wl.llama8b_decode("cpu", batch=6, len_lo=10, len_hi=300)
    b = wl.llama8b_decode("cpu", batch=6, len_lo=10, len_hi=300)
    assert np.array_equal(a.block_table, b.block_table) and np.array_equal(wl.as_u16(a.q), wl.as_u16(b.q))
    used = a.block_table[a.block_table >= 0]
    assert used.size == np.unique(used).size == a.pool_pages == a.unique_pages
    t = wl.tiny_decode("cpu")
    assert list(t.context_lens) == [64, 128, 256, 512] and t.pool_pages == 64 and t.unique_pages == 60
    p = wl.append_prefill("cpu", batch=4, new_lo=3, new_hi=20, prefix_lo=10, prefix_hi=50,
                          num_q_heads=4, num_kv_heads=2)
    assert p.total_q == int(p.q_lens.sum()) == p.q.shape[0]
    assert np.all(p.context_lens > p.q_lens)
    r = wl.long_horizon_restore("cpu", batch=10, median=80, sigma=0.75, len_lo=8, len_cap=300,
                                num_q_heads=4, num_kv_heads=2)
    resident = np.setdiff1d(np.arange(10), r.restore.programs)
    res_pages = np.concatenate([r.block_table[b][r.block_table[b] >= 0] for b in resident])
    assert np.intersect1d(res_pages, r.restore.dst_slots).size == 0
    assert np.unique(r.restore.dst_slots).size == r.restore.dst_slots.size
    f = wl.forked_decode("cpu", batch=8, group=4, prefix_len=32, suffix_lo=1, suffix_hi=20,
                         num_q_heads=8, num_kv_heads=2)
    assert f.unique_tokens() == 2 * 32 + int((f.context_lens - 32).sum())
