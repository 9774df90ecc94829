"""Pins for the CPU oracle: closed forms, invariants, brute force and library routines.

None of these re-type the oracle's loops: each expected value comes from a different
formulation (numpy matmul on one slot at a time, an explicit dense W' = W + s*B*A, an outer
product, python's sorted(), torch's bf16 cast) or from an invariant that a dropped term, a wrong
sign/index or a transposed operand would break.
"""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.timeout(300)


def f64(bits):
    """Independent bf16-bits -> float64 (numpy bit view, not the oracle's helper)."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def ints_bf16(g, shape, lo=-4, hi=5):
    """Small integers as bf16 bits (exactly representable, so fp64 sums are exact)."""
    return W.to_bf16_bits(g.integers(lo, hi, size=shape).astype(np.float32))


# ---------------------------------------------------------------- bf16 helpers

def test_bf16_widen_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.bf16_to_f64(bits)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[np.isinf(want)], want[np.isinf(want)])


def test_bf16_round_trip_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    vals = f64(bits)
    keep = ~np.isnan(vals)
    assert np.array_equal(oracle.round_to_bf16(vals[keep]), bits[keep])


def test_bf16_rne_against_torch_and_hand_picked_ties(oracle):
    g = W.rng(7)
    v = np.concatenate([
        g.standard_normal(200000), g.standard_normal(50000) * 1e-3, g.standard_normal(50000) * 1e4,
        g.standard_normal(1000) * 1e-39])
    v = v.astype(np.float32).astype(np.float64)      # torch rounds from fp32, so start there
    want = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.round_to_bf16(v), want)
    # exact halves between neighbours: 1 + 2^-8 ties to even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 2 + 2.0 ** -7,
                     1 + 2.0 ** -8 + 2.0 ** -40, 1 + 2.0 ** -8 - 2.0 ** -40])
    want = np.array([0x3F80, 0x3F82, 0xBF80, 0x4000, 0x3F81, 0x3F80], dtype=np.uint16)
    assert np.array_equal(oracle.round_to_bf16(ties), want)
    # a double that a detour through fp32 would round the wrong way (double rounding)
    v = np.array([1 + 2.0 ** -8 + 2.0 ** -30])
    assert oracle.round_to_bf16(v)[0] == 0x3F81


# ---------------------------------------------------------------- decode: closed forms

def small(seed, T=12, d_in=24, d_out=16, S=3, r=4, alpha=8.0, **kw):
    return W.dense_case("small", seed, T, d_in, d_out, S, r, alpha, **kw)


def numpy_per_slot(c):
    """Library-routine formulation: one matmul pair per slot over the rows that use it."""
    x, y, A, B = f64(c.x), f64(c.y0).copy(), f64(c.A), f64(c.B)
    for s in range(c.n_slots):
        r = int(c.rank[s])
        rows = np.nonzero(c.token_slot == s)[0]
        if r == 0 or rows.size == 0:
            continue
        y[rows] += (c.alpha[s] / r) * (x[rows] @ A[s, :r].T) @ B[s, :, :r].T
    return y


def test_decode_matches_numpy_matmul(oracle):
    for seed, kw in [(1, {}), (2, dict(T=33, d_in=40, d_out=56, S=5, r=8, alpha=16.0)),
                     (3, dict(T=7, d_in=8, d_out=8, S=2, r=1, alpha=1.0))]:
        c = small(seed, **kw)
        got = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        np.testing.assert_allclose(got, numpy_per_slot(c), rtol=1e-12, atol=1e-13)


def test_dense_brute_force_exact(oracle):
    """Tiny integers, alpha/r a power of two: x W'^T with W' = W + (alpha/r) B A must equal
    x W^T + delta with zero error, for every slot."""
    g = W.rng(11)
    T, d_in, d_out, S, r = 6, 8, 7, 3, 2
    x, Wd = ints_bf16(g, (T, d_in)), g.integers(-3, 4, size=(d_out, d_in)).astype(np.float64)
    A, B = ints_bf16(g, (S, r, d_in), -2, 3), ints_bf16(g, (S, d_out, r), -2, 3)
    alpha = np.array([4.0, 1.0, 8.0])                      # alpha/r = 2, 0.5, 4
    slots = np.array([0, 1, 2, 0, 1, 2], dtype=np.int32)
    base = f64(x) @ Wd.T                                   # small integers: exact in bf16
    y0 = W.to_bf16_bits(base.astype(np.float32))
    assert np.array_equal(f64(y0), base)
    got = oracle.apply_decode(x, y0, A, B, np.full(S, r), alpha, slots)
    for t in range(T):
        s = slots[t]
        Wp = Wd + (alpha[s] / r) * f64(B[s]) @ f64(A[s])   # [d_out, d_in]
        assert np.array_equal(got[t], Wp @ f64(x[t]))


def test_rank1_outer_product(oracle):
    c = small(21, T=9, d_in=32, d_out=24, S=4, r=1, alpha=3.0)
    got = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    x, y, A, B = f64(c.x), f64(c.y0), f64(c.A), f64(c.B)
    for t in range(c.T):
        s = c.token_slot[t]
        want = y[t] if s < 0 else y[t] + 3.0 * np.dot(x[t], A[s, 0]) * B[s, :, 0]
        np.testing.assert_allclose(got[t], want, rtol=1e-13, atol=1e-14)


def test_zero_B_or_zero_A_leaves_y_bitwise(oracle):
    c = small(31)
    y = f64(c.y0)
    assert np.array_equal(oracle.apply_decode(c.x, c.y0, c.A, np.zeros_like(c.B), c.rank, c.alpha, c.token_slot), y)
    assert np.array_equal(oracle.apply_decode(c.x, c.y0, np.zeros_like(c.A), c.B, c.rank, c.alpha, c.token_slot), y)


def test_minus_one_and_empty_slot_rows_untouched(oracle):
    c = small(41, T=20)
    c.token_slot[::3] = -1
    got = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    assert np.array_equal(got[::3], f64(c.y0)[::3])
    assert not np.array_equal(got[c.token_slot >= 0], f64(c.y0)[c.token_slot >= 0])
    allm = np.full(c.T, -1, dtype=np.int32)
    assert np.array_equal(oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, allm), f64(c.y0))
    rank = c.rank.copy()
    rank[1] = 0                                            # slot 1 never became ready
    got = oracle.apply_decode(c.x, c.y0, c.A, c.B, rank, c.alpha, c.token_slot)
    assert np.array_equal(got[c.token_slot == 1], f64(c.y0)[c.token_slot == 1])
    with pytest.raises(ValueError):
        oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, np.full(c.T, c.n_slots, dtype=np.int32))


def test_token_permutation_invariance(oracle):
    c = small(51, T=25)
    base = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    perm = W.rng(5).permutation(c.T)
    got = oracle.apply_decode(c.x[perm], c.y0[perm], c.A, c.B, c.rank, c.alpha, c.token_slot[perm])
    assert np.array_equal(got, base[perm])


def test_linearity_in_B_and_alpha_scaling_exact(oracle):
    g = W.rng(61)
    T, d_in, d_out, S, r = 8, 16, 12, 2, 4
    x, y0 = ints_bf16(g, (T, d_in)), ints_bf16(g, (T, d_out))
    A, B1, B2 = ints_bf16(g, (S, r, d_in)), ints_bf16(g, (S, d_out, r), -3, 4), ints_bf16(g, (S, d_out, r), -3, 4)
    B12 = W.to_bf16_bits((f64(B1) + f64(B2)).astype(np.float32))
    slots = g.integers(0, S, size=T).astype(np.int32)
    rank, alpha = np.full(S, r), np.full(S, 4.0)
    ap = lambda B, al=alpha: oracle.apply_decode(x, y0, A, B, rank, al, slots)
    assert np.array_equal(ap(B12), ap(B1) + ap(B2) - f64(y0))
    d1, d2 = ap(B1) - f64(y0), ap(B1, alpha * 2) - f64(y0)
    assert np.array_equal(d2, 2 * d1) and np.abs(d1).max() > 0


def test_alpha_over_true_rank_and_padding(oracle):
    """A rank-3 adapter padded into an r_max = 8 slot equals the same adapter in a rank-3
    table, and its scale is alpha/3 (not alpha/8)."""
    g = W.rng(71)
    T, d_in, d_out = 5, 16, 8
    x, y0 = ints_bf16(g, (T, d_in)), ints_bf16(g, (T, d_out))
    A3, B3 = ints_bf16(g, (1, 3, d_in)), ints_bf16(g, (1, d_out, 3))
    A8, B8 = np.zeros((1, 8, d_in), np.uint16), np.zeros((1, d_out, 8), np.uint16)
    A8[:, :3], B8[:, :, :3] = A3, B3
    A8[:, 3:] = W.to_bf16_bits(np.float32([7.0]))[0]       # garbage beyond the rank must be ignored
    slots = np.zeros(T, dtype=np.int32)
    a = oracle.apply_decode(x, y0, A3, B3, [3], [6.0], slots)
    b = oracle.apply_decode(x, y0, A8, B8, [3], [6.0], slots)
    assert np.array_equal(a, b)
    want = f64(y0) + 2.0 * (f64(x) @ f64(A3[0]).T) @ f64(B3[0]).T
    assert np.array_equal(a, want)


def test_transposed_operands_would_fail(oracle):
    """Square shapes hide transposes; check one where d_in == d_out == r_max so that any swap of
    A/B or of their axes still type-checks but changes the numbers."""
    c = small(81, T=6, d_in=4, d_out=4, S=2, r=4, alpha=4.0)
    got = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    np.testing.assert_allclose(got, numpy_per_slot(c), rtol=1e-12, atol=1e-13)
    sw = oracle.apply_decode(c.x, c.y0, c.B, c.A, c.rank, c.alpha, c.token_slot)
    assert np.abs(sw - got).max() > 1e-3


# ---------------------------------------------------------------- segmented

def test_segmented_equals_decode_exactly(oracle):
    c = W.seg_case("s", 91, 40, 5, 24, 16, 3, 4, 8.0, mu=2.0, sigma=0.5)
    seg = oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.seg_off, c.seg_slot)
    dec = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    assert np.array_equal(seg, dec)
    one = oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha,
                                 np.arange(c.T + 1, dtype=np.int32), c.token_slot)
    assert np.array_equal(one, dec)
    np.testing.assert_allclose(seg, numpy_per_slot(c), rtol=1e-12, atol=1e-13)


def test_segmented_rejects_bad_offsets_and_allows_empty_segments(oracle):
    c = W.seg_case("s", 92, 10, 2, 8, 8, 2, 2, 2.0, seg_off=[0, 4, 10], seg_slot=[0, 1])
    with pytest.raises(ValueError):
        oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha, [0, 6, 4], [0, 1])
    with pytest.raises(ValueError):
        oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha, [0, 4, 9], [0, 1])
    a = oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha, [0, 4, 4, 10], [0, 1, 1])
    b = oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha, [0, 4, 10], [0, 1])
    assert np.array_equal(a, b)
    m = oracle.apply_segmented(c.x, c.y0, c.A, c.B, c.rank, c.alpha, [0, 4, 10], [-1, 1])
    assert np.array_equal(m[:4], f64(c.y0)[:4]) and np.array_equal(m[4:], b[4:])


# ---------------------------------------------------------------- MoE

def moe_small(seed, **kw):
    p = dict(T=10, K=2, E=4, d_in=16, d_out=12, n_slots=3, r_max=2, alpha=4.0)
    p.update(kw)
    return W.moe_case("m", seed, **p)


def test_moe_single_expert_reduces_to_decode(oracle):
    c = moe_small(101, K=1, E=1)
    got = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    dec = oracle.apply_decode(c.x, c.y0, c.A[:, 0], c.B[:, 0], c.rank, c.alpha, c.token_slot)
    assert np.array_equal(got, dec)


def test_moe_pairwise_brute_force(oracle):
    c = moe_small(102)
    c.token_slot[3] = -1
    got = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    x, y, A, B = f64(c.x), f64(c.y0), f64(c.A), f64(c.B)
    for t in range(c.T):
        for k in range(c.K):
            p, s, e = t * c.K + k, c.token_slot[t], c.topk[t, k]
            want = y[p] if s < 0 else y[p] + (c.alpha[s] / c.r_max) * B[s, e] @ (A[s, e] @ x[t])
            np.testing.assert_allclose(got[p], want, rtol=1e-12, atol=1e-13)


def test_moe_same_slot_is_a_grouped_gemm(oracle):
    c = moe_small(103, T=16, K=3, E=5, token_slot=np.full(16, 2, dtype=np.int32))
    got = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    x, want, A, B = f64(c.x), f64(c.y0).copy(), f64(c.A), f64(c.B)
    flat = c.topk.reshape(-1)
    for e in range(c.E):
        p = np.nonzero(flat == e)[0]
        want[p] += (c.alpha[2] / c.r_max) * (x[p // c.K] @ A[2, e].T) @ B[2, e].T
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def down_small(seed, **kw):
    p = dict(T=9, K=3, E=5, d_in=20, d_out=14, n_slots=3, r_max=2, alpha=4.0)
    p.update(kw)
    return W.moe_down_case("d", seed, **p)


def down_numpy(c, w=None):
    """The definition with numpy matmuls on independently widened values."""
    w = c.w.astype(np.float64) if w is None else w
    x, want, A, B = f64(c.x), f64(c.y0).copy(), f64(c.A), f64(c.B)
    for t in range(c.T):
        s = c.token_slot[t]
        if s < 0 or c.rank[s] == 0:
            continue
        for k in range(c.K):
            p, e = t * c.K + k, c.topk[t, k]
            want[t] += w[t, k] * (c.alpha[s] / c.rank[s]) * (B[s, e] @ (A[s, e] @ x[p]))
    return want


def test_moe_down_against_numpy_matmul(oracle):
    c = down_small(111, ranks=[2, 1, 2])
    c.token_slot[4] = -1
    got = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.w, c.token_slot)
    np.testing.assert_allclose(got, down_numpy(c), rtol=1e-12, atol=1e-13)
    assert np.array_equal(got[4], f64(c.y0)[4])                       # no slot: copied


def test_moe_down_merged_weight_brute_force(oracle):
    """Tiny case against the merged per-(slot, expert) matrix W' = (alpha/r) B A, formed first."""
    c = down_small(112, T=5, K=2, E=3, d_in=6, d_out=4, r_max=2)
    got = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.w, c.token_slot)
    x, want, A, B = f64(c.x), f64(c.y0).copy(), f64(c.A), f64(c.B)
    Wm = np.einsum("seoj,seji->seoi", B, A) * (c.alpha / c.rank)[:, None, None, None]
    for t in range(c.T):
        for k in range(c.K):
            for o in range(c.d_out):
                for i in range(c.d_in):
                    want[t, o] += float(c.w[t, k]) * Wm[c.token_slot[t], c.topk[t, k], o, i] * x[t * c.K + k, i]
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


def test_moe_down_single_pair_with_unit_weight_is_the_gate_up_form(oracle):
    """K = 1 and w = 1: one input row and one output row per token, i.e. the pair-major apply."""
    c = down_small(113, K=1)
    ones = np.ones((c.T, 1), dtype=np.float32)
    got = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, ones, c.token_slot)
    ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-14)


def test_moe_down_weights_are_linear_and_zero_weight_pairs_vanish(oracle):
    c = down_small(114)
    y0 = f64(c.y0)
    base = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.w, c.token_slot) - y0
    twice = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, 2 * c.w, c.token_slot) - y0
    np.testing.assert_allclose(twice, 2 * base, rtol=1e-12, atol=1e-13)
    none = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, 0 * c.w, c.token_slot)
    assert np.array_equal(none, y0)
    w1 = c.w.copy()
    w1[:, 1:] = 0                                                     # only the first pair of each token counts
    first = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, w1, c.token_slot)
    np.testing.assert_allclose(first, down_numpy(c, w1.astype(np.float64)), rtol=1e-12, atol=1e-13)
    assert not np.allclose(first, base + y0)                          # and the other pairs did matter


def test_moe_down_order_of_a_tokens_pairs_does_not_matter(oracle):
    """Reordering the K (expert, weight, input row) triples of every token only reassociates the sum."""
    c = down_small(115)
    got = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.w, c.token_slot)
    perm = np.array([2, 0, 1])
    x2 = c.x.reshape(c.T, c.K, c.d_in)[:, perm].reshape(c.T * c.K, c.d_in)
    got2 = oracle.apply_moe_down(x2, c.y0, c.A, c.B, c.rank, c.alpha, np.ascontiguousarray(c.topk[:, perm]),
                                 np.ascontiguousarray(c.w[:, perm]), c.token_slot)
    np.testing.assert_allclose(got2, got, rtol=1e-12, atol=1e-13)


def test_route_sort_against_python_sorted(oracle):
    for seed, kw in [(111, {}), (112, dict(T=64, K=4, E=8, n_slots=5)), (113, dict(T=5, K=1, E=1))]:
        c = moe_small(seed, **kw)
        c.token_slot[::4] = -1
        rank = c.rank.copy()
        rank[0] = 0
        sp, off = oracle.route_sort(c.topk, c.token_slot, rank, c.E)
        flat = c.topk.reshape(-1)
        elig = [p for p in range(c.T * c.K) if c.token_slot[p // c.K] >= 0 and rank[c.token_slot[p // c.K]] > 0]
        key = lambda p: int(c.token_slot[p // c.K]) * c.E + int(flat[p])
        want = sorted(elig, key=key)                      # python's sort is stable
        n = len(want)
        assert off[-1] == n and off[0] == 0
        assert sp[:n].tolist() == want and (sp[n:] == -1).all()
        counts = np.bincount([key(p) for p in elig], minlength=c.n_slots * c.E)
        assert np.array_equal(np.diff(off), counts)
        for gk in range(c.n_slots * c.E):                 # ascending p inside every group
            seg = sp[off[gk]:off[gk + 1]]
            assert (np.diff(seg) > 0).all() and all(key(p) == gk for p in seg)


def test_route_sort_rejects_bad_ids(oracle):
    c = moe_small(114)
    bad = c.topk.copy()
    bad[0, 0] = c.E
    with pytest.raises(ValueError):
        oracle.route_sort(bad, c.token_slot, c.rank, c.E)
