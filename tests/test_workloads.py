"""The input recipes: shapes, distributions and the paper-printed adapter census."""
import os

import numpy as np
import pytest

import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "adapter_census.txt")


def census():
    out = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_paper_census_fixes_the_moe_geometry():
    """The paper prints 37,248 tensors (37,152 of them <= 4 KB, 105.5 MB declared) for a rank-1
    adapter of the 30B MoE model and 672 keys after packing.  Those counts are reproduced by
    48 layers x 128 experts x {gate, up, down} x {A, B} per-expert tensors with hidden 2048 and
    expert intermediate 768, plus 8 attention tensors per layer -- the geometry workload c4 uses."""
    c = census()
    L, E, H, I = 48, 128, 2048, 768
    q_out, kv_out = 4096, 512
    expert = L * E * 3 * 2
    attn = L * 8
    assert expert + attn == c["tensors_unpacked"]
    # rank-1 bf16: a tensor is <= 4 KB iff its long side is <= 2048 elements
    attn_small = L * sum(1 for d in (H, q_out, H, kv_out, H, kv_out, q_out, H) if d * 2 <= 4096)
    assert expert + attn_small == c["tensors_le_4kb"]
    nbytes = 2 * (L * E * 3 * (H + I) + L * (H + q_out + 2 * (H + kv_out) + q_out + H))
    assert round(nbytes / 1e6, 1) == c["declared_bytes_mb"]
    assert L * 3 * 2 == c["packed_groups"] and attn == c["packed_copied"]
    assert c["packed_groups"] + c["packed_copied"] == c["packed_keys"]
    m = W.moe_case("probe", 1, 4, 2, 4, H, I, 1, 1, 1.0)
    assert m.A.shape[-1] == H and m.B.shape[-2] == I


def test_dense4b_census():
    c = census()
    per_rank = 2560 + 4096 + 2 * (2560 + 1024) + 4096 + 2560 + 2 * (2560 + 9728) + 9728 + 2560
    assert per_rank == 57344
    payload = 36 * 32 * per_rank * 4
    assert 0 < c["dense4b_rank32_file_bytes"] - payload < 100_000


def test_bf16_bits_rne():
    f = np.float32([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -2.5, 0.0, 3.0e-3])
    b = W.to_bf16_bits(f)
    assert b.tolist()[:5] == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0]
    back = (b.astype(np.uint32) << 16).view(np.float32)
    assert abs(back[5] - f[5]) <= abs(f[5]) * 2.0 ** -8


def test_zipf_head_probability():
    s = W.zipf_slots(W.rng(3), 200_000, 64, 1.1)
    w = np.arange(1, 65) ** -1.1
    p = np.bincount(s, minlength=64) / s.size
    assert s.min() >= 0 and s.max() <= 63
    np.testing.assert_allclose(p[:8], (w / w.sum())[:8], atol=4e-3)


def test_segments_sum_and_minimum():
    for seed in range(20):
        off = W.lognormal_segments(W.rng(seed), 8192, 16, 6.0, 0.8)
        L = np.diff(off)
        assert off[0] == 0 and off[-1] == 8192 and (L >= 1).all() and len(L) == 16
    off = W.lognormal_segments(W.rng(1), 20, 16, 6.0, 2.0)
    assert off[-1] == 20 and (np.diff(off) >= 1).all()


def test_topk_routing_is_topk():
    g = W.rng(9)
    ids = W.topk_routing(g, 50, 16, 4)
    logits = W.rng(9).standard_normal((50, 16), dtype=np.float32)
    for t in range(50):
        assert len(set(ids[t])) == 4
        assert sorted(logits[t])[-4:][::-1] == [logits[t, e] for e in ids[t]]


def test_benchmark_configs_have_the_stated_shapes():
    c1 = W.c1_tiny_decode()
    assert (c1.T, c1.d_in, c1.d_out, c1.n_slots, c1.r_max) == (64, 256, 256, 8, 8)
    assert c1.token_slot.min() == -1 and c1.token_slot.max() == 7 and c1.alpha[0] == 16
    c3 = W.c3_rank1_catalog()
    assert len(set(c3.token_slot.tolist())) == 512 and c3.A.shape == (1024, 1, 4096)
    assert len(set(c3.catalog_id.tolist())) == 1024 and c3.catalog_id.max() < 10 ** 6
    c5 = W.c5_segmented()
    assert c5.seg_off[-1] == 8192 and c5.A.shape == (16, 64, 7168) and c5.B.shape == (16, 7168, 64)


@pytest.mark.timeout(120)
def test_generators_are_deterministic():
    a, b = W.c1_tiny_decode(), W.c1_tiny_decode()
    for f in ("x", "y0", "A", "B", "token_slot"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    s1 = W.c2_dense_decode()[0].token_slot
    assert 40 <= len(set(s1.tolist())) <= 60
