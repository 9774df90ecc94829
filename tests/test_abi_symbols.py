"""The C-ABI library builds, loads and exports every symbol the header declares (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mlora.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2605_13779_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_13779_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith(("mlora_", "lora_", "moe_"))})


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"lora_slots_upload", "lora_apply_decode", "lora_apply_segmented", "moe_lora_apply_packed"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_the_header():
    from paper_2605_13779_amd import binding
    assert set(declared_functions()) == set(binding.SIGNATURES)


def test_host_side_validation_without_a_gpu(lib):
    from paper_2605_13779_amd.binding import SiteDesc
    sz = [C.c_size_t() for _ in range(4)]
    ok = SiteDesc(2560, 9728, 16, 64, 0, 0)
    assert lib.mlora_site_bytes(C.byref(ok), *[C.byref(s) for s in sz]) == 0
    assert sz[0].value == 64 * 16 * 2560 * 2 and sz[1].value == 64 * 9728 * 16 * 2
    pad = SiteDesc(64, 64, 3, 2, 0, 0)      # r_max 3 is stored with stride 4
    assert lib.mlora_site_bytes(C.byref(pad), *[C.byref(s) for s in sz]) == 0
    assert sz[0].value == 2 * 4 * 64 * 2
    moe = SiteDesc(2048, 768, 8, 32, 128, 0)
    assert lib.mlora_site_bytes(C.byref(moe), *[C.byref(s) for s in sz]) == 0
    assert sz[0].value == 32 * 128 * 8 * 2048 * 2 and sz[1].value == 32 * 128 * 768 * 8 * 2
    for bad, code in [(SiteDesc(100, 64, 8, 2, 0, 0), -2), (SiteDesc(64, 64, 0, 2, 0, 0), -2),
                      (SiteDesc(64, 64, 65, 2, 0, 0), -2), (SiteDesc(64, 64, 8, 0, 0, 0), -1),
                      (SiteDesc(-8, 64, 8, 2, 0, 0), -1)]:
        assert lib.mlora_site_bytes(C.byref(bad), *[C.byref(s) for s in sz]) == code
    assert lib.mlora_site_bytes(None, *[C.byref(s) for s in sz]) == -1
    n = C.c_size_t()
    assert lib.mlora_plan_bytes(256, 64, C.byref(n)) == 0 and n.value % 256 == 0 and n.value > 256 * 16
    assert lib.mlora_plan_bytes(0, 64, C.byref(n)) == -1
    assert lib.mlora_status_str(-4) == b"segment offsets malformed"
    # null handles are rejected before any device work
    assert lib.lora_apply_decode(None, None, 0, None, 0, None, 4, None) == -1
    assert lib.lora_slots_upload(None, 0, 0, None, None, 1, 1.0, 0, None) == -1
    assert lib.moe_lora_apply_packed(None, None, 0, None, 0, None, None, 1, 1, None, None, None) == -1


def test_noop_is_rejected_by_the_parity_rules():
    """Mutation control for the comparison rules themselves: an implementation that leaves y
    unchanged must fail the delta check that every GPU parity test applies."""
    from tests import parity as P
    delta = np.random.default_rng(0).standard_normal((8, 16)) * 0.02
    with pytest.raises(AssertionError):
        P.noop_must_fail(np.zeros((8, 16), np.uint16), np.zeros((8, 16)), np.arange(8))
    P.noop_must_fail(np.zeros((8, 16), np.uint16), delta, np.arange(8))


def test_pack_experts_stacks_and_pads_like_numpy(lib):
    """Host-only packing of per-expert tensors into the slot image (the packed adapter form: one
    stacked tensor per projection and A|B instead of one per expert), against plain numpy."""
    from paper_2605_13779_amd import binding
    g = np.random.default_rng(7)
    for E, r, r_max, d_in, d_out in [(5, 3, 6, 24, 16), (4, 8, 8, 16, 40), (1, 1, 1, 8, 8), (128, 8, 8, 64, 24)]:
        desc = binding.SiteDesc(d_in, d_out, r_max, 2, E if E > 1 else 0, 0)
        A_e = [g.integers(1, 65535, size=(r, d_in), dtype=np.uint16) for _ in range(E)]
        B_e = [g.integers(1, 65535, size=(d_out, r), dtype=np.uint16) for _ in range(E)]
        a_img, b_img = binding.pack_experts(desc, A_e, B_e, r)
        rp = 1
        while rp < r_max:
            rp *= 2
        want_a = np.zeros((E, rp, d_in), dtype=np.uint16)
        want_b = np.zeros((E, d_out, rp), dtype=np.uint16)
        want_a[:, :r] = np.stack(A_e)
        want_b[:, :, :r] = np.stack(B_e)
        assert np.array_equal(a_img.reshape(E, rp, d_in), want_a)
        assert np.array_equal(b_img.reshape(E, d_out, rp), want_b)
    # the census of the paper's 30B-MoE adapter: per layer and projection 128 experts x {A, B} = 256
    # tensors become 2 stacked ones, 48 layers x 3 projections -> 36,864 become 288
    # (tests/golden/adapter_census.txt holds the printed totals)
    assert 48 * 3 * 128 * 2 == 36864 and 48 * 3 * 2 == 288
    desc = binding.SiteDesc(16, 16, 4, 2, 3, 0)
    A_e = [np.ones((2, 16), dtype=np.uint16)] * 3
    B_e = [np.ones((16, 2), dtype=np.uint16)] * 3
    with pytest.raises(binding.MLoraError):
        binding.pack_experts(desc, A_e, B_e, 5)        # rank above r_max
