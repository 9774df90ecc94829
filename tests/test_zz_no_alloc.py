"""The decode entry point that allocates nothing (lora_apply_decode_noalloc) against
lora_apply_decode, through the C ABI: same bits, on calls in a row that share the library's
device array (the second smaller than the first, then other sites and launch shapes)."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as W
from tests import parity as P

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


@pytest.fixture(scope="module")
def M():
    import paper_2605_13779_amd as m
    m.load_library()
    return m


def _site(M, c):
    site = M.Site(c.d_in, c.d_out, c.r_max, c.n_slots)
    for s in range(c.n_slots):
        r = int(c.rank[s])
        if r:
            M.lora_slots_upload(site, s, s, np.ascontiguousarray(c.A[s][:r]), np.ascontiguousarray(c.B[s][:, :r]), r, float(c.alpha[s]))
    torch.cuda.synchronize()
    return site


def _both(M, oracle, c, site):
    x, ts = P.dev_bf16(c.x), torch.from_numpy(c.token_slot).cuda()
    ya, yb = P.dev_bf16(c.y0), P.dev_bf16(c.y0)
    M.lora_apply_decode(site, x, ya, ts)
    M.lora_apply_decode_noalloc(site, x, yb, ts)
    torch.cuda.synchronize()
    a, b = P.host_bits(ya), P.host_bits(yb)
    assert np.array_equal(a, b), f"{c.name}: the two entry points differ"
    ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    P.check_close(b, ref, c.name)
    eff = np.array([s >= 0 and c.rank[s] > 0 for s in c.token_slot])
    P.check_untouched(b, c.y0, ~eff, c.name)
    assert not np.array_equal(b[eff], c.y0[eff])


def test_noalloc_decode_matches_decode_on_calls_in_a_row(M, oracle):
    # few chunks and a large d_in: parts that trade partial sums through the exchange words of the array;
    # then a smaller batch on the same site; then sites of other ranks and shapes sharing the same array
    big = W.dense_case("na_big", 8801, 200, 4608, 520, 12, 16, 32.0, ranks=[16, 9, 0, 16, 3, 16, 16, 16, 1, 16, 16, 16],
                       std_a=0.05, std_b=0.05)
    site = _site(M, big)
    _both(M, oracle, big, site)
    small = dataclasses.replace(big, name="na_small", T=37, x=big.x[:37].copy(), y0=big.y0[:37].copy(),
                                token_slot=big.token_slot[:37].copy())       # same adapters, a smaller batch
    _both(M, oracle, small, site)
    _both(M, oracle, big, site)
    for name, T, d_in, d_out, S, r in (("na_planner", 700, 264, 136, 40, 8),      # more rows than a launch plans for itself
                                       ("na_r1", 300, 1024, 264, 400, 1),        # row-by-row form, no plan at all
                                       ("na_r64", 90, 520, 136, 6, 64),
                                       ("na_r4", 1024, 64, 72, 1024, 4)):         # the limits: 1024 rows, 1024 slots
        c = W.dense_case(name, 8810 + T, T, d_in, d_out, S, r, 2.0 * r, std_a=0.05, std_b=0.05)
        _both(M, oracle, c, _site(M, c))
    site.check()


def test_noalloc_decode_rejects_what_its_array_cannot_hold(M):
    site = M.Site(64, 64, 8, 4)
    x = torch.zeros((1025, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MLoraError) as e:
        M.lora_apply_decode_noalloc(site, x, x.clone(), torch.zeros(1025, dtype=torch.int32, device="cuda"))
    assert e.value.status == -6
    wide = M.Site(64, 64, 8, 1025)
    with pytest.raises(M.MLoraError) as e:
        M.lora_apply_decode_noalloc(wide, x[:8], x[:8].clone(), torch.zeros(8, dtype=torch.int32, device="cuda"))
    assert e.value.status == -6
    M.lora_apply_decode_noalloc(site, x[:0], x[:0].clone(), torch.zeros(0, dtype=torch.int32, device="cuda"))   # T = 0


def test_noalloc_decode_inside_a_captured_graph(M, oracle):
    # the callers the entry point is for: once the device's array is set up (first call, outside any
    # capture), a call can be captured and replayed; inputs change between replays
    c = W.dense_case("na_graph", 8830, 120, 2304, 264, 7, 16, 32.0, std_a=0.05, std_b=0.05)
    site = _site(M, c)
    x, y, ts = P.dev_bf16(c.x), P.dev_bf16(c.y0), torch.from_numpy(c.token_slot.copy()).cuda()
    M.lora_apply_decode_noalloc(site, x, y, ts)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        M.lora_apply_decode_noalloc(site, x, y, ts)
    for rep in range(3):
        xr = W.normal_bf16(W.rng(8840 + rep), c.x.shape, 1.0)
        sl = W.rng(8850 + rep).integers(-1, 7, size=c.T).astype(np.int32)
        x.copy_(P.dev_bf16(xr)); y.copy_(P.dev_bf16(c.y0)); ts.copy_(torch.from_numpy(sl))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.apply_decode(xr, c.y0, c.A, c.B, c.rank, c.alpha, sl)
        P.check_close(P.host_bits(y), ref, f"replay {rep}")
        P.check_untouched(P.host_bits(y), c.y0, sl < 0, c.name)
    site.check()
