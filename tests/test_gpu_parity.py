"""HIP path vs the fp64 oracle, element by element, through the C ABI (needs an MI355X)."""
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


def upload_all(M, site, c, ranks=None):
    """Upload every slot in its true (unpadded) PEFT shape."""
    for s in range(c.n_slots):
        r = int(c.rank[s])
        if r == 0:
            continue
        A = np.ascontiguousarray(c.A[s][..., :r, :])
        B = np.ascontiguousarray(c.B[s][..., :, :r])
        M.lora_slots_upload(site, s, int(c.catalog_id[s]) if getattr(c, "catalog_id", None) is not None else s,
                            A, B, r, float(c.alpha[s]))
    torch.cuda.synchronize()


def dense_site(M, c):
    site = M.Site(c.d_in, c.d_out, c.r_max, c.n_slots)
    upload_all(M, site, c)
    return site


def run_decode(M, site, c, y0_bits, planned=False):
    x, y = P.dev_bf16(c.x), P.dev_bf16(y0_bits)
    ts = torch.from_numpy(c.token_slot).cuda()
    if planned:
        plan = M.Plan(max(c.T, 1), c.n_slots)
        M.lora_plan_decode(plan, ts, c.n_slots)
        M.lora_apply_decode_planned(site, plan, x, y)
    else:
        M.lora_apply_decode(site, x, y, ts)
    torch.cuda.synchronize()
    return P.host_bits(y)


def check_dense(M, oracle, c, runner, rows=None, report=None):
    """Full comparison + the three vacuity guards.  rows: optional subset of rows sent to the oracle
    (never used on the benchmark configurations); report: name of a line of the error table."""
    sel = np.arange(c.T) if rows is None else np.asarray(rows)
    ref = oracle.apply_decode(c.x[sel], c.y0[sel], c.A, c.B, c.rank, c.alpha, c.token_slot[sel])
    got = runner(c.y0)
    P.check_close(got[sel], ref, c.name)
    if report:
        assert rows is None
        P.report(report, got, ref, c.T, "rows")
    eff = np.array([s >= 0 and c.rank[s] > 0 for s in c.token_slot])
    P.check_untouched(got, c.y0, ~eff, c.name)
    zero = np.zeros_like(c.y0)
    dref = oracle.apply_decode(c.x[sel], zero[sel], c.A, c.B, c.rank, c.alpha, c.token_slot[sel])
    gz = runner(zero)
    P.check_delta(gz[sel], dref, c.name + " delta")
    P.noop_must_fail(c.y0[sel], dref, np.nonzero(eff[sel])[0])


# ------------------------------------------------------------------ decode

def test_c1_tiny_decode(M, oracle):
    c = W.c1_tiny_decode()
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0), report=c.name)
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0, planned=True))


@pytest.mark.parametrize("r", [1, 2, 4, 8, 16, 32, 64])
def test_decode_all_ranks_ragged(M, oracle, r):
    """Several d_out tiles, a ragged tail (d_out = 1064 is not a multiple of the pass width),
    -1 rows, groups larger than one chunk."""
    c = W.dense_case(f"rag_r{r}", 1000 + r, 77, 328, 1064, 5, r, 2.0 * r, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0))


def test_decode_mixed_ranks_padding_and_empty_slots(M, oracle):
    ranks = [3, 16, 0, 7, 1, 12]
    c = W.dense_case("mixed", 2001, 90, 256, 512, 6, 16, 24.0, ranks=ranks, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    rank, scale, cat = site.meta()
    assert rank.tolist() == ranks
    np.testing.assert_allclose(scale[[0, 1, 3]], [24 / 3, 24 / 16, 24 / 7], rtol=1e-6)
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0))
    # evicting a slot turns its rows into no-ops; re-uploading with a smaller rank must clear the padding
    M.lora_slots_evict(site, 1)
    c2 = W.dense_case("mixed", 2001, 90, 256, 512, 6, 16, 24.0, ranks=[3, 0, 0, 7, 1, 12], std_a=0.05, std_b=0.05)
    check_dense(M, oracle, c2, lambda y0: run_decode(M, site, c2, y0))
    c3 = W.dense_case("mixed", 2001, 90, 256, 512, 6, 16, 24.0, ranks=[3, 5, 0, 7, 1, 12], std_a=0.05, std_b=0.05)
    M.lora_slots_upload(site, 1, 77, np.ascontiguousarray(c3.A[1][:5]), np.ascontiguousarray(c3.B[1][:, :5]), 5, 24.0)
    check_dense(M, oracle, c3, lambda y0: run_decode(M, site, c3, y0))
    assert site.meta()[2][1] == 77


@pytest.mark.parametrize("r", [8, 1])
def test_decode_edge_cases(M, oracle, r):
    """(rank 8 goes through a plan, rank 1 through the row-by-row form of lora_apply_decode)"""
    c = W.dense_case("edge", 3001, 40, 64, 64, 4, r, 2.0 * r, std_a=0.1, std_b=0.1)
    site = dense_site(M, c)
    # all rows without an adapter
    c.token_slot[:] = -1
    got = run_decode(M, site, c, c.y0)
    assert np.array_equal(got, c.y0)
    # every row on one slot (one big group)
    c.token_slot[:] = 2
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0))
    # out-of-range indices are treated like -1
    c.token_slot[::5] = 9
    c.token_slot[1::5] = -7
    got = run_decode(M, site, c, c.y0)
    bad = (c.token_slot < 0) | (c.token_slot >= 4)
    assert np.array_equal(got[bad], c.y0[bad])
    # T = 0
    x0 = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    M.lora_apply_decode(site, x0, x0.clone(), torch.empty(0, dtype=torch.int32, device="cuda"))
    # single row
    c1 = W.dense_case("one", 3002, 1, 64, 64, 4, r, 2.0 * r, std_a=0.1, std_b=0.1, token_slot=[3])
    upload_all(M, site, c1)
    check_dense(M, oracle, c1, lambda y0: run_decode(M, site, c1, y0))


def test_decode_strided_rows(M, oracle):
    """x and y as column slices of wider buffers (row stride != width)."""
    c = W.dense_case("stride", 3003, 33, 128, 256, 3, 8, 16.0, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    xb = torch.zeros((c.T, 200), dtype=torch.bfloat16, device="cuda")
    yb = torch.zeros((c.T, 320), dtype=torch.bfloat16, device="cuda")
    xb[:, 8:136] = P.dev_bf16(c.x)
    yb[:, 16:272] = P.dev_bf16(c.y0)
    guard = yb.clone()
    M.lora_apply_decode(site, xb[:, 8:136], yb[:, 16:272], torch.from_numpy(c.token_slot).cuda())
    torch.cuda.synchronize()
    ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    P.check_close(P.host_bits(yb[:, 16:272]), ref, "strided")
    assert torch.equal(yb[:, :16], guard[:, :16]) and torch.equal(yb[:, 272:], guard[:, 272:])


def _far_rows(bits, ld):
    """The rows of `bits` as a view into a buffer whose rows lie `ld` elements apart."""
    buf = torch.empty((bits.shape[0], ld), dtype=torch.bfloat16, device="cuda")
    view = buf[:, :bits.shape[1]]
    view.copy_(P.dev_bf16(bits))
    return view


def test_rows_more_than_4_gib_apart(M, oracle):
    """Row strides of 64 MiB: the last rows of x and y start beyond 4 GiB from the first, so any
    32-bit row offset in a kernel would land in the wrong row.  Decode (planned in the launch and
    the row-by-row form of rank 1), the matrix-core prefill pair and the packed MoE call."""
    ld = (1 << 25) + 8
    for r in (8, 1):
        c = W.dense_case(f"far_r{r}", 3090 + r, 72, 128, 192, 3, r, 2.0 * r, std_a=0.05, std_b=0.05)
        c.token_slot[5] = -1
        site = dense_site(M, c)
        x, y = _far_rows(c.x, ld), _far_rows(c.y0, ld)
        M.lora_apply_decode(site, x, y, torch.from_numpy(c.token_slot).cuda())
        torch.cuda.synchronize()
        ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.check_close(P.host_bits(y.contiguous()), ref, c.name)
        del x, y
    c = W.seg_case("far_seg", 3093, 72, 3, 256, 192, 2, 64, 128.0, seg_off=[0, 30, 31, 72], seg_slot=[1, -1, 0],
                   std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    x, y = _far_rows(c.x, ld), _far_rows(c.y0, ld)
    M.lora_apply_segmented(site, x, y, c.seg_off, c.seg_slot)
    torch.cuda.synchronize()
    ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    got = P.host_bits(y.contiguous())
    P.check_close(got, ref, c.name)
    P.check_untouched(got, c.y0, c.token_slot < 0, c.name)
    del x, y
    c = W.moe_case("far_moe", 3094, 36, 2, 4, 136, 200, 3, 8, 16.0, std_a=0.05, std_b=0.05)
    site = moe_site(M, c)
    x, y = _far_rows(c.x, 2 * ld), _far_rows(c.y0, ld)
    M.moe_lora_apply_packed(site, x, y, torch.from_numpy(c.topk).cuda(), torch.from_numpy(c.token_slot).cuda(), None, None)
    torch.cuda.synchronize()
    ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    P.check_close(P.host_bits(y.contiguous()), ref, c.name)
    del x, y
    torch.cuda.empty_cache()


def test_decode_large_batch_general_planner(M, oracle):
    """More rows than the one-workgroup planner takes: the histogram/scan/scatter pipeline."""
    c = W.dense_case("big", 3004, 2500, 64, 96, 37, 4, 8.0, std_a=0.1, std_b=0.1)
    site = dense_site(M, c)
    for pipeline in (0, 1):                               # the one-launch form and the four-launch pipeline
        M.set_tuning("plan_general", 1)
        M.set_tuning("plan_pipeline", pipeline)
        try:
            check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0))
        finally:
            M.set_tuning("plan_general", 0)
            M.set_tuning("plan_pipeline", 0)
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0))


def test_decode_multi_site_launch(M, oracle):
    """Sites that share a plan in one launch (the q/k/v pattern): right against the oracle and, up to
    the order of the fp32 partial sums (a grouped launch may cut d_in into a different number of
    slices), equal to separate calls; a site that cannot be grouped (small d_in) still gets its own
    launch."""
    shapes = [(2304, 264, 16), (2304, 1032, 16), (2304, 2056, 16), (128, 72, 16), (2304, 520, 16), (2304, 264, 16)]
    slots = W.rng(31).integers(-1, 5, size=61).astype(np.int32)
    cases = [W.dense_case(f"multi{i}", 3100 + i, 61, di, do, 5, r, 32.0, token_slot=slots, std_a=0.05, std_b=0.05)
             for i, (di, do, r) in enumerate(shapes)]
    sites = [dense_site(M, c) for c in cases]
    plan = M.Plan(61, 5)
    M.lora_plan_decode(plan, torch.from_numpy(slots).cuda(), 5)
    xs = [P.dev_bf16(c.x) for c in cases]
    ys = [P.dev_bf16(c.y0) for c in cases]
    M.lora_apply_decode_multi(sites, plan, xs, ys)
    torch.cuda.synchronize()
    for c, site, x, y in zip(cases, sites, xs, ys):
        ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        got = P.host_bits(y)
        P.check_close(got, ref, c.name)
        P.check_untouched(got, c.y0, c.token_slot < 0, c.name)
        y1 = P.dev_bf16(c.y0)
        M.lora_apply_decode_planned(site, plan, x, y1)
        torch.cuda.synchronize()
        single = P.host_bits(y1)
        P.check_close(single, ref, c.name + " (own launch)")
        wa, wb = P.widen(single), P.widen(got)
        # one bf16 step at most (plus, where y0 and the delta cancel, the rounding noise of the fp32 sums)
        assert np.all(np.abs(wa - wb) <= 2.0 ** -7 * np.maximum(np.abs(wa), np.abs(wb)) + 2.0 ** -22 * P.summed_magnitude(c)), c.name
        assert np.mean(single != got) < 0.02, c.name
        dref = oracle.apply_decode(c.x, np.zeros_like(c.y0), c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.noop_must_fail(c.y0, dref, np.nonzero(c.token_slot >= 0)[0])


def test_decode_parts_when_partners_never_answer(M, oracle):
    """A chunk of a dense site is cut into parts that trade partial sums.  With the wait for a
    partner's words cut to nothing, every part that has not been answered yet takes its item on its
    own (whole shrink): the result must meet the same bar, alone and in a grouped launch."""
    shapes = [(2304, 1032, 16), (4096, 520, 8), (2304, 2056, 16)]
    slots = W.rng(37).integers(-1, 6, size=77).astype(np.int32)
    cases = [W.dense_case(f"solo{i}", 3300 + i, 77, di, do, 6, r, 32.0, token_slot=slots, std_a=0.05, std_b=0.05)
             for i, (di, do, r) in enumerate(shapes)]
    sites = [dense_site(M, c) for c in cases]
    plan = M.Plan(77, 6)
    M.lora_plan_decode(plan, torch.from_numpy(slots).cuda(), 6)
    grp = [0, 2]                                       # same rank: one launch

    def run_all():
        out = []
        for c, site in zip(cases, sites):
            y = P.dev_bf16(c.y0)
            M.lora_apply_decode_planned(site, plan, P.dev_bf16(c.x), y)
            out.append(y)
        xs = [P.dev_bf16(cases[k].x) for k in grp]
        ys = [P.dev_bf16(cases[k].y0) for k in grp]
        M.lora_apply_decode_multi([sites[k] for k in grp], plan, xs, ys)
        torch.cuda.synchronize()
        return [P.host_bits(y) for y in out + ys]
    traded = run_all()
    M.set_tuning("rows_poll_limit", -1)
    try:
        alone = run_all()
    finally:
        M.set_tuning("rows_poll_limit", 0)
    for k, (c, a, b) in enumerate(zip(cases + [cases[k] for k in grp], traded, alone)):
        ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.check_close(b, ref, c.name + (" (grouped)" if k >= len(cases) else ""))
        P.check_untouched(b, c.y0, c.token_slot < 0, c.name)
        # (an item on its own adds the k-slices of d_in in one sweep instead of slice by slice: the two
        # fp32 sums carry different rounding errors, each a few 2^-24 of the magnitudes that were added,
        # so the outputs may differ in their last bit -- or, where y0 and the delta cancel, by that much
        # of what was summed: 2^-22 of sum_j |B_oj| sum_i |x_i A_ji| * alpha / r)
        wa, wb = P.widen(a), P.widen(b)
        bad = np.argwhere(np.abs(wa - wb) > 2.0 ** -7 * np.maximum(np.abs(wa), np.abs(wb)) + 2.0 ** -22 * P.summed_magnitude(c))
        assert len(bad) == 0, (c.name, len(bad), [(tuple(i), float(wa[tuple(i)]), float(wb[tuple(i)])) for i in bad[:5]])
    for site in sites:
        site.check()


def test_decode_after_an_exchange_wait_gave_up(M, oracle):
    """If the last workgroup of a launch ever gives up waiting for the other workgroups' sign-ins, it
    leaves the site's launch tag at a value that switches the exchange of partial sums off: every
    later item runs on its own until mlora_site_check has reported the flag and reset the control
    block.  The host plants that state here (the control block sits in front of the 1 MiB of
    exchange words at the end of a site's scratch buffer); results must stay right, the check must
    report once, and the launches after it must trade partial sums again (same bits as before)."""
    c = W.dense_case("poison", 3360, 77, 4608, 520, 6, 16, 32.0, std_a=0.05, std_b=0.05)     # few chunks, large d_in: parts that trade
    site = dense_site(M, c)
    plan = M.Plan(77, 6)
    M.lora_plan_decode(plan, torch.from_numpy(c.token_slot).cuda(), 6)
    x = P.dev_bf16(c.x)
    ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)

    def run():
        y = P.dev_bf16(c.y0)
        M.lora_apply_decode_planned(site, plan, x, y)
        torch.cuda.synchronize()
        return P.host_bits(y)
    before = run()
    P.check_close(before, ref, "before")
    site.check()
    ctrl = site.bufs[3][site.bytes[3] - (1 << 20) - 1024:][:1024].view(torch.int32)
    assert int(ctrl[0]) >= 2 and int(ctrl[1]) == 0           # the launch tag has moved on, no flag
    ctrl[0] = -1                                             # the switched-off value
    ctrl[1] = 2
    torch.cuda.synchronize()
    for _ in range(2):
        P.check_close(run(), ref, "exchange switched off")
        assert int(ctrl[0]) == -1
    with pytest.raises(M.MLoraError):
        site.check()
    site.check()                                             # reported once, then clear
    assert int(ctrl[0]) == 1 and int(ctrl[1]) == 0
    assert np.array_equal(run(), before)
    assert int(ctrl[0]) == 2


@pytest.mark.parametrize("mode", [1, 3])
def test_decode_launch_shapes_forced(M, oracle, mode):
    """The launch shapes a dense site does not get by default at these sizes: parts that each redo
    the whole shrink (1) and one item per chunk whatever the chunk count (3); alone and grouped."""
    shapes = [(2304, 1032, 16), (4096, 520, 8), (2304, 2056, 16), (1024, 264, 4)]
    slots = W.rng(38).integers(-1, 6, size=77).astype(np.int32)
    cases = [W.dense_case(f"shape{mode}_{i}", 3350 + i, 77, di, do, 6, r, 32.0, token_slot=slots, std_a=0.05, std_b=0.05)
             for i, (di, do, r) in enumerate(shapes)]
    sites = [dense_site(M, c) for c in cases]
    plan = M.Plan(77, 6)
    M.lora_plan_decode(plan, torch.from_numpy(slots).cuda(), 6)
    M.set_tuning("rows_mode", mode)
    try:
        for c, site in zip(cases, sites):
            y = P.dev_bf16(c.y0)
            M.lora_apply_decode_planned(site, plan, P.dev_bf16(c.x), y)
            torch.cuda.synchronize()
            ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
            P.check_close(P.host_bits(y), ref, c.name)
            P.check_untouched(P.host_bits(y), c.y0, c.token_slot < 0, c.name)
        grp = [0, 2]
        xs = [P.dev_bf16(cases[k].x) for k in grp]
        ys = [P.dev_bf16(cases[k].y0) for k in grp]
        M.lora_apply_decode_multi([sites[k] for k in grp], plan, xs, ys)
        torch.cuda.synchronize()
        for k, y in zip(grp, ys):
            c = cases[k]
            ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
            P.check_close(P.host_bits(y), ref, c.name + " (grouped)")
    finally:
        M.set_tuning("rows_mode", 0)


def _plan_words(plan, max_items, n_keys):
    """hdr, sorted and chunk records of a plan buffer (layout: 8 header words, three tables of
    n_keys + 1, four of max_items, then the records)."""
    w = plan.buf.view(torch.int32).cpu().numpy()
    off_sorted = 8 + 3 * (n_keys + 1) + 3 * max_items
    return w[:2].copy(), w[off_sorted:off_sorted + max_items].copy(), w[off_sorted + max_items:].copy()


@pytest.mark.parametrize("T,S", [(61, 5), (256, 64), (1, 3), (200, 64), (300, 7), (256, 65), (250, 300), (256, 1000)])
def test_decode_step_that_plans_inside_its_first_launch(M, oracle, T, S):
    """lora_plan_apply_decode_multi = lora_plan_decode + lora_apply_decode_multi, bit for bit, in the
    results and in the plan it leaves behind (which a later planned apply uses); 300 rows are more
    than a launch plans for itself and take the two-call path, as does a first site that cannot
    share a launch."""
    shapes = [(2304, 264, 16), (2304, 1032, 16), (2304, 520, 16), (128, 72, 16)]
    slots = W.rng(90 + T).integers(-1, S, size=T).astype(np.int32)
    cases = [W.dense_case(f"pl{i}", 3200 + i, T, di, do, S, r, 32.0, token_slot=slots, ranks=[16 if k % 5 else 0 for k in range(S)] if S > 3 else None,
                          std_a=0.05, std_b=0.05) for i, (di, do, r) in enumerate(shapes)]
    sites = [dense_site(M, c) for c in cases]
    ts = torch.from_numpy(slots).cuda()
    for order in ([0, 1, 2, 3], [3, 0, 1]):
        cs, ss = [cases[k] for k in order], [sites[k] for k in order]
        xs = [P.dev_bf16(c.x) for c in cs]
        ya, yb = [P.dev_bf16(c.y0) for c in cs], [P.dev_bf16(c.y0) for c in cs]
        pa, pb = M.Plan(max(T, 1), S), M.Plan(max(T, 1), S)
        pa.buf.zero_(); pb.buf.zero_()
        M.lora_plan_decode(pa, ts, S, ready_from=ss[0])
        M.lora_apply_decode_multi(ss, pa, xs, ya)
        M.lora_plan_apply_decode_multi(ss, pb, ts, S, xs, yb, ready_from=ss[0])
        torch.cuda.synchronize()
        for c, a, b in zip(cs, ya, yb):
            ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
            if not torch.equal(a, b):                  # say where before failing
                ga, gb = P.host_bits(a), P.host_bits(b)
                d = ga != gb
                rows, cols = np.nonzero(d.any(axis=1))[0], np.nonzero(d.any(axis=0))[0]
                tol = 2e-2 + 2e-2 * np.abs(ref)
                print(f"{c.name} order {order}: {int(d.sum())} elements differ, rows {rows.tolist()} (slots {slots[rows].tolist()}), "
                      f"columns {cols.min()}..{cols.max()} ({len(cols)}), two calls outside tolerance {int((np.abs(P.widen(ga) - ref) > tol).sum())}, "
                      f"one call {int((np.abs(P.widen(gb) - ref) > tol).sum())}, max |a - b| {np.abs(P.widen(ga) - P.widen(gb)).max():.4g}", flush=True)
                for k_, s_ in zip(order, ss):
                    ctrl = s_.bufs[3][s_.bytes[3] - (1 << 20) - 1024:][:1024].view(torch.int32)
                    print(f"   site {k_}: tag {int(ctrl[0])} flag {int(ctrl[1])}", flush=True)
            assert torch.equal(a, b), c.name
            P.check_close(P.host_bits(b), ref, c.name)
        (ha, sa, ra), (hb, sb, rb) = _plan_words(pa, max(T, 1), S), _plan_words(pb, max(T, 1), S)
        assert np.array_equal(ha, hb), (ha, hb)
        n_chunks, n_rows = int(ha[0]), int(ha[1])
        assert np.array_equal(sa[:n_rows], sb[:n_rows])
        ra, rb = ra[:8 * ((T + 3 * min(S, T)) // 4)].reshape(-1, 8), rb[:8 * ((T + 3 * min(S, T)) // 4)].reshape(-1, 8)
        assert np.array_equal(ra[:, 1], rb[:, 1]) and np.all(ra[n_chunks:, 1] == 0)
        for k in range(n_chunks):
            assert np.array_equal(ra[k, :3], rb[k, :3]) and np.array_equal(ra[k, 4:4 + ra[k, 1]], rb[k, 4:4 + rb[k, 1]])
        # the plan that the fused launch left behind drives a later planned apply
        y2 = P.dev_bf16(cs[0].y0)
        M.lora_apply_decode_planned(ss[0], pb, xs[0], y2)
        torch.cuda.synchronize()
        ref = oracle.apply_decode(cs[0].x, cs[0].y0, cs[0].A, cs[0].B, cs[0].rank, cs[0].alpha, cs[0].token_slot)
        P.check_close(P.host_bits(y2), ref, "later apply")


def test_single_site_plans_inside_its_launch(M, oracle):
    """A rank-1 catalog site (every row its own slot, 1024 slots) and sites of the other ranks on their own:
    the launch plans for itself up to 256 rows and 1024 slots (more rows take the two calls); same
    bits as plan + planned apply."""
    for name, T, S, d_in, d_out, r in (("cat", 256, 1024, 4096, 264, 1), ("cat_ragged", 199, 700, 4096, 136, 1),
                                       ("cat_two_calls", 333, 700, 4096, 136, 1), ("one16", 200, 40, 2304, 264, 16),
                                       ("one2", 100, 9, 4096, 72, 2), ("one4", 130, 20, 4096, 136, 4),
                                       ("one32", 90, 12, 1024, 200, 32), ("one64", 70, 6, 520, 136, 64)):
        slots = W.rng(95 + T).permutation(S)[:T].astype(np.int32) if r == 1 else W.rng(95 + T).integers(-1, S, size=T).astype(np.int32)
        slots[::11] = -1
        c = W.dense_case(name, 3300 + T, T, d_in, d_out, S, r, 2.0 * r, token_slot=slots, std_a=0.05, std_b=0.05)
        site = dense_site(M, c)
        ts = torch.from_numpy(slots).cuda()
        x = P.dev_bf16(c.x)
        ya, yb = P.dev_bf16(c.y0), P.dev_bf16(c.y0)
        pa, pb = M.Plan(T, S), M.Plan(T, S)
        pa.buf.zero_(); pb.buf.zero_()
        M.lora_plan_decode(pa, ts, S)
        M.lora_apply_decode_planned(site, pa, x, ya)
        M.lora_plan_apply_decode_multi([site], pb, ts, S, [x], [yb])
        yc = P.dev_bf16(c.y0)
        M.lora_apply_decode(site, x, yc, ts)               # the one-call form takes the same path on its private plan
        torch.cuda.synchronize()
        assert torch.equal(ya, yb), name
        ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.check_close(P.host_bits(yb), ref, name)
        if r > 2:
            assert torch.equal(ya, yc), name
        else:       # ranks 1 and 2: the one-call form applies row by row without a plan (other order of the fp32 partial sums)
            P.check_close(P.host_bits(yc), ref, name + " ungrouped")
            P.check_untouched(P.host_bits(yc), c.y0, c.token_slot < 0, name)
        (ha, sa, ra), (hb, sb, rb) = _plan_words(pa, T, S), _plan_words(pb, T, S)
        assert np.array_equal(ha, hb) and np.array_equal(sa[:ha[1]], sb[:hb[1]]), name
        nrec = (T + 3 * min(S, T)) // 4
        ra, rb = ra[:8 * nrec].reshape(-1, 8), rb[:8 * nrec].reshape(-1, 8)
        assert np.array_equal(ra[:, 1], rb[:, 1]) and np.array_equal(ra[:ha[0], :3], rb[:hb[0], :3]), name
        live = np.arange(4)[None, :] < ra[:ha[0], 1:2]
        assert np.array_equal(ra[:ha[0], 4:][live], rb[:hb[0], 4:][live]), name


@pytest.mark.parametrize("r", [1, 2])
def test_tiny_rank_rows_without_a_plan(M, oracle, r):
    """lora_apply_decode on a rank-1 / rank-2 site applies the rows one by one (no plan): many rows per
    slot, rows without adapter, an evicted slot, a batch far beyond any plan size (out-of-range indices
    are covered by the edge-case test)."""
    c = W.dense_case(f"rows_r{r}", 3400 + r, 5003, 520, 264, 37, r, 4.0 * r, std_a=0.1, std_b=0.1)
    c.token_slot[::13] = -1
    site = dense_site(M, c)
    M.lora_slots_evict(site, 3)
    c.rank[3] = 0
    rows = np.sort(W.rng(34).choice(c.T, 700, replace=False))
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0), rows=rows)


def test_graph_replay_keeps_results_right(M, oracle):
    """A captured graph replays the same kernel arguments; the launches that exchange partial
    results between workgroups must still tell one replay from the next.  Inputs change between
    replays, every replay is compared with the eager result."""
    c = W.dense_case("graph", 3200, 40, 4608, 264, 4, 16, 32.0, std_a=0.05, std_b=0.05)     # few chunks, large d_in: the chunk parts trade k-slice sums through the tagged exchange words
    site = dense_site(M, c)
    plan = M.Plan(40, 4)
    ts = torch.from_numpy(c.token_slot).cuda()
    x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)

    def step():
        M.lora_plan_decode(plan, ts, 4)
        M.lora_apply_decode_planned(site, plan, x, y)
    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(4):
        xr = W.normal_bf16(W.rng(3300 + rep), c.x.shape, 1.0)
        x.copy_(P.dev_bf16(xr))
        y.copy_(P.dev_bf16(c.y0))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = P.host_bits(y)
        y2 = P.dev_bf16(c.y0)
        M.lora_apply_decode_planned(site, plan, x, y2)          # eager, same inputs
        torch.cuda.synchronize()
        assert np.array_equal(got, P.host_bits(y2)), f"replay {rep} differs from the eager launch"
        ref = oracle.apply_decode(xr, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.check_close(got, ref, f"replay {rep}")
    site.check()


def test_decode_layer_graph_replay_with_changing_slots(M, oracle):
    """A layer step as the benchmark issues it (the first launch plans for itself and leaves the plan
    for the planned and grouped launches behind it), captured once and replayed with another
    token -> slot map and other inputs each time: the plan of the replay before must not show, the
    exchange tags must be fresh, every replay goes to the oracle."""
    T, S = 150, 9
    shapes = [(2304, 264, 16), (2304, 520, 16), (2304, 264, 16), (2304, 1032, 16), (1032, 2304, 16), (1032, 2056, 16)]
    slots0 = W.rng(71).integers(-1, S, size=T).astype(np.int32)
    cases = [W.dense_case(f"lg{i}", 3400 + i, T, di, do, S, r, 32.0, token_slot=slots0, std_a=0.05, std_b=0.05)
             for i, (di, do, r) in enumerate(shapes)]
    sites = [dense_site(M, c) for c in cases]
    ts = torch.from_numpy(slots0.copy()).cuda()
    xs = [P.dev_bf16(c.x) for c in cases]
    ys = [P.dev_bf16(c.y0) for c in cases]
    plan = M.Plan(T, S)

    def step():
        M.lora_plan_apply_decode_multi(sites[:3], plan, ts, S, xs[:3], ys[:3])
        M.lora_apply_decode_planned(sites[3], plan, xs[3], ys[3])
        M.lora_apply_decode_multi(sites[4:], plan, xs[4:], ys[4:])
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        g = W.rng(3500 + rep)
        sl = g.integers(-1, S, size=T).astype(np.int32)
        if rep == 1:
            sl[:] = 4                                  # one slot takes every row
        if rep == 2:
            sl[:] = -1; sl[7] = 2                      # a single live row
        ts.copy_(torch.from_numpy(sl))
        xr = [W.normal_bf16(W.rng(3600 + 10 * rep + i), c.x.shape, 1.0) for i, c in enumerate(cases)]
        for x, v, y, c in zip(xs, xr, ys, cases):
            x.copy_(P.dev_bf16(v)); y.copy_(P.dev_bf16(c.y0))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (c, v, y) in enumerate(zip(cases, xr, ys)):
            ref = oracle.apply_decode(v, c.y0, c.A, c.B, c.rank, c.alpha, sl)
            P.check_close(P.host_bits(y), ref, f"{c.name}, replay {rep}")
            P.check_untouched(P.host_bits(y), c.y0, sl < 0, c.name)
    for site in sites:
        site.check()


def test_c2_dense_decode_layer(M, oracle):
    """The seven projections at full size, each in a launch of its own and then in the launch
    configuration the benchmark times (the step's first launch plans inside itself for q|k|v, then o,
    gate|up grouped, down); every one of the 256 rows goes to the oracle, also in the y0 = 0 run."""
    cases = W.c2_dense_decode()
    ts = torch.from_numpy(cases[0].token_slot).cuda()
    plan = M.Plan(256, 64)
    M.lora_plan_decode(plan, ts, 64)
    sites = []
    for c in cases:
        site = dense_site(M, c)
        sites.append(site)

        def runner(y0, site=site, c=c):
            x, y = P.dev_bf16(c.x), P.dev_bf16(y0)
            M.lora_apply_decode_planned(site, plan, x, y)
            torch.cuda.synchronize()
            return P.host_bits(y)
        check_dense(M, oracle, c, runner, report=c.name + " (own launch)")

    def layer(y0s):
        """One layer step as bench.py issues it: four launches, the first one plans."""
        step_plan = M.Plan(256, 64)
        xs = [P.dev_bf16(c.x) for c in cases]
        ys = [P.dev_bf16(y0) for y0 in y0s]
        for gi, grp in enumerate([(0, 1, 2), (3,), (4, 5), (6,)]):
            if gi == 0:
                M.lora_plan_apply_decode_multi([sites[k] for k in grp], step_plan, ts, 64, [xs[k] for k in grp], [ys[k] for k in grp])
            elif len(grp) == 1:
                M.lora_apply_decode_planned(sites[grp[0]], step_plan, xs[grp[0]], ys[grp[0]])
            else:
                M.lora_apply_decode_multi([sites[k] for k in grp], step_plan, [xs[k] for k in grp], [ys[k] for k in grp])
        torch.cuda.synchronize()
        return [P.host_bits(y) for y in ys]

    got = layer([c.y0 for c in cases])
    gz = layer([np.zeros_like(c.y0) for c in cases])
    for c, site, g, z in zip(cases, sites, got, gz):
        ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.check_close(g, ref, c.name + " (layer launches)")
        P.report(c.name + " (layer step launches)", g, ref, c.T, "rows")
        P.check_untouched(g, c.y0, c.token_slot < 0, c.name)
        dref = oracle.apply_decode(c.x, np.zeros_like(c.y0), c.A, c.B, c.rank, c.alpha, c.token_slot)
        P.check_delta(z, dref, c.name + " delta (layer launches)")
        site.check()
        site.close()


def test_c3_rank1_catalog(M, oracle):
    c = W.c3_rank1_catalog()
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0), report=c.name)
    assert np.array_equal(site.meta()[2], c.catalog_id)


# ------------------------------------------------------------------ segmented

def run_seg(M, site, c, y0_bits, seg_off=None, seg_slot=None):
    x, y = P.dev_bf16(c.x), P.dev_bf16(y0_bits)
    M.lora_apply_segmented(site, x, y, c.seg_off if seg_off is None else seg_off,
                           c.seg_slot if seg_slot is None else seg_slot)
    torch.cuda.synchronize()
    return P.host_bits(y)


@pytest.mark.parametrize("r,d_in,d_out", [(64, 208, 328), (64, 1024, 520), (16, 200, 264), (4, 64, 72)])
def test_segmented_small(M, oracle, r, d_in, d_out):
    """Segments that are shorter than, equal to and longer than a tile, an empty segment, a
    segment without adapter; d_out with a ragged last block."""
    seg_off = [0, 1, 33, 33, 100, 132, 140, 205]
    seg_slot = [0, 1, 2, 1, -1, 3, 0]
    c = W.seg_case(f"seg_r{r}", 4000 + r + d_in, 205, 7, d_in, d_out, 4, r, 2.0 * r,
                   seg_off=seg_off, seg_slot=seg_slot, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))
    # the decode path on the same rows must agree with the segmented path to the same bar
    a = run_seg(M, site, c, c.y0)
    b = run_decode(M, site, c, c.y0)
    ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.token_slot)
    P.check_close(a, ref, "seg")
    P.check_close(b, ref, "dec")
    if r == 64:
        # small batches carry their tile tables in the kernel arguments; the copied table must give the same bits
        M.set_tuning("seg_table_copy", 1)
        try:
            assert np.array_equal(run_seg(M, site, c, c.y0), a)
        finally:
            M.set_tuning("seg_table_copy", 0)


def test_segmented_many_tiles_in_batches(M, oracle):
    """More 64-row tiles than one pair of prefill launches covers (several batches per call), one
    long segment, many short ones, segments without adapter and on an empty slot, d_in that is not
    a multiple of the k-unit and d_out that is not a multiple of a wave's 64 outputs."""
    g = W.rng(51)
    lens = [3000] + g.integers(1, 110, size=329).tolist()
    T = int(sum(lens))                                 # about 21000 rows, about 650 tiles
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_slot = g.integers(-1, 6, size=len(lens)).astype(np.int32)
    c = W.seg_case("seg_batches", 4100, T, len(lens), 272, 136, 6, 64, 128.0, ranks=[64, 64, 0, 48, 64, 17],
                   seg_off=seg_off, seg_slot=seg_slot, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))


@pytest.mark.parametrize("n_sub", [2, 3])
def test_segmented_batches_in_flight(M, oracle, n_sub):
    """The rank-64 prefill with several batches in flight (shrinks on the site's second stream, one
    batch ahead of the expands, the partial-result buffers used in halves): the same rows against
    the oracle, twice in a row on one site (the buffers and events are used again), and the same
    bits both times."""
    g = W.rng(52)
    lens = [1500] + g.integers(1, 110, size=200).tolist()
    T = int(sum(lens))
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_slot = g.integers(-1, 6, size=len(lens)).astype(np.int32)
    c = W.seg_case("seg_in_flight", 4200 + n_sub, T, len(lens), 272, 136, 6, 64, 128.0, ranks=[64, 64, 0, 48, 64, 17],
                   seg_off=seg_off, seg_slot=seg_slot, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    M.set_tuning("seg_overlap", n_sub)
    try:
        check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))
        a = run_seg(M, site, c, c.y0)
        assert np.array_equal(a, run_seg(M, site, c, c.y0))
    finally:
        M.set_tuning("seg_overlap", 0)


def test_segmented_in_one_launch(M, oracle):
    """The rank-64 prefill runs as ONE launch by default (the expand's workgroups wait for the flags of
    their tiles): several batches per call, long and short segments, rows without adapter, an empty
    slot; every row against the oracle, three calls in a row on one site (a fresh epoch each time),
    same bits every time, the site reports no wait that gave up, and the pair of launches
    (seg_fused = -1) gives the same bits."""
    g = W.rng(54)
    lens = [2500] + g.integers(1, 110, size=260).tolist()
    T = int(sum(lens))
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_slot = g.integers(-1, 6, size=len(lens)).astype(np.int32)
    c = W.seg_case("seg_one_launch", 4400, T, len(lens), 272, 136, 6, 64, 128.0, ranks=[64, 64, 0, 48, 64, 17],
                   seg_off=seg_off, seg_slot=seg_slot, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))
    a = run_seg(M, site, c, c.y0)
    assert np.array_equal(a, run_seg(M, site, c, c.y0))
    site.check()
    M.set_tuning("seg_fused", -1)
    try:
        b = run_seg(M, site, c, c.y0)
        check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))
    finally:
        M.set_tuning("seg_fused", 0)
    assert np.array_equal(a, b), "the pair of launches and the one launch differ"


def test_prefill_graph_replay_keeps_results_right(M, oracle):
    """The one-launch prefill tells its launches apart by an epoch in device memory, which the launch's
    last workgroup advances: a captured graph, which replays the same kernel arguments, must get a
    fresh epoch per replay, also with eager calls on the same site in between.  Inputs change between
    replays; every replay is compared with the eager result and the oracle."""
    g = W.rng(57)
    lens = [150, 1, 64, 0, 97, 33, 260]
    T = int(sum(lens))
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_slot = np.array([0, 2, 1, 0, -1, 2, 1], np.int32)
    c = W.seg_case("seg_graph", 4500, T, len(lens), 272, 520, 3, 64, 128.0, ranks=[64, 40, 64],
                   seg_off=seg_off, seg_slot=seg_slot, std_a=0.05, std_b=0.05)
    site = dense_site(M, c)
    x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)
    M.lora_apply_segmented(site, x, y, c.seg_off, c.seg_slot)      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        M.lora_apply_segmented(site, x, y, c.seg_off, c.seg_slot)
    for rep in range(4):
        xr = W.normal_bf16(W.rng(4600 + rep), c.x.shape, 1.0)
        x.copy_(P.dev_bf16(xr))
        y.copy_(P.dev_bf16(c.y0))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = P.host_bits(y)
        y2 = P.dev_bf16(c.y0)
        M.lora_apply_segmented(site, x, y2, c.seg_off, c.seg_slot)  # eager, same inputs
        torch.cuda.synchronize()
        assert np.array_equal(got, P.host_bits(y2)), f"replay {rep} differs from the eager call"
        ref = oracle.apply_segmented(xr, c.y0, c.A, c.B, c.rank, c.alpha, c.seg_off, c.seg_slot)
        P.check_close(got, ref, f"replay {rep}")
    site.check()


@pytest.mark.parametrize("seed", [1, 2])
def test_prefill_random_segment_structures(M, oracle, seed):
    """Rank-64 prefill on segment structures nobody picked by hand: segments of 0 .. 200 rows, runs
    of tiny segments (several per 32-row block), one long segment among short ones; slots of rank
    64, of a smaller true rank and empty ones, segments without adapter; widths that are not
    multiples of a workgroup's slice.  (The expand cuts the rows into equal groups of blocks
    wherever the count falls, so every boundary case of that cut shows up here.)"""
    rng = np.random.default_rng(9900 + seed)
    for it in range(12):
        S = int(rng.integers(1, 7))
        ranks = [int(rng.choice([64, 64, 64, 37, 0])) for _ in range(S)]
        if max(ranks) == 0:
            ranks[0] = 64
        nseg = int(rng.integers(1, 40))
        if it % 3 == 0:
            lens = rng.integers(0, 200, size=nseg)
        elif it % 3 == 1:
            lens = rng.integers(0, 12, size=nseg)
        else:
            lens = np.concatenate([rng.integers(0, 40, size=nseg), [int(rng.integers(500, 2500))]])
        lens[0] += 1
        seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        seg_slot = rng.integers(-1, S, size=len(lens)).astype(np.int32)
        d_in, d_out = int(rng.integers(1, 40)) * 16, int(rng.integers(1, 160)) * 8
        print(f"prefill{seed}_{it}: T {int(lens.sum())} segs {len(lens)} d_in {d_in} d_out {d_out} ranks {ranks}", flush=True)
        c = W.seg_case(f"prefill{seed}_{it}", 9950 + 16 * seed + it, int(lens.sum()), len(lens), d_in, d_out, S, 64,
                       (rng.random(S) * 100 + 1).round(2), ranks=ranks, seg_off=seg_off, seg_slot=seg_slot,
                       std_a=0.05, std_b=0.05)
        site = dense_site(M, c)
        rows = None if c.T <= 600 else np.sort(rng.permutation(c.T)[:400])
        check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0), rows=rows)
        site.close()


def test_segmented_small_rank_beyond_one_table(M, oracle):
    """A small-rank segmented call with more 4-row chunks than the site's table area holds (24,575 per
    batch) goes through in several batches: long and short segments, some without adapter, every row
    against the oracle."""
    g = W.rng(53)
    lens = [40000, 3, 25000, 1] + g.integers(1, 900, size=120).tolist()
    T = int(sum(lens))                                 # about 120,000 rows, about 30,000 chunks
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_slot = g.integers(-1, 3, size=len(lens)).astype(np.int32)
    seg_slot[0], seg_slot[2] = 0, 2
    c = W.seg_case("seg_long", 4300, T, len(lens), 16, 24, 3, 4, 8.0, seg_off=seg_off, seg_slot=seg_slot,
                   std_a=0.3, std_b=0.3)
    assert (T + 3) // 4 > 24575
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))


def test_segmented_rejects_bad_offsets(M):
    site = M.Site(64, 64, 64, 2)
    x = torch.zeros((10, 64), dtype=torch.bfloat16, device="cuda")
    for off, sl, code in [([0, 6, 4, 10], [0, 1, 0], -4), ([0, 4, 9], [0, 1], -4), ([1, 4, 10], [0, 1], -4),
                          ([0, 4, 10], [0, 2], -3)]:
        with pytest.raises(M.MLoraError) as e:
            M.lora_apply_segmented(site, x, x.clone(), off, sl)
        assert e.value.status == code


@pytest.mark.parametrize("wide", [False, True])
def test_c5_segmented_full(M, oracle, wide):
    """Full-size prefill (7168 -> 7168 and 7168 -> 18432): all 8192 rows go to the oracle, with the
    batch's y0 and with y0 = 0."""
    c = W.c5_segmented(wide)
    site = dense_site(M, c)
    check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0), report=c.name)
    site.close()
    del site
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ MoE

def moe_site(M, c):
    site = M.Site(c.d_in, c.d_out, c.r_max, c.n_slots, n_experts=c.E)
    upload_all(M, site, c)
    return site


def run_moe(M, site, c, y0_bits, want_idx=True):
    x, y = P.dev_bf16(c.x), P.dev_bf16(y0_bits)
    topk, ts = torch.from_numpy(c.topk).cuda(), torch.from_numpy(c.token_slot).cuda()
    sp = torch.full((c.T * c.K,), -5, dtype=torch.int32, device="cuda") if want_idx else None
    go = torch.full((c.n_slots * c.E + 1,), -5, dtype=torch.int32, device="cuda") if want_idx else None
    M.moe_lora_apply_packed(site, x, y, topk, ts, sp, go)
    torch.cuda.synchronize()
    return P.host_bits(y), (sp.cpu().numpy() if want_idx else None), (go.cpu().numpy() if want_idx else None)


def check_moe(M, oracle, c, site, pairs=None, report=None):
    sel = np.arange(c.T * c.K) if pairs is None else np.asarray(pairs)
    got, sp, go = run_moe(M, site, c, c.y0)
    rsp, rgo = oracle.route_sort(c.topk, c.token_slot, c.rank, c.E)
    assert np.array_equal(go, rgo), "group offsets differ"
    assert np.array_equal(sp, rsp), "sorted pairs differ"
    # oracle on the selected pairs: one-token-per-pair view of the same computation
    tok = sel // c.K
    sub_topk = c.topk.reshape(-1)[sel].reshape(-1, 1)
    ref = oracle.apply_moe(c.x[tok], c.y0[sel], c.A, c.B, c.rank, c.alpha, sub_topk, c.token_slot[tok])
    P.check_close(got[sel], ref, c.name)
    if report:
        assert pairs is None
        P.report(report, got, ref, c.T * c.K, "pairs")
    eff = np.repeat(np.array([s >= 0 and c.rank[s] > 0 for s in c.token_slot]), c.K)
    P.check_untouched(got, c.y0, ~eff, c.name)
    zero = np.zeros_like(c.y0)
    dref = oracle.apply_moe(c.x[tok], zero[sel], c.A, c.B, c.rank, c.alpha, sub_topk, c.token_slot[tok])
    gz, _, _ = run_moe(M, site, c, zero, want_idx=False)
    P.check_delta(gz[sel], dref, c.name + " delta")
    P.noop_must_fail(c.y0[sel], dref, np.nonzero(eff[sel])[0])


@pytest.mark.parametrize("T,K,E,S,r", [(37, 2, 4, 3, 8), (200, 4, 16, 5, 4), (64, 8, 8, 2, 16), (9, 1, 1, 2, 2)])
def test_moe_small(M, oracle, T, K, E, S, r):
    c = W.moe_case(f"moe_{T}_{K}_{E}", 5000 + T, T, K, E, 136, 200, S, r, 2.0 * r, std_a=0.05, std_b=0.05)
    c.token_slot[::7] = -1
    site = moe_site(M, c)
    check_moe(M, oracle, c, site)


def test_moe_empty_slot_and_single_adapter(M, oracle):
    c = W.moe_case("moe_one", 5100, 300, 4, 8, 64, 96, 3, 4, 8.0, ranks=[4, 0, 2],
                   token_slot=np.full(300, 0, dtype=np.int32), std_a=0.1, std_b=0.1)
    site = moe_site(M, c)
    check_moe(M, oracle, c, site)          # every pair on one adapter: groups of ~150 pairs
    c.token_slot[::2] = 1                  # half the tokens point at a slot that never became ready
    c.token_slot[1::4] = 2
    check_moe(M, oracle, c, site)


def test_moe_gate_up_in_one_launch(M, oracle):
    """Gate and up of an expert layer share x and the route plan: moe_lora_apply_multi gives the
    bits of separate calls and the oracle's values; a site of another rank in the list gets a
    launch of its own."""
    T, K, E, S = 150, 4, 8, 4
    shapes = [(256, 136, 8), (256, 136, 8), (256, 72, 4), (2304, 264, 16), (2304, 136, 16)]
    base = W.moe_case("route", 5400, T, K, E, 64, 64, S, 8, 16.0)
    base.token_slot[::6] = -1
    cases = []
    for i, (di, do, r) in enumerate(shapes):
        c = W.moe_case(f"mm{i}", 5401 + i, T, K, E, di, do, S, r, 2.0 * r, std_a=0.05, std_b=0.05)
        c.topk, c.token_slot = base.topk, base.token_slot
        cases.append(c)
    sites = [moe_site(M, c) for c in cases]
    plan = M.Plan(T * K, S * E)
    M.moe_plan_route(plan, torch.from_numpy(base.topk).cuda(), torch.from_numpy(base.token_slot).cuda(), S, E)
    xs = [P.dev_bf16(c.x) for c in cases]
    ys = [P.dev_bf16(c.y0) for c in cases]
    M.moe_lora_apply_multi(sites, plan, xs, ys)
    torch.cuda.synchronize()
    for c, site, x, y in zip(cases, sites, xs, ys):
        ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
        P.check_close(P.host_bits(y), ref, c.name)
        y1 = P.dev_bf16(c.y0)
        M.moe_lora_apply_planned(site, plan, x, y1)
        torch.cuda.synchronize()
        assert torch.equal(y, y1), c.name
    with pytest.raises(M.MLoraError):
        M.lora_apply_decode_multi(sites[:2], plan, xs[:2], ys[:2])      # a route plan is not a decode plan


def test_moe_gate_up_with_long_chunk_runs(M, oracle):
    """The measurement switch rows_chunk_run = 256 (runs of 256 chunks per XCD in the grouped rank-8
    MoE launch) only changes which workgroup takes which chunk: same bits as the default dealing,
    over more chunks than one round of runs holds and a ragged tail."""
    T, K, E, S = 2601, 4, 8, 4
    base = W.moe_case("route", 5500, T, K, E, 64, 64, S, 8, 16.0)
    base.token_slot[::7] = -1
    cases = []
    for i in range(2):
        c = W.moe_case(f"run{i}", 5501 + i, T, K, E, 256, 136, S, 8, 16.0, std_a=0.05, std_b=0.05)
        c.topk, c.token_slot = base.topk, base.token_slot
        cases.append(c)
    sites = [moe_site(M, c) for c in cases]
    plan = M.Plan(T * K, S * E)
    M.moe_plan_route(plan, torch.from_numpy(base.topk).cuda(), torch.from_numpy(base.token_slot).cuda(), S, E)
    xs = [P.dev_bf16(c.x) for c in cases]
    ys = [P.dev_bf16(c.y0) for c in cases]
    M.moe_lora_apply_multi(sites, plan, xs, ys)
    M.set_tuning("rows_chunk_run", 256)
    try:
        zs = [P.dev_bf16(c.y0) for c in cases]
        M.moe_lora_apply_multi(sites, plan, xs, zs)
        torch.cuda.synchronize()
    finally:
        M.set_tuning("rows_chunk_run", 0)
    for c, y, z in zip(cases, ys, zs):
        ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
        P.check_close(P.host_bits(z), ref, c.name)
        assert torch.equal(y, z), c.name


def test_rank_bounded_reads_of_padded_slots(M, oracle):
    """Slots of different true rank in one padded table: with rank-bounded reads a wave fetches
    only the slot's real rows of A (forced on and off here; by default the launch code enables it
    for big launches over tables that hold a padded slot, as in the last case)."""
    ranks = [3, 16, 0, 7, 1, 12]
    cd = W.dense_case("rb_dense", 5500, 90, 256, 520, 6, 16, 24.0, ranks=ranks, std_a=0.05, std_b=0.05)
    cm = W.moe_case("rb_moe", 5501, 120, 4, 8, 136, 200, 4, 8, np.array([4.0, 16.0, 2.0, 10.0]),
                    ranks=[2, 8, 1, 5], std_a=0.05, std_b=0.05)
    c32 = W.dense_case("rb_r32", 5502, 50, 328, 264, 3, 32, 16.0, ranks=[9, 32, 17], std_a=0.05, std_b=0.05)
    sd, sm, s32 = dense_site(M, cd), moe_site(M, cm), dense_site(M, c32)
    for force in (1, -1):
        M.set_tuning("rows_rank_bound", force)
        try:
            check_dense(M, oracle, cd, lambda y0: run_decode(M, sd, cd, y0))
            check_dense(M, oracle, c32, lambda y0: run_decode(M, s32, c32, y0))
            check_moe(M, oracle, cm, sm)
        finally:
            M.set_tuning("rows_rank_bound", 0)
    # a launch with more chunks than the GPU runs at once turns it on by itself
    big = W.moe_case("rb_big", 5503, 1500, 4, 64, 72, 136, 8, 8, 16.0, ranks=[2, 4, 8, 8, 1, 3, 8, 6],
                     std_a=0.05, std_b=0.05)
    rng = np.random.default_rng(5504)
    check_moe(M, oracle, big, moe_site(M, big), pairs=np.sort(rng.choice(1500 * 4, 500, replace=False)))


def test_route_index_build_from_an_unaligned_routing_table(M, oracle):
    """The one-launch build reads a token's experts as 16-byte pieces where it can; a routing table
    that does not start on a 16-byte boundary (a view into a larger buffer) must give the same index."""
    T, K, E, S = 333, 8, 32, 6
    g = W.rng(7790)
    topk = g.integers(0, E, size=(T, K)).astype(np.int32)
    slots = g.integers(-1, S, size=T).astype(np.int32)
    ref_sp, ref_go = oracle.route_sort(topk, slots, np.ones(S, dtype=np.int32), E)
    big = torch.zeros(T * K + 4, dtype=torch.int32, device="cuda")
    for shift in (1, 2, 3):
        tk = big[shift:shift + T * K].view(T, K)
        tk.copy_(torch.from_numpy(topk))
        assert tk.data_ptr() % 16 != 0
        plan = M.Plan(T * K, S * E)
        sp = torch.full((T * K,), -7, dtype=torch.int32, device="cuda")
        go = torch.full((S * E + 1,), -7, dtype=torch.int32, device="cuda")
        M.moe_plan_route(plan, tk, torch.from_numpy(slots).cuda(), S, E, out_sorted_pair=sp, out_group_off=go)
        torch.cuda.synchronize()
        assert np.array_equal(go.cpu().numpy(), ref_go)
        assert np.array_equal(sp.cpu().numpy(), ref_sp)


def test_moe_planned_reuse(M, oracle):
    """One route plan shared by two sites (gate and up share the routing)."""
    ca = W.moe_case("gate", 5200, 120, 4, 8, 128, 64, 4, 8, 16.0, std_a=0.05, std_b=0.05)
    cb = W.moe_case("up", 5201, 120, 4, 8, 128, 64, 4, 8, 16.0, std_a=0.05, std_b=0.05)
    cb.topk, cb.token_slot = ca.topk, ca.token_slot
    plan = M.Plan(120 * 4, 4 * 8)
    topk, ts = torch.from_numpy(ca.topk).cuda(), torch.from_numpy(ca.token_slot).cuda()
    M.moe_plan_route(plan, topk, ts, 4, 8)
    for c in (ca, cb):
        site = moe_site(M, c)
        x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)
        M.moe_lora_apply_planned(site, plan, x, y)
        torch.cuda.synchronize()
        ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
        P.check_close(P.host_bits(y), ref, c.name)


@pytest.mark.parametrize("T,K,E,S", [(37, 2, 4, 3), (1000, 3, 7, 5), (300, 1, 1, 9), (2048, 8, 128, 32), (4096, 8, 64, 64),
                                     (4097, 8, 64, 64), (640, 4, 160, 32), (50, 12, 20, 3), (30, 20, 24, 2), (1500, 16, 64, 8)])
def test_route_index_build_paths_agree(M, oracle, T, K, E, S):
    """The route index build has a one-launch form (every workgroup histograms all pairs in LDS) for
    up to 32768 pairs and 4096 (slot, expert) keys, and a four-launch pipeline for everything else:
    both must give the oracle's stable counting sort bit for bit (sorted pairs, group offsets) and
    leave the same chunk records.  Repeated experts inside a token, rows without adapter, sizes
    that are not multiples of a workgroup's range, one pair more than the one-launch form takes,
    and one key space larger than it takes."""
    g = W.rng(7700 + T + K)
    topk = g.integers(0, E, size=(T, K)).astype(np.int32)
    slots = g.integers(-1, S, size=T).astype(np.int32)
    if T > 100:
        slots[10:90] = 2                              # one crowded group: many members in one range
        topk[10:90, 0] = E - 1
    ref_sp, ref_go = oracle.route_sort(topk, slots, np.ones(S, dtype=np.int32), E)
    tk, ts = torch.from_numpy(topk).cuda(), torch.from_numpy(slots).cuda()
    outs = []
    for pipeline in (0, 1):
        M.set_tuning("plan_pipeline", pipeline)
        try:
            plan = M.Plan(T * K, S * E)
            sp = torch.full((T * K,), -7, dtype=torch.int32, device="cuda")
            go = torch.full((S * E + 1,), -7, dtype=torch.int32, device="cuda")
            for _ in range(2):                         # a plan buffer is used again and again
                M.moe_plan_route(plan, tk, ts, S, E, out_sorted_pair=sp, out_group_off=go)
            torch.cuda.synchronize()
        finally:
            M.set_tuning("plan_pipeline", 0)
        assert np.array_equal(go.cpu().numpy(), ref_go), f"group offsets differ (pipeline={pipeline})"
        assert np.array_equal(sp.cpu().numpy(), ref_sp), f"sorted pairs differ (pipeline={pipeline})"
        hdr, srt, rec = _plan_words(plan, T * K, S * E)
        n_chunks = int(hdr[0])
        assert int(hdr[1]) == int(ref_go[-1])
        assert np.array_equal(srt, ref_sp)
        bound = (T * K + 3 * min(S * E, T * K)) // 4              # records a launch may read: sum of ceil(n_g / 4) <= this
        rec = rec[:8 * bound].reshape(-1, 8)[:, :4].copy()         # key, count, first position, flag (members: through the apply tests)
        rec[n_chunks:, [0, 2, 3]] = 0                             # past the live records only the count (0) is defined
        outs.append((n_chunks, rec))
    assert outs[0][0] == outs[1][0]
    assert np.array_equal(outs[0][1], outs[1][1]), "chunk records differ between the two forms"
    assert np.all(outs[0][1][outs[0][0]:, 1] == 0)


def run_moe_down(M, site, c, y0_bits):
    x, y = P.dev_bf16(c.x), P.dev_bf16(y0_bits)
    topk, ts = torch.from_numpy(c.topk).cuda(), torch.from_numpy(c.token_slot).cuda()
    w = torch.from_numpy(c.w).cuda()
    plan = M.Plan(c.T * c.K, c.n_slots * c.E)
    M.moe_plan_route(plan, topk, ts, c.n_slots, c.E, ready_from=site)
    ws = torch.empty(M.moe_down_workspace_bytes(c.T, c.K, c.d_out), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                     # NaN patterns: rows that must not be read would show
    M.moe_lora_apply_down(site, plan, x, w, ts, ws, y)
    torch.cuda.synchronize()
    return P.host_bits(y)


def check_moe_down(M, oracle, c, site, tokens=None, report=None):
    sel = np.arange(c.T) if tokens is None else np.asarray(tokens)
    pairs = (sel[:, None] * c.K + np.arange(c.K)[None, :]).reshape(-1)
    args = (c.A, c.B, c.rank, c.alpha, c.topk[sel], c.w[sel], c.token_slot[sel])
    ref = oracle.apply_moe_down(c.x[pairs], c.y0[sel], *args)
    got = run_moe_down(M, site, c, c.y0)
    P.check_close(got[sel], ref, c.name)
    if report:
        assert tokens is None
        P.report(report, got, ref, c.T, "tokens")
    eff = np.array([s >= 0 and c.rank[s] > 0 for s in c.token_slot])
    P.check_untouched(got, c.y0, ~eff, c.name)
    zero = np.zeros_like(c.y0)
    dref = oracle.apply_moe_down(c.x[pairs], zero[sel], *args)
    gz = run_moe_down(M, site, c, zero)
    P.check_delta(gz[sel], dref, c.name + " delta")
    P.noop_must_fail(c.y0[sel], dref, np.nonzero(eff[sel])[0])
    assert np.array_equal(got, run_moe_down(M, site, c, c.y0)), "two runs differ: the combine must be deterministic"


@pytest.mark.parametrize("T,K,E,S,r", [(37, 2, 4, 3, 8), (200, 4, 16, 5, 4), (64, 8, 8, 2, 16), (9, 1, 1, 2, 2), (50, 3, 6, 4, 1),
                                       (300, 2, 5, 2, 8), (70, 2, 4, 2, 32), (40, 2, 3, 2, 64), (260, 4, 40, 2, 16),
                                       (300, 2, 4, 70, 8), (64, 4, 300, 2, 8), (33, 16, 520, 1, 4)])
def test_moe_down_small(M, oracle, T, K, E, S, r):
    """Down projection with the routing-weight combine: ragged widths, tokens without adapter, an
    empty slot, K from 1 to 16, every padded rank, odd expert counts (a half-filled last contraction
    step), slots with more tokens than one tile holds, several chunks of the contraction axis, more
    slots than a wave has lanes, expert counts whose tables take most of a compute unit's LDS."""
    ranks = [r] * S
    if S > 2:
        ranks[1] = 0
    c = W.moe_down_case(f"down_{T}_{K}_{E}", 5300 + T, T, K, E, 136, 200, S, r, 2.0 * r, ranks=ranks,
                        std_a=0.05, std_b=0.05)
    c.token_slot[::7] = -1
    site = moe_site(M, c)
    check_moe_down(M, oracle, c, site)


def test_moe_down_pairs_the_plan_left_out(M, oracle):
    """Pairs that the route plan drops must add nothing: expert ids outside [0, E) (masked or padded
    routing tables), and tokens whose slot was not ready at the site the plan was built against
    although it is at the down site.  Whatever the workspace held before (NaN patterns here) must
    not reach y."""
    c = W.moe_down_case("down_masked", 5390, 90, 4, 8, 136, 200, 4, 8, 16.0, std_a=0.05, std_b=0.05)
    c.token_slot[::9] = -1
    masked = c.topk.copy()
    masked[::3, 1] = -1                                # a masked entry in every third token
    masked[5::7, 3] = c.E + 2                          # and some ids past the last expert
    site = moe_site(M, c)
    # the oracle takes valid ids only: the dropped pairs get weight 0 on expert 0
    dropped = (masked < 0) | (masked >= c.E)
    ok_topk, ok_w = np.where(dropped, 0, masked).astype(np.int32), np.where(dropped, 0.0, c.w).astype(np.float32)
    ref = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, ok_topk, ok_w, c.token_slot)

    def run(topk, ready_from):
        x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)
        ts = torch.from_numpy(c.token_slot).cuda()
        plan = M.Plan(c.T * c.K, c.n_slots * c.E)
        M.moe_plan_route(plan, torch.from_numpy(topk).cuda(), ts, c.n_slots, c.E, ready_from=ready_from)
        ws = torch.empty(M.moe_down_workspace_bytes(c.T, c.K, c.d_out), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        M.moe_lora_apply_down(site, plan, x, torch.from_numpy(c.w).cuda(), ts, ws, y)
        torch.cuda.synchronize()
        return P.host_bits(y)
    for pipeline in (0, 1):                            # both forms of the route index build record the pairs' keys
        M.set_tuning("plan_pipeline", pipeline)
        try:
            got = run(masked, site)
        finally:
            M.set_tuning("plan_pipeline", 0)
        P.check_close(got, ref, f"masked ids (pipeline={pipeline})")
        P.check_untouched(got, c.y0, c.token_slot < 0, "masked ids")
    # a plan built against a site where slot 2 is empty: the tokens of slot 2 stay untouched here
    other = moe_site(M, c)
    M.lora_slots_evict(other, 2)
    got = run(c.topk, other)
    slots2 = np.where(c.token_slot == 2, -1, c.token_slot).astype(np.int32)
    ref2 = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.w, slots2)
    P.check_close(got, ref2, "plan from another site")
    P.check_untouched(got, c.y0, slots2 < 0, "plan from another site")
    assert not np.array_equal(got[slots2 >= 0], c.y0[slots2 >= 0])


@pytest.mark.parametrize("seed", [1, 2])
def test_moe_down_random_routing(M, oracle, seed):
    """Down projection over seeded draws of token count, expert count (up to 200), top-k (up to 16), slot
    count (up to 40, so that many slots hold no or one token), rank, widths; tokens without a slot,
    empty slots, and masked routing entries (ids of -1 and ids past the last expert), which must add
    nothing.  Every token goes to the oracle."""
    rng = np.random.default_rng(8800 + seed)
    for it in range(10):
        T, E = int(rng.integers(1, 400)), int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64, 128, 200]))
        K = int(rng.integers(1, min(E, 16) + 1))
        S = int(rng.choice([1, 2, 3, 7, 40]))
        r_max = int(rng.choice([1, 2, 4, 5, 8, 16, 24, 32, 64]))
        ranks = [int(rng.integers(0, r_max + 1)) for _ in range(S)]
        ranks[int(rng.integers(0, S))] = r_max
        d_in, d_out = int(rng.integers(1, 30)) * 8, int(rng.integers(1, 60)) * 8
        print(f"down_rand{seed}_{it}: T {T} K {K} E {E} S {S} r_max {r_max} ranks {ranks[:8]} d_in {d_in} d_out {d_out}", flush=True)
        c = W.moe_down_case(f"down_rand{seed}_{it}", 8850 + 16 * seed + it, T, K, E, d_in, d_out, S, r_max,
                            (rng.random(S) * 30 + 1).round(2), ranks=ranks, std_a=0.05, std_b=0.05)
        c.token_slot[::6] = -1
        site = moe_site(M, c)
        if it % 2 == 0:
            check_moe_down(M, oracle, c, site)
            continue
        # masked routing entries: dropped by the plan; the oracle gets them as weight 0 on expert 0
        masked = c.topk.copy()
        masked[rng.random(masked.shape) < 0.15] = -1
        masked[rng.random(masked.shape) < 0.05] = E + int(rng.integers(0, 3))
        dropped = (masked < 0) | (masked >= E)
        ref = oracle.apply_moe_down(c.x, c.y0, c.A, c.B, c.rank, c.alpha, np.where(dropped, 0, masked).astype(np.int32),
                                    np.where(dropped, 0.0, c.w).astype(np.float32), c.token_slot)
        x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)
        ts = torch.from_numpy(c.token_slot).cuda()
        plan = M.Plan(c.T * c.K, c.n_slots * c.E)
        M.moe_plan_route(plan, torch.from_numpy(masked).cuda(), ts, c.n_slots, c.E, ready_from=site)
        ws = torch.empty(M.moe_down_workspace_bytes(c.T, c.K, c.d_out), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        M.moe_lora_apply_down(site, plan, x, torch.from_numpy(c.w).cuda(), ts, ws, y)
        torch.cuda.synchronize()
        got = P.host_bits(y)
        P.check_close(got, ref, c.name)
        eff = np.array([s_ >= 0 and c.rank[s_] > 0 for s_ in c.token_slot])
        P.check_untouched(got, c.y0, ~eff, c.name)
        site.close()


def test_moe_step_graph_replay_with_changing_routing(M, oracle):
    """Route plan, gate projection in place on the pair rows and down projection with the combine,
    captured once and replayed: the planner's counters must be back at zero for every replay and
    nothing may survive from the routing of the replay before.  The routing, the slots and the
    inputs change between replays (same device buffers); every replay goes to the oracle."""
    T, K, E, S = 150, 4, 12, 3
    cg = W.moe_case("graph_gate", 6100, T, K, E, 136, 264, S, 8, 16.0, std_a=0.05, std_b=0.05)
    cd = W.moe_down_case("graph_down", 6101, T, K, E, 264, 136, S, 8, 16.0, std_a=0.05, std_b=0.05)
    sg, sd = moe_site(M, cg), moe_site(M, cd)
    topk, ts = torch.from_numpy(cg.topk).cuda(), torch.from_numpy(cg.token_slot).cuda()
    w = torch.from_numpy(cd.w).cuda()
    xg, yg = P.dev_bf16(cg.x), P.dev_bf16(cg.y0)
    xd, yd = P.dev_bf16(cd.x), P.dev_bf16(cd.y0)
    plan = M.Plan(T * K, S * E)
    ws = torch.empty(M.moe_down_workspace_bytes(T, K, cd.d_out), dtype=torch.uint8, device="cuda")

    def step():
        M.moe_plan_route(plan, topk, ts, S, E)
        M.moe_lora_apply_planned(sg, plan, xg, yg)
        M.moe_lora_apply_down(sd, plan, xd, w, ts, ws, yd)
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        g = W.rng(6200 + rep)
        tk = W.topk_routing(g, T, E, K)
        sl = g.integers(-1, S, size=T).astype(np.int32)
        if rep == 2:
            sl[:] = 1                                  # one slot takes every token: most groups of the replay before are empty now
        xr = W.normal_bf16(W.rng(6300 + rep), cg.x.shape, 1.0)
        topk.copy_(torch.from_numpy(tk)); ts.copy_(torch.from_numpy(sl))
        xg.copy_(P.dev_bf16(xr)); yg.copy_(P.dev_bf16(cg.y0)); yd.copy_(P.dev_bf16(cd.y0))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_g = oracle.apply_moe(xr, cg.y0, cg.A, cg.B, cg.rank, cg.alpha, tk, sl)
        P.check_close(P.host_bits(yg), ref_g, f"gate, replay {rep}")
        ref_d = oracle.apply_moe_down(cd.x, cd.y0, cd.A, cd.B, cd.rank, cd.alpha, tk, cd.w, sl)
        P.check_close(P.host_bits(yd), ref_d, f"down, replay {rep}")


def test_moe_down_limits(M, oracle):
    """Sixteen experts per token is the most the down projection takes; more is refused before any launch."""
    c = W.moe_down_case("down_k16", 5395, 40, 16, 32, 72, 136, 3, 4, 8.0, std_a=0.05, std_b=0.05)
    check_moe_down(M, oracle, c, moe_site(M, c))
    c17 = W.moe_down_case("down_k17", 5396, 8, 17, 32, 72, 136, 3, 4, 8.0, std_a=0.05, std_b=0.05)
    site = moe_site(M, c17)
    plan = M.Plan(c17.T * c17.K, c17.n_slots * c17.E)
    ts = torch.from_numpy(c17.token_slot).cuda()
    M.moe_plan_route(plan, torch.from_numpy(c17.topk).cuda(), ts, c17.n_slots, c17.E)
    ws = torch.empty(M.moe_down_workspace_bytes(c17.T, c17.K, c17.d_out), dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MLoraError) as e:
        M.moe_lora_apply_down(site, plan, P.dev_bf16(c17.x), torch.from_numpy(c17.w).cuda(), ts, ws, P.dev_bf16(c17.y0))
    assert e.value.status == -6


def test_c4_moe_down_full(M, oracle):
    """The down projection at the c4 size: all 2048 tokens (16384 pairs) against the oracle."""
    c = W.c4_moe_down()
    site = moe_site(M, c)
    check_moe_down(M, oracle, c, site, report=c.name)


def test_upload_from_per_expert_tensors_equals_packed_upload(M, oracle):
    """lora_slots_upload_experts (fragments -> pinned slot image -> one copy per table) must leave
    the same tables as the packed upload: identical outputs bit for bit, also after a re-upload with
    a smaller rank (padding cleared), and right against the oracle."""
    c = W.moe_case("frag", 5400, 90, 4, 16, 136, 200, 3, 8, 16.0, ranks=[8, 5, 8], std_a=0.05, std_b=0.05)
    packed, frag = moe_site(M, c), M.Site(c.d_in, c.d_out, c.r_max, c.n_slots, n_experts=c.E)
    for s_ in range(c.n_slots):
        r = int(c.rank[s_])
        M.lora_slots_upload_experts(frag, s_, s_, [c.A[s_, e, :r, :] for e in range(c.E)],
                                    [c.B[s_, e, :, :r] for e in range(c.E)], r, float(c.alpha[s_]))
    torch.cuda.synchronize()
    a, _, _ = run_moe(M, packed, c, c.y0, want_idx=False)
    b, _, _ = run_moe(M, frag, c, c.y0, want_idx=False)
    assert np.array_equal(a, b)
    ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    P.check_close(b, ref, "fragments")
    c2 = W.moe_case("frag", 5400, 90, 4, 16, 136, 200, 3, 8, 16.0, ranks=[3, 5, 8], std_a=0.05, std_b=0.05)
    M.lora_slots_upload_experts(frag, 0, 9, [c2.A[0, e, :3, :] for e in range(c.E)],
                                [c2.B[0, e, :, :3] for e in range(c.E)], 3, float(c2.alpha[0]))
    torch.cuda.synchronize()
    b2, _, _ = run_moe(M, frag, c2, c2.y0, want_idx=False)
    P.check_close(b2, oracle.apply_moe(c2.x, c2.y0, c2.A, c2.B, c2.rank, c2.alpha, c2.topk, c2.token_slot), "re-upload")
    assert frag.meta()[0].tolist() == [3, 5, 8] and frag.meta()[2][0] == 9


def test_c4_moe_packed_full(M, oracle):
    """moe_lora_apply_packed at the c4 size: all 16384 pairs against the oracle, indices bit for bit."""
    c = W.c4_moe_packed("gate")
    site = moe_site(M, c)
    check_moe(M, oracle, c, site, report=c.name + " (moe_lora_apply_packed)")


def test_c4_gate_up_one_launch_full(M, oracle):
    """The benchmark's launch configuration of c4: gate and up in one launch over one route plan, at
    full size, every pair against the oracle, with the batch's y0 and with y0 = 0."""
    cg, cu = W.c4_moe_packed("gate"), W.c4_moe_packed("up")
    sites = [moe_site(M, cg), moe_site(M, cu)]
    plan = M.Plan(cg.T * cg.K, cg.n_slots * cg.E)
    M.moe_plan_route(plan, torch.from_numpy(cg.topk).cuda(), torch.from_numpy(cg.token_slot).cuda(), cg.n_slots, cg.E)
    x = P.dev_bf16(cg.x)
    for zero in (False, True):
        y0s = [np.zeros_like(c.y0) if zero else c.y0 for c in (cg, cu)]
        ys = [P.dev_bf16(y0) for y0 in y0s]
        M.moe_lora_apply_multi(sites, plan, [x, x], ys)
        torch.cuda.synchronize()
        for c, y0, y in zip((cg, cu), y0s, ys):
            ref = oracle.apply_moe(cg.x, y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
            if zero:
                P.check_delta(P.host_bits(y), ref, c.name + " delta (one launch)")
                P.noop_must_fail(c.y0, ref, np.arange(c.T * c.K))
            else:
                P.check_close(P.host_bits(y), ref, c.name)
                P.report(c.name + " (gate|up in one launch)", P.host_bits(y), ref, c.T * c.K, "pairs")


def test_c4_mixed_rank_full(M, oracle):
    """The gate site with slot ranks drawn from {2, 4, 8} in rank-8 tables, as bench.py times it
    (route plan, then moe_lora_apply_planned, rank-bounded reads by default and switched off): all
    16384 pairs against the oracle."""
    c = W.c4_moe_mixed_rank()
    site = moe_site(M, c)
    plan = M.Plan(c.T * c.K, c.n_slots * c.E)
    M.moe_plan_route(plan, torch.from_numpy(c.topk).cuda(), torch.from_numpy(c.token_slot).cuda(), c.n_slots, c.E)
    x = P.dev_bf16(c.x)
    ref = oracle.apply_moe(c.x, c.y0, c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    dref = oracle.apply_moe(c.x, np.zeros_like(c.y0), c.A, c.B, c.rank, c.alpha, c.topk, c.token_slot)
    for force in (0, -1):
        M.set_tuning("rows_rank_bound", force)
        try:
            y, z = P.dev_bf16(c.y0), P.dev_bf16(np.zeros_like(c.y0))
            M.moe_lora_apply_planned(site, plan, x, y)
            M.moe_lora_apply_planned(site, plan, x, z)
            torch.cuda.synchronize()
        finally:
            M.set_tuning("rows_rank_bound", 0)
        P.check_close(P.host_bits(y), ref, c.name)
        P.check_delta(P.host_bits(z), dref, c.name + " delta")
        if force == 0:
            P.report(c.name, P.host_bits(y), ref, c.T * c.K, "pairs")
    P.noop_must_fail(c.y0, dref, np.arange(c.T * c.K))
    check_moe(M, oracle, c, site)                      # and through the one-call entry point, indices included


# ------------------------------------------------------------------ ABI errors on the device box

def test_catalog_traffic_through_the_residency_manager(M, oracle):
    """Tokens carry catalog ids; the host-side manager maps them to slots (loads on a miss, evicts
    the least recently used adapter), the site tables follow, and every step's result matches the
    oracle applied with the adapters that the requests name."""
    n_cat, n_slots, T = 7, 3, 40
    c = W.dense_case("catalog", 5500, T, 136, 200, n_cat, 8, 16.0, ranks=[8, 5, 8, 1, 8, 3, 8], std_a=0.05, std_b=0.05)
    cat_ids = [1000 * (k + 1) + 7 for k in range(n_cat)]            # catalog id of adapter k
    site = M.Site(c.d_in, c.d_out, c.r_max, n_slots)
    res = M.Resident(n_slots, max_in_flight=1, max_queue=0)
    for cid in cat_ids:
        res.register(cid)
    g = W.rng(5501)
    for step in range(6):
        live = g.choice(n_cat, size=n_slots, replace=False)         # a batch names at most n_slots adapters
        want = g.choice(live, size=T).astype(np.int32)              # adapter index per token
        want[::9] = -1
        pinned = []
        for k in sorted(set(want[want >= 0].tolist())):
            r, slot, _ = res.request(cat_ids[k])
            if r == res.LOAD:
                rk = int(c.rank[k])
                M.lora_slots_upload(site, slot, cat_ids[k], np.ascontiguousarray(c.A[k][:rk]),
                                    np.ascontiguousarray(c.B[k][:, :rk]), rk, float(c.alpha[k]))
                assert res.complete(cat_ids[k])[0] == -1
            else:
                assert r == res.READY
            res.pin(slot)
            pinned.append(slot)
        token_slot = np.array([res.lookup(cat_ids[k]) if k >= 0 else -1 for k in want], dtype=np.int32)
        assert (token_slot[want >= 0] >= 0).all()
        x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)
        M.lora_apply_decode(site, x, y, torch.from_numpy(token_slot).cuda())
        torch.cuda.synchronize()
        ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, want)    # by adapter, not by slot
        P.check_close(P.host_bits(y), ref, f"step {step}")
        P.check_untouched(P.host_bits(y), c.y0, want < 0, f"step {step}")
        cat = site.meta()[2]
        for k in set(want[want >= 0].tolist()):
            assert cat[res.lookup(cat_ids[k])] == cat_ids[k]
        for slot in pinned:
            res.pin(slot, False)
    st = res.stats()
    assert st["loads"] >= n_slots and st["evictions"] >= 1 and st["rejects"] == 0


def test_device_side_catalog_id_lookup(M, oracle):
    """Tokens name adapters by catalog id; the device maps them to slots (bit-exact against the host
    mapping: ready slots only, unknown and negative ids -> -1) and the decode built on it is right."""
    c = W.c3_rank1_catalog()                           # 1024 slots with distinct ids from [0, 10^6)
    site = dense_site(M, c)
    M.lora_slots_evict(site, 5)
    ids = c.catalog_id.copy()
    tok = ids[c.token_slot].astype(np.int64)
    tok[::11] = -1
    tok[1::13] = 999_999_999                           # not in the catalog
    tok[2] = ids[5]                                    # evicted: not ready
    host = {int(v): k for k, v in enumerate(ids) if k != 5}
    want = np.array([host.get(int(v), -1) if v >= 0 else -1 for v in tok], dtype=np.int32)
    out = torch.full((len(tok),), -7, dtype=torch.int32, device="cuda")
    M.lora_slot_lookup(site, torch.from_numpy(tok).cuda(), out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)
    x, y = P.dev_bf16(c.x), P.dev_bf16(c.y0)
    M.lora_apply_decode(site, x, y, out)
    torch.cuda.synchronize()
    ref = oracle.apply_decode(c.x, c.y0, c.A, c.B, c.rank, c.alpha, want)
    P.check_close(P.host_bits(y), ref, "by catalog id")
    P.check_untouched(P.host_bits(y), c.y0, want < 0, "by catalog id")


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes_against_oracle(M, oracle, seed):
    """Shapes nobody picked by hand: seeded draws of rank (powers of two and not), per-slot true ranks
    (empty slots included), d_in / d_out (any multiple of 8), slot and expert counts, batch and
    segment lengths, cycling over the four entry points."""
    rng = np.random.default_rng(7700 + seed)
    dim = lambda lo, hi: int(rng.integers(lo // 8, hi // 8 + 1)) * 8
    for it in range(16):
        kind = ("dense", "moe", "seg", "down")[it % 4]
        r_max = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64]))
        S = int(rng.integers(1, 9))
        ranks = [int(rng.integers(0, r_max + 1)) for _ in range(S)]
        if max(ranks) == 0:
            ranks[0] = r_max
        alpha = (rng.random(S) * 30 + 1).round(2)
        d_in, d_out = dim(16, 1400), dim(8, 1100)
        if kind == "seg" and r_max == 64:
            d_in = (d_in + 15) // 16 * 16
        name, kw = f"rand{seed}_{it}_{kind}", dict(ranks=ranks, std_a=0.05, std_b=0.05)
        print(name, "r_max", r_max, "ranks", ranks, "d_in", d_in, "d_out", d_out, flush=True)
        if kind == "dense":
            c = W.dense_case(name, 7800 + 16 * seed + it, int(rng.integers(1, 400)), d_in, d_out, S, r_max, alpha, **kw)
            site = dense_site(M, c)
            check_dense(M, oracle, c, lambda y0: run_decode(M, site, c, y0, planned=bool(it & 4)))
            continue
        if kind == "seg":
            lens = rng.integers(0, 300, size=int(rng.integers(1, 12)))
            lens[0] += 5
            seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            seg_slot = rng.integers(-1, S, size=len(lens)).astype(np.int32)
            c = W.seg_case(name, 7800 + 16 * seed + it, int(lens.sum()), len(lens), d_in, d_out, S, r_max, alpha,
                           seg_off=seg_off, seg_slot=seg_slot, **kw)
            site = dense_site(M, c)
            check_dense(M, oracle, c, lambda y0: run_seg(M, site, c, y0))
            continue
        T, E = int(rng.integers(1, 200)), int(rng.choice([1, 2, 4, 8, 16]))
        K = int(rng.integers(1, min(E, 8) + 1))
        make = W.moe_case if kind == "moe" else W.moe_down_case
        c = make(name, 7800 + 16 * seed + it, T, K, E, d_in, d_out, S, r_max, alpha, **kw)
        c.token_slot[::5] = -1
        (check_moe if kind == "moe" else check_moe_down)(M, oracle, c, moe_site(M, c))


def test_abi_error_codes(M):
    with pytest.raises(M.MLoraError) as e:
        M.Site(100, 64, 8, 2)                       # d_in not a multiple of 8
    assert e.value.status == -2
    with pytest.raises(M.MLoraError) as e:
        M.Site(64, 64, 65, 2)
    assert e.value.status == -2
    site = M.Site(64, 64, 8, 2)
    A = np.zeros((9, 64), np.uint16)
    B = np.zeros((64, 9), np.uint16)
    with pytest.raises(M.MLoraError) as e:
        M.lora_slots_upload(site, 0, 0, A, B, 9, 1.0)
    assert e.value.status == -2
    with pytest.raises(M.MLoraError) as e:
        M.lora_slots_upload(site, 2, 0, A[:8], B[:, :8].copy(), 8, 1.0)
    assert e.value.status == -3
    moe = M.Site(64, 64, 8, 2, n_experts=2)
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MLoraError) as e:
        M.lora_apply_decode(moe, x, x.clone(), torch.zeros(4, dtype=torch.int32, device="cuda"))
    assert e.value.status == -6
