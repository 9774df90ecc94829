"""Comparison rules shared by the GPU parity tests (not a test module itself).

Floating point: |y_gpu - y_ref| <= 2e-2 + 2e-2 * |y_ref| elementwise against the fp64 oracle
(bf16 in / fp32 accumulate).  Because an N(0, 0.02) adapter can move y by less than that
tolerance, three guards keep the check from passing vacuously: rows without an adapter must be
bit-identical, the run is repeated with y0 = 0 where the output is the LoRA delta alone and must
match to bf16 precision, and the unchanged y0 itself must FAIL the same check.
"""
import numpy as np
import torch

ATOL, RTOL = 2e-2, 2e-2


def dev_bf16(bits, device="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def host_bits(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def widen(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_close(got_bits, ref, what=""):
    got = widen(got_bits)
    err = np.abs(got - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} elements outside 2e-2 + 2e-2|ref|; "
                           f"max abs err {err.max():.4g}")
    return float(err.max()), float((err / np.maximum(np.abs(ref), 1e-30)).max())


def report(config, got_bits, ref, n_units, unit):
    """One line of the per-config error table (max abs error; max relative error where |ref| >= 1e-3).
    Collected by running the GPU tests with -s."""
    got = widen(got_bits)
    err = np.abs(got - ref)
    big = np.abs(ref) >= 1e-3
    rel = float((err[big] / np.abs(ref[big])).max()) if big.any() else 0.0
    print(f"PARITY {config}: {n_units} {unit} compared (all of them), max_abs_err {err.max():.3g}, max_rel_err {rel:.3g}",
          flush=True)


def check_delta(got_bits, delta_ref, what=""):
    """y0 = 0 run: the output is the LoRA delta, rounded once to bf16."""
    got = widen(got_bits)
    rms = float(np.sqrt(np.mean(delta_ref ** 2))) if delta_ref.size else 0.0
    err = np.abs(got - delta_ref)
    bad = err > 2.0 ** -7 * np.abs(delta_ref) + 1e-3 * rms
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} delta elements off; max err {err.max():.4g}, rms {rms:.4g}")
    return rms


def check_untouched(got_bits, y0_bits, rows, what=""):
    assert np.array_equal(got_bits[rows], y0_bits[rows]), f"{what}: rows without an adapter changed"


def noop_must_fail(y0_bits, delta_ref, touched_rows):
    """The y0 = 0 delta check must reject an implementation that does nothing."""
    if len(touched_rows) == 0:
        return
    z = np.zeros_like(y0_bits)
    try:
        check_delta(z[touched_rows], delta_ref[touched_rows])
    except AssertionError:
        return
    raise AssertionError("delta check would accept a no-op kernel")


def summed_magnitude(c):
    """Per output of a dense case: alpha / r * sum_j |B_oj| sum_i |x_i| |A_ji| -- what the fp32 sums of
    shrink and expand add up in absolute value.  Two correct ways of ordering those sums differ by a
    few 2^-24 of it."""
    mag = np.zeros(c.y0.shape)
    xa, Aa, Ba = (np.abs(widen(v)).astype(np.float64) for v in (c.x, c.A, c.B))
    for t in np.nonzero(c.token_slot >= 0)[0]:
        sl = c.token_slot[t]
        mag[t] = (c.alpha[sl] / c.rank[sl]) * (Ba[sl] @ (Aa[sl] @ xa[t]))
    return mag
