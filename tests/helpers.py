"""Shared comparison helpers for the parity tests (no method arithmetic)."""
import sys

import numpy as np

TOL = 2e-2   # max relative error for bf16-compute / fp32-accumulate outputs


def announce(*parts):
    """Name the case on stdout before the GPU step, flushed, so a fault can be traced."""
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def assert_close(got, ref, what, tol=TOL, stored=None, updates=1, scale=None):
    """Floating-point parity bar.
    Headline: max|got-ref| / max|ref| <= tol  (`scale` replaces max|ref| when `got` is a
    sub-selection of a larger tensor).
    Systematic error: rms(got-ref) <= tol/2 * rms(ref); catches a wrong-by-a-factor result
    that a single large reference element could hide in the headline.
    When `got` is an in-place update of a bf16 tensor taken as a difference (y - x), `stored`
    is the reference value of y and `updates` the number of residual updates behind it: each
    one rounds the bf16 stream once (half an ulp, <= 2^-9 |y|), which no kernel can avoid, so
    updates * 2^-9 * rms(y) is allowed on top of the rms bound."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    scale = np.abs(ref).max() if scale is None else scale
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.abs(got - ref)
    headline = err.max() / max(scale, 1e-30)
    rms_err = np.sqrt(np.mean(err ** 2))
    rms_bound = 0.5 * tol * rms
    if stored is not None:
        rms_bound += updates * 2.0 ** -9 * np.sqrt(np.mean(np.asarray(stored, np.float64) ** 2))
    print(f"[parity] {what}: max_rel={headline:.3e} rms_err/rms_ref={rms_err / max(rms, 1e-30):.3e}", flush=True)
    assert headline <= tol, f"{what}: max relative error {headline:.3e} > {tol}"
    assert rms_err <= rms_bound, f"{what}: rms error {rms_err:.3e} > {rms_bound:.3e}"
    return headline


def to_np(t):
    return t.detach().float().cpu().numpy()
