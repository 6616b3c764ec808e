"""Shared comparison helpers for the parity tests (no method arithmetic)."""
import sys

import numpy as np

TOL = 2e-2   # max relative error for bf16-compute / fp32-accumulate outputs


def announce(*parts):
    """Name the case on stdout before the GPU step, flushed, so a fault can be traced."""
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def assert_close(got, ref, what, tol=TOL):
    """Headline: max|got-ref| / max|ref| <= tol.  Elementwise: |got-ref| <= tol*|ref| + tol*rms(ref)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    scale = np.abs(ref).max()
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.abs(got - ref)
    headline = err.max() / max(scale, 1e-30)
    bound = tol * np.abs(ref) + tol * rms
    worst = (err - bound).max()
    print(f"[parity] {what}: max_rel={headline:.3e} rms_rel={np.sqrt(np.mean(err**2))/max(rms,1e-30):.3e}", flush=True)
    assert headline <= tol, f"{what}: max relative error {headline:.3e} > {tol}"
    assert worst <= 0, f"{what}: elementwise bound exceeded by {worst:.3e}"
    return headline


def to_np(t):
    return t.detach().float().cpu().numpy()
