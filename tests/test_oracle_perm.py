"""Pins for the oracle's integer layer: Z-order, stripe-sort, window table, A-shape mask.

Each check is independent of the oracle's own formula: a recursive quadrant walk,
closed forms on 2^k grids, hand-derived prefixes (tests/golden), the phase-view
property of Sec. 4.1 and closed-form tile counts of Alg. 1.
"""
import os

import numpy as np
import pytest

import oracle


def z_walk(gh, gw):
    """Independent derivation: depth-first walk of the bounding 2^k square in
    Z order (top-left, top-right, bottom-left, bottom-right), skipping cells
    outside the gh x gw grid."""
    side = 1
    while side < max(gh, gw):
        side *= 2
    out = []

    def rec(r0, c0, s):
        if r0 >= gh or c0 >= gw:
            return
        if s == 1:
            out.append(r0 * gw + c0)
            return
        hs = s // 2
        rec(r0, c0, hs)
        rec(r0, c0 + hs, hs)
        rec(r0 + hs, c0, hs)
        rec(r0 + hs, c0 + hs, hs)

    rec(0, 0, side)
    return np.array(out, np.int32)


@pytest.mark.parametrize("gh,gw", [(1, 1), (2, 2), (4, 4), (14, 14), (28, 28), (64, 64), (70, 70), (5, 9), (16, 3)])
def test_morton_matches_quadrant_walk(gh, gw):
    assert np.array_equal(oracle.morton_order(gh, gw), z_walk(gh, gw))


@pytest.mark.parametrize("k", [1, 2, 3, 6])
def test_morton_closed_form_pow2(k):
    g = 1 << k
    pi = oracle.morton_order(g, g)
    p = np.arange(g * g)
    col = np.zeros_like(p)
    row = np.zeros_like(p)
    for b in range(k):
        col |= ((p >> (2 * b)) & 1) << b
        row |= ((p >> (2 * b + 1)) & 1) << b
    assert np.array_equal(pi, row * g + col)


def _golden(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "zorder_prefixes.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals = line.split(":")
            name, gh, gw = head.split()
            rows.append((name, int(gh), int(gw), np.array(vals.split(), np.int32)))
    return rows


def test_golden_prefixes(golden_dir):
    rows = _golden(golden_dir)
    assert len(rows) >= 6
    for name, gh, gw, vals in rows:
        pi = oracle.morton_order(gh, gw)
        if name == "pi":
            got = pi
        else:
            got, _ = oracle.stripe_sort(pi, 4)
        assert np.array_equal(got[: vals.size], vals), (name, gh, gw)


@pytest.mark.parametrize("w,G", [(14, 4), (28, 4), (64, 4), (14, 1), (6, 4), (8, 2)])
def test_stripe_definition_and_bijection(w, G):
    pi = oracle.morton_order(w, w)
    sigma, sinv = oracle.stripe_sort(pi, G)
    n = w * w
    # sigma visits every G-th element of pi before the next offset (Sec. 4.1)
    T = pi.reshape(n // G, G)
    assert np.array_equal(sigma, T.T.reshape(-1))
    assert np.array_equal(np.sort(sigma), np.arange(n))
    assert np.array_equal(sigma[sinv], np.arange(n))
    x = np.random.default_rng(0).normal(size=(n, 3)).astype(np.float32)
    assert np.array_equal(x[sigma][sinv], x)          # inverse restores the input bit for bit


@pytest.mark.parametrize("w", [14, 28, 64, 6])
def test_stripe_phase_views(w):
    """G = 4 on an even grid: block g of sigma is exactly the cells with
    (row&1, col&1) == (g>>1, g&1) -- a phase-shifted half-resolution view --
    ordered by the Z-order of (row>>1, col>>1) on the (w/2)^2 grid (Sec. 4.1)."""
    sigma, _ = oracle.grid_sigma(w, 4)
    n = w * w
    half = z_walk(w // 2, w // 2)
    hr, hc = half // (w // 2), half % (w // 2)
    for g in range(4):
        blk = sigma[g * n // 4:(g + 1) * n // 4]
        expect = (2 * hr + (g >> 1)) * w + (2 * hc + (g & 1))
        assert np.array_equal(blk, expect)


def test_stripe_rejects_indivisible():
    with pytest.raises(ValueError):
        oracle.stripe_sort(oracle.morton_order(3, 3), 4)


@pytest.mark.parametrize("g,ws", [(64, 14), (28, 14), (16, 6), (14, 14)])
def test_window_table(g, ws):
    t = oracle.window_table(g, ws, 4)
    nws = -(-g // ws)
    S = ws * ws
    assert t.size == nws * nws * S
    real = t[t >= 0]
    assert np.array_equal(np.sort(real), np.arange(g * g))      # every token exactly once
    assert (t < 0).sum() == (nws * ws) ** 2 - g * g             # 804 pads at g=64, ws=14
    sigma, _ = oracle.grid_sigma(ws, 4)
    for wi in range(nws * nws):
        wr, wc = divmod(wi, nws)
        for p in (0, 1, S // 2, S - 1):
            lr, lc = divmod(int(sigma[p]), ws)
            row, col = wr * ws + lr, wc * ws + lc
            exp = row * g + col if (row < g and col < g) else -1
            assert t[wi * S + p] == exp
    if (g, ws) == (64, 14):
        assert (t < 0).sum() == 804


# closed-form active-tile counts: n_pre*T + (T - n_pre), n_pre = floor(r*T)
@pytest.mark.parametrize("S,Bm,r,count,n_pre", [
    (196, 32, 0.2, 13, 1), (196, 32, 0.3, 19, 2), (196, 32, 0.4, 19, 2), (196, 32, 0.6, 31, 4),
    (196, 32, 1.0, 49, 7), (4096, 128, 0.2, 218, 6), (4096, 128, 0.3, 311, 9), (4096, 128, 0.4, 404, 12),
    (4096, 128, 0.6, 621, 19), (4096, 128, 1.0, 1024, 32), (4096, 128, 0.25, 8 * 32 + 24, 8),
])
def test_block_mask_counts(S, Bm, r, count, n_pre):
    m, npre = oracle.block_mask(S, Bm, r)
    T = -(-S // Bm)
    assert m.shape == (T, T) and npre == n_pre
    assert int(m.sum()) == count
    assert m.any(axis=0).all()                 # every key tile is visible to some row: full K/V set kept
    assert np.all(np.diag(m) == 1)
    for i in range(T):
        assert int(m[i].sum()) == n_pre + (1 if i >= n_pre else 0)
    if r == 1.0:
        assert m.all()


def test_block_mask_rejects_bad_density():
    for r in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(ValueError):
            oracle.block_mask(196, 32, r)
