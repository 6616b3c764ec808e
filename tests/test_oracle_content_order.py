"""Pins for the oracle's content-aware Stripe-Sort order (Sec. 4.1): hand-derived example
(tests/golden), a library sort + the paper's matrix transpose, rank invariants, tie / NaN / -0
rules, the per-window tables, and two properties of the attention that uses it: at r = 1 the
order cannot matter, and scores that decrease along the Z-order reproduce the position-only path."""
import os

import numpy as np
import pytest

import oracle
from paper_2605_17633_amd import inputs


def golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "content_order_example.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        head, sc, sg = line.split(":")
        yield int(head.split()[1]), np.array(sc.split(), np.float32), np.array(sg.split(), np.int32)


def test_worked_example():
    n = 0
    for G, scores, sigma in golden():
        got, inv = oracle.content_order(scores, G)
        assert np.array_equal(got, sigma)
        assert np.array_equal(inv[sigma], np.arange(sigma.size))
        n += 1
    assert n == 3


@pytest.mark.parametrize("n,G", [(196, 4), (4096, 4), (784, 4), (16, 1), (36, 2)])
def test_against_library_sort_and_transpose(n, G):
    rng = np.random.default_rng(n)
    scores = inputs.lognormal_scores(rng, 1, n)[0]
    scores[rng.integers(0, n, n // 8)] = scores[0]                 # planted ties
    pi = np.lexsort((np.arange(n), -scores.astype(np.float64)))    # score descending, then index ascending
    want = pi.reshape(n // G, G).T.reshape(-1)                     # T[t,g] = pi[tG+g]; flatten(T^T)
    sigma, inv = oracle.content_order(scores, G)
    assert np.array_equal(sigma, want.astype(np.int32))
    assert np.array_equal(np.sort(sigma), np.arange(n))            # bijection
    assert np.array_equal(sigma[inv], np.arange(n))


def test_rank_structure():
    """Block g of sigma holds the ranks g, g+G, g+2G, ...: every block is a uniformly subsampled
    mixture from the most to the least salient token, and the very first position is the arg-max."""
    n, G = 4096, 4
    rng = np.random.default_rng(3)
    scores = rng.random(n).astype(np.float32)                      # distinct with probability ~1
    assert np.unique(scores).size == n
    sigma, _ = oracle.content_order(scores, G)
    rank = np.empty(n, np.int64)
    rank[np.argsort(-scores, kind="stable")] = np.arange(n)
    blocks = rank[sigma].reshape(G, n // G)
    for g in range(G):
        assert np.array_equal(blocks[g], g + G * np.arange(n // G))
    assert sigma[0] == int(np.argmax(scores))
    assert sigma[n // G - 1 + (G - 1) * (n // G)] == int(np.argmin(scores))


def test_ties_nan_and_signed_zero():
    n, G = 16, 4
    sigma, _ = oracle.content_order(np.ones(n, np.float32), G)     # all equal: pi = identity
    assert np.array_equal(sigma, np.arange(n).reshape(n // G, G).T.reshape(-1))
    s = np.array([0.0, -0.0, np.nan, 1.0, -np.inf, np.nan, 2.0, -0.0], np.float32)
    sigma, _ = oracle.content_order(s, 1)
    # 2.0, 1.0, the three zeros in index order (-0 == +0), then NaN and -inf together in index order
    assert list(sigma) == [6, 3, 0, 1, 7, 2, 4, 5]


@pytest.mark.parametrize("g,ws", [(28, 14), (64, 14), (16, 0), (9, 4)])
def test_content_tables(g, ws):
    rng = np.random.default_rng(g)
    scores = rng.random((g, g)).astype(np.float32)
    table, sig = oracle.content_tables(scores, g, ws, 4)
    w = ws if ws > 0 else g
    nws = -(-g // w)
    S = w * w
    table = table.reshape(nws * nws, S)
    real = table[table >= 0]
    assert np.array_equal(np.sort(real), np.arange(g * g))         # every token exactly once
    for win in range(nws * nws):
        wr, wc = divmod(win, nws)
        assert np.array_equal(np.sort(sig[win]), np.arange(S))     # a permutation of the window's cells
        row, col = wr * w + sig[win] // w, wc * w + sig[win] % w
        inside = (row < g) & (col < g)
        assert np.array_equal(table[win][inside], (row * g + col)[inside])
        assert np.all(table[win][~inside] == -1)
        # padding ranks last: undoing the stripe interleave, the ranks of pad cells are the highest
        pi = sig[win].reshape(4, S // 4).T.reshape(-1)
        n_real = int(inside.sum())
        prow, pcol = wr * w + pi // w, wc * w + pi % w
        assert np.all((prow[:n_real] < g) & (pcol[:n_real] < g))
        m = scores[prow[:n_real], pcol[:n_real]]
        assert np.all(np.diff(m) <= 0)                              # real cells in descending score


def small_block(seed, g, ws):
    rng = np.random.default_rng(seed)
    D, heads, Dm = 64, 2, 128
    w = ws if ws > 0 else g
    wt = inputs.block_weights(rng, D, heads, Dm, w)
    for k in ("wqkv", "rel_h", "rel_w"):
        wt[k] = inputs.bf16_round(wt[k] * 8)                       # peaky softmax: the mask matters
    x = inputs.token_field(rng, 1, g, D)[0]
    keep = oracle.select_tokens(oracle.score_tokens(x), oracle.keep_count(g * g, 0.5))
    return wt, x, keep, heads


@pytest.mark.parametrize("g,ws,Bm", [(8, 4, 4), (8, 0, 16), (10, 4, 4)])
def test_dense_limit_ignores_the_order(g, ws, Bm):
    """r = 1: every key is visible whatever the order, so the content-aware block equals the
    position-only block."""
    wt, x, keep, heads = small_block(5, g, ws)
    scores = np.random.default_rng(6).random((g, g)).astype(np.float32)
    a = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, 1.0, keep)
    b = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, 1.0, keep, order_scores=scores)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-6)


@pytest.mark.parametrize("g,ws,Bm,r", [(8, 4, 4, 0.5), (8, 0, 16, 0.5), (16, 8, 8, 0.3)])
def test_scores_along_the_z_order_give_the_position_only_block(g, ws, Bm, r):
    """If the scores decrease along each group's Z-order, ranking by score IS the Z-order, and the
    content-aware block must reproduce the position-only block at r < 1 (no padding here)."""
    wt, x, keep, heads = small_block(7, g, ws)
    w = ws if ws > 0 else g
    zrank = np.empty(w * w, np.int64)
    zrank[oracle.morton_order(w, w)] = np.arange(w * w)
    local = -zrank.reshape(w, w).astype(np.float32)
    scores = np.tile(local, (g // w, g // w))
    a = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, r, keep)
    b = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, r, keep, order_scores=scores)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-6)
    # and a different order does change the result at r < 1 (the mask is not vacuous)
    c = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, r, keep, order_scores=-scores)
    assert np.abs(a - c).max() > 1e-3
