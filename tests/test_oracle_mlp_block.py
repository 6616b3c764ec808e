"""Pins for the oracle's token scores (Eq. 1), keep-set selection, the
Residual-Consistency MLP (Sec. 4.2) and the whole block.

Library routines (scipy correlate, numpy sort, torch layer_norm/linear/gelu/
softmax) and closed forms stand on the other side of every comparison.
"""
import numpy as np
import pytest
import scipy.ndimage
import torch
import torch.nn.functional as F

import oracle
from paper_2605_17633_amd import inputs


# ------------------------------------------------------------------ scores
def test_sobel_matches_library_correlation():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(9, 13, 5)).astype(np.float32)
    c = x.astype(np.float64).sum(-1)
    sx = np.array([[-1, 0, 1], [-2, 0, 2], [-1, 0, 1]], np.float64)
    gx = scipy.ndimage.correlate(c, sx, mode="constant", cval=0.0)
    gy = scipy.ndimage.correlate(c, sx.T, mode="constant", cval=0.0)
    np.testing.assert_allclose(oracle.score_tokens(x), np.sqrt(gx ** 2 + gy ** 2), rtol=1e-6, atol=1e-6)


def test_sobel_closed_forms():
    g, D = 8, 3
    const = np.full((g, g, D), 0.75, np.float32)
    M = oracle.score_tokens(const)
    assert np.all(M[1:-1, 1:-1] == 0.0) and np.all(M[0] > 0)       # zero padding makes an edge at the border
    a = 0.5
    ramp = np.zeros((g, g, D), np.float32)
    ramp[..., 0] = a * np.arange(g)[None, :]                         # c = a*col  ->  gx = 8a, gy = 0
    np.testing.assert_allclose(oracle.score_tokens(ramp)[1:-1, 1:-1], 8 * a, rtol=1e-6)
    ramp_r = np.zeros((g, g, D), np.float32)
    ramp_r[..., 1] = a * np.arange(g)[:, None]                       # c = a*row  ->  gx = 0, gy = 8a
    np.testing.assert_allclose(oracle.score_tokens(ramp_r)[1:-1, 1:-1], 8 * a, rtol=1e-6)
    # channels are summed BEFORE squaring: two opposite channels cancel
    anti = np.zeros((g, g, 2), np.float32)
    anti[..., 0] = np.arange(g)[None, :]
    anti[..., 1] = -np.arange(g)[None, :]
    assert np.all(oracle.score_tokens(anti) == 0.0)


# ------------------------------------------------------------------ select
def test_keep_count():
    assert oracle.keep_count(4096, 0.4) == 1638
    assert oracle.keep_count(4096, 0.3) == 1228
    assert oracle.keep_count(784, 0.4) == 313
    assert oracle.keep_count(4096, 1.0) == 4096
    assert oracle.keep_count(10, 0.01) == 1
    assert oracle.keep_count(4096, 0.2) == 819 and oracle.keep_count(4096, 0.6) == 2457


@pytest.mark.parametrize("n,K,seed", [(17, 5, 0), (784, 313, 1), (4096, 1638, 2), (64, 64, 3), (64, 1, 4)])
def test_select_matches_full_sort(n, K, seed):
    rng = np.random.default_rng(seed)
    s = np.exp(rng.normal(size=n)).astype(np.float32)
    s[rng.integers(0, n, n // 4)] = s[rng.integers(0, n, n // 4)]     # plant duplicates
    order = np.lexsort((np.arange(n), -s.astype(np.float64)))          # score desc, index asc
    ref = np.sort(order[:K]).astype(np.int32)
    assert np.array_equal(oracle.select_tokens(s, K), ref)


def test_select_ties_and_signed_zero():
    assert np.array_equal(oracle.select_tokens(np.ones(10, np.float32), 4), [0, 1, 2, 3])
    s = np.array([1, 5, 5, 5, 0, 5, 9], np.float32)
    assert np.array_equal(oracle.select_tokens(s, 3), [1, 2, 6])       # tie at the threshold -> lower index
    z = np.array([-0.0, 0.0, -0.0, 0.0], np.float32)
    assert np.array_equal(oracle.select_tokens(z, 2), [0, 1])          # -0.0 == +0.0
    nan = np.array([np.nan, 1.0, -np.inf, 2.0], np.float32)
    assert np.array_equal(oracle.select_tokens(nan, 3), [0, 1, 3])     # NaN ranks as -inf; tie with -inf -> lower index


# ------------------------------------------------------------------ MLP
def _mlp_torch(x, wt, eps=1e-6):
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    xx = t(x)
    u = F.layer_norm(xx, (xx.shape[-1],), t(wt["ln2_g"]), t(wt["ln2_b"]), eps)
    return (xx + F.linear(F.gelu(F.linear(u, t(wt["w1"]), t(wt["b1"]))), t(wt["w2"]), t(wt["b2"]))).numpy()


def test_routed_mlp_dense_limit_and_bypass():
    rng = np.random.default_rng(7)
    n, D, Dm = 50, 32, 96
    wt = inputs.block_weights(rng, D, 4, Dm, 6)
    for kname in ("w1", "w2", "b1", "b2"):
        wt[kname] = wt[kname] * 10                                    # make the update sizeable
    x = rng.normal(size=(n, D)).astype(np.float32)
    args = (wt["ln2_g"], wt["ln2_b"], wt["w1"], wt["b1"], wt["w2"], wt["b2"])
    dense = oracle.routed_mlp(x, np.arange(n), *args)
    ref = _mlp_torch(x, wt)
    np.testing.assert_allclose(dense, ref, rtol=1e-6, atol=1e-6)
    assert np.abs(dense - x).max() > 1e-2
    keep = np.array([3, 4, 17, 41], np.int32)
    y = oracle.routed_mlp(x, keep, *args)
    rest = np.setdiff1d(np.arange(n), keep)
    assert np.array_equal(y[rest].view(np.uint32), x[rest].view(np.uint32))      # bypass rows bit-identical
    np.testing.assert_array_equal(y[keep], dense[keep])                          # per-token formula
    single = oracle.routed_mlp(x, np.array([17], np.int32), *args)
    np.testing.assert_array_equal(single[17], dense[17])


# ------------------------------------------------------------------ block
def dense_sam_block_torch(x, wt, heads, ws, eps=1e-6):
    """Dense SAM ViT block from library ops, fp64: pre-LN, window partition with
    zero padding after the norm, attention with decomposed rel-pos, un-partition,
    residual, pre-LN MLP with erf GELU, residual."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    xx = t(x)[None]                                                  # [1,g,g,D]
    g, D = xx.shape[1], xx.shape[3]
    d = D // heads
    u = F.layer_norm(xx, (D,), t(wt["ln1_g"]), t(wt["ln1_b"]), eps)
    w = ws if ws > 0 else g
    pad = (w - g % w) % w
    u = F.pad(u, (0, 0, 0, pad, 0, pad))
    gp = g + pad
    nw = gp // w
    win = u.view(1, nw, w, nw, w, D).permute(0, 1, 3, 2, 4, 5).reshape(nw * nw, w * w, D)
    qkv = F.linear(win, t(wt["wqkv"]), t(wt["bqkv"])).reshape(nw * nw, w * w, 3, heads, d).permute(2, 0, 3, 1, 4)
    q, k, v = qkv[0], qkv[1], qkv[2]                                # [nW,h,S,d]
    coords = torch.arange(w)
    idx = coords[:, None] - coords[None, :] + (w - 1)
    Rh, Rw = t(wt["rel_h"])[idx], t(wt["rel_w"])[idx]
    r_q = q.reshape(nw * nw, heads, w, w, d)
    bh = torch.einsum("nbhwc,hkc->nbhwk", r_q, Rh)
    bw = torch.einsum("nbhwc,wkc->nbhwk", r_q, Rw)
    attn = (q * d ** -0.5) @ k.transpose(-2, -1)
    attn = (attn.view(nw * nw, heads, w, w, w, w) + bh[..., :, None] + bw[..., None, :]).view(nw * nw, heads, w * w, w * w)
    o = (torch.softmax(attn, -1) @ v).permute(0, 2, 1, 3).reshape(nw * nw, w * w, D)
    o = F.linear(o, t(wt["wproj"]), t(wt["bproj"]))
    o = o.view(1, nw, nw, w, w, D).permute(0, 1, 3, 2, 4, 5).reshape(1, gp, gp, D)[:, :g, :g]
    x1 = xx + o
    u2 = F.layer_norm(x1, (D,), t(wt["ln2_g"]), t(wt["ln2_b"]), eps)
    y = x1 + F.linear(F.gelu(F.linear(u2, t(wt["w1"]), t(wt["b1"]))), t(wt["w2"]), t(wt["b2"]))
    return y[0].numpy(), x1[0].numpy()


@pytest.mark.parametrize("g,ws,Bm", [(16, 6, 8), (12, 0, 32), (14, 14, 32)])
def test_block_density_one_is_dense_sam_block(g, ws, Bm):
    rng = np.random.default_rng(11)
    D, heads, Dm = 32, 4, 64
    w = ws if ws > 0 else g
    wt = inputs.block_weights(rng, D, heads, Dm, w)
    for kname in ("wqkv", "wproj", "w1", "w2", "rel_h", "rel_w"):
        wt[kname] = wt[kname] * 8                                     # non-trivial attention and MLP
    x = inputs.token_field(rng, 1, g, D)[0]
    n = g * g
    y = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, 1.0, np.arange(n))
    ref, ref_x1 = dense_sam_block_torch(x, wt, heads, ws)
    np.testing.assert_allclose(y, ref, rtol=1e-5, atol=1e-5)
    assert np.abs(ref - x).max() > 0.05
    # sparse block: rows outside the keep-set carry exactly the attention half, untouched by the MLP
    keep = oracle.select_tokens(oracle.score_tokens(x), oracle.keep_count(n, 0.4))
    ys = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, 1.0, keep)
    y_attn_only = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, 1.0, np.zeros(0, np.int32))
    np.testing.assert_allclose(y_attn_only.reshape(n, D), ref_x1.reshape(n, D), rtol=1e-5, atol=1e-5)
    rest = np.setdiff1d(np.arange(n), keep)
    assert np.array_equal(ys.reshape(n, D)[rest].view(np.uint32), y_attn_only.reshape(n, D)[rest].view(np.uint32))
    np.testing.assert_array_equal(ys.reshape(n, D)[keep], y.reshape(n, D)[keep])


def test_block_sparse_attention_differs_and_matches_parts():
    """At r < 1 the block must equal: attention routine on the block's own qkv
    (library linear) + library proj + oracle MLP -- i.e. the composition adds nothing."""
    rng = np.random.default_rng(12)
    g, ws, D, heads, Dm, Bm, r = 12, 6, 32, 4, 64, 8, 0.4
    d = D // heads
    wt = inputs.block_weights(rng, D, heads, Dm, ws)
    for kname in ("wqkv", "wproj", "w1", "w2", "rel_h", "rel_w"):
        wt[kname] = wt[kname] * 8
    x = inputs.token_field(rng, 1, g, D)[0]
    n = g * g
    keep = np.arange(0, n, 3, dtype=np.int32)
    y = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, r, keep)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    u = F.layer_norm(t(x), (D,), t(wt["ln1_g"]), t(wt["ln1_b"]), 1e-6)
    x1 = np.array(x, np.float64)
    for wr in range(g // ws):
        for wc in range(g // ws):
            win = u[wr * ws:(wr + 1) * ws, wc * ws:(wc + 1) * ws].reshape(ws * ws, D)
            qkv = F.linear(win, t(wt["wqkv"]), t(wt["bqkv"])).reshape(ws * ws, 3, heads, d).permute(1, 2, 0, 3).numpy()
            o = oracle.attention(qkv[0], qkv[1], qkv[2], wt["rel_h"], wt["rel_w"], ws, 4, Bm, r)   # [h,S,d]
            o = F.linear(t(o).permute(1, 0, 2).reshape(ws * ws, D), t(wt["wproj"]), t(wt["bproj"])).numpy()
            x1[wr * ws:(wr + 1) * ws, wc * ws:(wc + 1) * ws] += o.reshape(ws, ws, D)
    ref = oracle.routed_mlp(x1.reshape(n, D).astype(np.float32), keep, wt["ln2_g"], wt["ln2_b"],
                            wt["w1"], wt["b1"], wt["w2"], wt["b2"]).reshape(g, g, D)
    np.testing.assert_allclose(y, ref, rtol=1e-5, atol=1e-5)
    dense = oracle.encoder_block(x, oracle.BlockWeights(**wt), heads, ws, 4, Bm, 1.0, keep)
    assert np.abs(dense - y).max() > 1e-3


def test_encoder_reuses_one_keep_set():
    rng = np.random.default_rng(13)
    shape = inputs.ModelShape("tiny", 32, 3, 4, 64, (2,), 6)
    g = 12
    blocks = [oracle.BlockWeights(**b) for b in inputs.encoder_weights(5, shape, g)]
    x = inputs.token_field(rng, 1, g, shape.D)[0]
    y, keep = oracle.encoder(x, blocks, shape.heads, shape.ws, shape.global_blocks, 4, 0.5, 0.4,
                             Bm_window=8, Bm_global=32)
    assert keep.size == oracle.keep_count(g * g, 0.4)
    assert np.array_equal(keep, oracle.select_tokens(oracle.score_tokens(x), keep.size))
    assert y.shape == x.shape and np.isfinite(y).all()


@pytest.mark.parametrize("global_blocks,content_order", [((1,), False), ((0, 3), False), ((), False), ((2,), True)])
def test_encoder_is_the_loop_over_its_pinned_blocks(global_blocks, content_order):
    """Pin of the stack composition: `oracle.encoder` must equal a loop written out here over the pinned
    single-block routine, with the window / global dispatch, the mask tile of either kind of block, the one
    keep-set and (content-aware order) the one score map taken from the encoder INPUT.  The global flags are
    non-trivial (first block, middle blocks, none), the two mask tiles differ and the rel-pos tables of the two
    kinds of block have different shapes, so a wrong flag, a swapped tile or a keep-set recomputed per block fails."""
    rng = np.random.default_rng(17)
    depth, g, ws, heads, D, Dm = 4, 12, 6, 4, 32, 64
    shape = inputs.ModelShape("tiny", D, depth, heads, Dm, tuple(global_blocks), ws)
    wts = inputs.encoder_weights(6, shape, g)
    for w in wts:                                   # large enough that every block visibly changes the stream
        for kname in ("wqkv", "wproj", "w1", "w2", "rel_h", "rel_w"):
            w[kname] = inputs.bf16_round(w[kname] * 8)
    blocks = [oracle.BlockWeights(**w) for w in wts]
    x = inputs.token_field(rng, 1, g, D)[0]
    r, rho, Bw, Bg = 0.5, 0.4, 8, 32
    y, keep = oracle.encoder(x, blocks, heads, ws, global_blocks, 4, r, rho, Bm_window=Bw, Bm_global=Bg,
                             content_order=content_order)
    scores = oracle.score_tokens(x)
    keep_ref = oracle.select_tokens(scores, oracle.keep_count(g * g, rho))
    assert np.array_equal(keep, keep_ref)
    z = x
    for i in range(depth):
        is_global = i in global_blocks
        z_next = oracle.encoder_block(z, blocks[i], heads, 0 if is_global else ws, 4, Bg if is_global else Bw, r, keep_ref,
                                      order_scores=scores if content_order else None)
        assert np.abs(z_next - z).max() > 1e-3       # the block is live
        # the other kind of block gives something else here (so the flag matters); only possible where the
        # rel-pos tables fit, i.e. never: a swapped flag is rejected by the shape check instead
        with pytest.raises(AssertionError):
            oracle.encoder_block(z, blocks[i], heads, ws if is_global else 0, 4, Bw if is_global else Bg, r, keep_ref)
        z = z_next
    assert np.array_equal(y, z)
    # a keep-set recomputed from a later block's input would differ: the stream's scores move
    assert not np.array_equal(keep_ref, oracle.select_tokens(oracle.score_tokens(z), keep_ref.size))
    if content_order:
        y_pos, _ = oracle.encoder(x, blocks, heads, ws, global_blocks, 4, r, rho, Bm_window=Bw, Bm_global=Bg)
        assert np.abs(y_pos - y).max() > 1e-4        # the option is live


def test_block_halves_compose_to_the_block():
    """encoder_block_halves (attention half with an empty keep-set, then the routed MLP) is the block, bit for bit."""
    rng = np.random.default_rng(19)
    shape = inputs.ModelShape("tiny", 32, 1, 4, 64, (), 6)
    g = 12
    wt = oracle.BlockWeights(**inputs.encoder_weights(7, shape, g)[0])
    x = inputs.token_field(rng, 1, g, shape.D)[0]
    keep = oracle.select_tokens(oracle.score_tokens(x), 50)
    for ws, Bm in ((6, 8), ):
        x1, y = oracle.encoder_block_halves(x, wt, shape.heads, ws, 4, Bm, 0.5, keep)
        assert np.array_equal(y, oracle.encoder_block(x, wt, shape.heads, ws, 4, Bm, 0.5, keep))
        rest = np.setdiff1d(np.arange(g * g), keep)
        assert np.array_equal(x1.reshape(g * g, -1)[rest], y.reshape(g * g, -1)[rest])     # bypass rows: y is x1
        assert np.abs(x1 - x).max() > 1e-4 and np.abs(y - x1).max() > 1e-4
