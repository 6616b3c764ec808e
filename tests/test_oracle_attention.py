"""Pins for the oracle's Stripe-Sort attention (Alg. 1).

- density 1.0 equals dense SAM attention built from library routines (torch fp64)
- a tiny case equals a literal masked N x N softmax written out here in numpy
- at density 1.0 any token order gives the same result (the order only moves the mask)
- constant V gives a constant output; zero rel-pos tables give plain masked SDPA
"""
import numpy as np
import pytest
import torch

import oracle


def _rand(rng, *s, scale=1.0):
    return (scale * rng.normal(size=s)).astype(np.float32)


def dense_sam_attention_torch(q, k, v, rel_h, rel_w, w):
    """softmax(q k^T / sqrt(d) + B) v with SAM's decomposed bias, via torch fp64.
    B[q,(kr,kc)] = q . Rh[qr-kr+w-1] + q . Rw[qc-kc+w-1]."""
    q, k, v, rel_h, rel_w = (torch.from_numpy(np.asarray(a, np.float64)) for a in (q, k, v, rel_h, rel_w))
    h, S, d = q.shape
    coords = torch.arange(w)
    rel_idx = coords[:, None] - coords[None, :] + (w - 1)           # [q, k]
    Rh = rel_h[rel_idx]                                              # [w, w, d]
    Rw = rel_w[rel_idx]
    r_q = q.reshape(h, w, w, d)
    bh = torch.einsum("bhwc,hkc->bhwk", r_q, Rh)                    # [h, qr, qc, kr]
    bw = torch.einsum("bhwc,wkc->bhwk", r_q, Rw)                    # [h, qr, qc, kc]
    attn = (q * d ** -0.5) @ k.transpose(-2, -1)
    attn = (attn.view(h, w, w, w, w) + bh[:, :, :, :, None] + bw[:, :, :, None, :]).view(h, S, S)
    return (torch.softmax(attn, dim=-1) @ v).numpy()


@pytest.mark.parametrize("w,d,h,Bm,G", [(6, 8, 2, 4, 4), (14, 16, 3, 32, 4), (8, 80, 2, 32, 1)])
def test_density_one_is_dense_sam_attention(w, d, h, Bm, G):
    rng = np.random.default_rng(1)
    S = w * w
    q, k, v = _rand(rng, h, S, d), _rand(rng, h, S, d), _rand(rng, h, S, d)
    rel_h, rel_w = _rand(rng, 2 * w - 1, d, scale=0.3), _rand(rng, 2 * w - 1, d, scale=0.3)
    got = oracle.attention(q, k, v, rel_h, rel_w, w, G, Bm, 1.0)
    ref = dense_sam_attention_torch(q, k, v, rel_h, rel_w, w)
    np.testing.assert_allclose(got, ref, rtol=2e-6, atol=2e-6)


def literal_masked_attention(q, k, v, rel_h, rel_w, w, sigma, Bm, n_pre):
    """Brute force, written independently: permute physically with sigma, build
    the S x S boolean tile mask in permuted coordinates, masked softmax, un-permute."""
    h, S, d = q.shape
    qp, kp, vp = q[:, sigma].astype(np.float64), k[:, sigma].astype(np.float64), v[:, sigma].astype(np.float64)
    out = np.zeros((h, S, d))
    tile = np.arange(S) // Bm
    vis = (tile[None, :] < n_pre) | (tile[None, :] == tile[:, None])
    for head in range(h):
        logits = qp[head] @ kp[head].T / np.sqrt(d)
        for a in range(S):
            qa_r, qa_c = divmod(int(sigma[a]), w)
            for b in range(S):
                kb_r, kb_c = divmod(int(sigma[b]), w)
                logits[a, b] += qp[head, a] @ rel_h[qa_r - kb_r + w - 1] + qp[head, a] @ rel_w[qa_c - kb_c + w - 1]
        logits[~vis] = -np.inf
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[head] = p @ vp[head]
    res = np.empty_like(out)
    res[:, sigma] = out
    return res


@pytest.mark.parametrize("w,Bm,r,G", [(4, 4, 0.5, 4), (4, 4, 0.25, 4), (6, 8, 0.4, 4), (4, 4, 0.5, 1), (6, 5, 0.3, 4)])
def test_tiny_brute_force(w, Bm, r, G):
    rng = np.random.default_rng(2)
    S, d, h = w * w, 8, 2
    q, k, v = _rand(rng, h, S, d, scale=2.0), _rand(rng, h, S, d, scale=2.0), _rand(rng, h, S, d)
    rel_h, rel_w = _rand(rng, 2 * w - 1, d), _rand(rng, 2 * w - 1, d)
    sigma, _ = oracle.grid_sigma(w, G)
    T = -(-S // Bm)
    n_pre = int(np.floor(r * T + 1e-6))
    ref = literal_masked_attention(q, k, v, rel_h, rel_w, w, sigma, Bm, n_pre)
    got = oracle.attention(q, k, v, rel_h, rel_w, w, G, Bm, r)
    np.testing.assert_allclose(got, ref, rtol=2e-6, atol=2e-6)
    # the sparse result must differ from the dense one (the mask really bites)
    dense = oracle.attention(q, k, v, rel_h, rel_w, w, G, Bm, 1.0)
    assert np.abs(dense - got).max() > 1e-3


def test_order_is_irrelevant_at_density_one():
    rng = np.random.default_rng(3)
    w, d, h = 6, 8, 2
    S = w * w
    q, k, v = _rand(rng, h, S, d), _rand(rng, h, S, d), _rand(rng, h, S, d)
    rel_h, rel_w = _rand(rng, 2 * w - 1, d), _rand(rng, 2 * w - 1, d)
    base = oracle.attention(q, k, v, rel_h, rel_w, w, 4, 8, 1.0)
    sinv = rng.permutation(S).astype(np.int32)
    other = oracle.attention(q, k, v, rel_h, rel_w, w, 4, 8, 1.0, sinv=sinv)
    np.testing.assert_array_equal(base, other)
    # and at r < 1 a different order gives a different result
    a = oracle.attention(q, k, v, rel_h, rel_w, w, 4, 8, 0.3)
    b = oracle.attention(q, k, v, rel_h, rel_w, w, 4, 8, 0.3, sinv=sinv)
    assert np.abs(a - b).max() > 1e-3


def test_explicit_order_equals_builtin_order():
    rng = np.random.default_rng(4)
    w, d, h = 6, 8, 1
    S = w * w
    q, k, v = _rand(rng, h, S, d), _rand(rng, h, S, d), _rand(rng, h, S, d)
    rel_h, rel_w = _rand(rng, 2 * w - 1, d), _rand(rng, 2 * w - 1, d)
    _, sinv = oracle.grid_sigma(w, 4)
    a = oracle.attention(q, k, v, rel_h, rel_w, w, 4, 8, 0.4)
    b = oracle.attention(q, k, v, rel_h, rel_w, w, 4, 8, 0.4, sinv=sinv)
    np.testing.assert_array_equal(a, b)


def test_constant_v_and_zero_bias():
    rng = np.random.default_rng(5)
    w, d, h, Bm, r = 6, 8, 2, 8, 0.4
    S = w * w
    q, k = _rand(rng, h, S, d), _rand(rng, h, S, d)
    v = np.tile(_rand(rng, 1, 1, d), (h, S, 1))
    zeros = np.zeros((2 * w - 1, d), np.float32)
    out = oracle.attention(q, k, v, zeros, zeros, w, 4, Bm, r)
    np.testing.assert_allclose(out, v, rtol=1e-6, atol=1e-6)        # softmax rows sum to 1
    # zero tables: plain masked SDPA, checked with torch on the literal mask
    v2 = _rand(rng, h, S, d)
    got = oracle.attention(q, k, v2, zeros, zeros, w, 4, Bm, r)
    sigma, sinv = oracle.grid_sigma(w, 4)
    T = -(-S // Bm)
    n_pre = int(np.floor(r * T + 1e-6))
    tile = sinv // Bm                                             # tile of each spatial token
    vis = (tile[None, :] < n_pre) | (tile[None, :] == tile[:, None])
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v2).double(),
        attn_mask=torch.from_numpy(vis)).numpy()
    np.testing.assert_allclose(got, ref, rtol=2e-6, atol=2e-6)
