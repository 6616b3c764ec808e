"""Pins for the oracle's encoder ends (patch embedding + position embedding, neck): the library
convolution and layer norm of PyTorch on the CPU, and special cases with closed forms."""
import numpy as np
import torch
import torch.nn.functional as F

import oracle


def test_patch_embed_against_library_convolution():
    rng = np.random.default_rng(0)
    H, W, P, D = 32, 48, 8, 20
    img = rng.normal(size=(3, H, W)).astype(np.float32)
    w = rng.normal(size=(D, 3, P, P)).astype(np.float32) * 0.1
    b = rng.normal(size=D).astype(np.float32)
    pos = rng.normal(size=((H // P) * (W // P), D)).astype(np.float32)
    got = oracle.patch_embed(img, w, b, pos, P)
    ref = F.conv2d(torch.from_numpy(img)[None].double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(), stride=P)[0]
    ref = ref.permute(1, 2, 0).numpy() + pos.reshape(H // P, W // P, D)
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-5)


def test_patch_embed_picks_pixels():
    """A weight that is 1 at (channel 1, ky 2, kx 3) of output 0 copies that pixel of every patch."""
    H = W = 16
    P, D = 4, 2
    img = np.arange(3 * H * W, dtype=np.float32).reshape(3, H, W)
    w = np.zeros((D, 3, P, P), np.float32)
    w[0, 1, 2, 3] = 1.0
    got = oracle.patch_embed(img, w, np.zeros(D, np.float32), np.zeros((16, D), np.float32), P)
    assert np.array_equal(got[:, :, 0], img[1, 2::P, 3::P])
    assert np.all(got[:, :, 1] == 0)


def test_neck_against_library():
    rng = np.random.default_rng(1)
    g, D, C = 7, 24, 16
    x = rng.normal(size=(g, g, D)).astype(np.float32)
    w1 = rng.normal(size=(C, D)).astype(np.float32) * 0.2
    w2 = rng.normal(size=(C, C, 3, 3)).astype(np.float32) * 0.1
    g1, b1, g2, b2 = (rng.normal(size=C).astype(np.float32) for _ in range(4))
    got = oracle.neck(x, w1, g1, b1, w2, g2, b2, eps=1e-6)
    t = torch.from_numpy(x).double().permute(2, 0, 1)[None]                       # [1, D, g, g]
    y = F.conv2d(t, torch.from_numpy(w1).double()[:, :, None, None])
    y = F.layer_norm(y.permute(0, 2, 3, 1), (C,), torch.from_numpy(g1).double(), torch.from_numpy(b1).double(), 1e-6).permute(0, 3, 1, 2)
    y = F.conv2d(y, torch.from_numpy(w2).double(), padding=1)
    y = F.layer_norm(y.permute(0, 2, 3, 1), (C,), torch.from_numpy(g2).double(), torch.from_numpy(b2).double(), 1e-6)
    np.testing.assert_allclose(got, y[0].numpy(), rtol=1e-5, atol=1e-5)


def test_neck_centre_tap_is_pointwise():
    """With only the centre tap of the 3x3 kernel set, the neck is a per-token function: permuting the
    tokens permutes the output (no spatial mixing), and the border needs no special case."""
    rng = np.random.default_rng(2)
    g, D, C = 5, 8, 8
    x = rng.normal(size=(g, g, D)).astype(np.float32)
    w1 = rng.normal(size=(C, D)).astype(np.float32)
    w2 = np.zeros((C, C, 3, 3), np.float32)
    w2[:, :, 1, 1] = rng.normal(size=(C, C)).astype(np.float32)
    ones, zeros = np.ones(C, np.float32), np.zeros(C, np.float32)
    a = oracle.neck(x, w1, ones, zeros, w2, ones, zeros)
    perm = rng.permutation(g * g)
    b = oracle.neck(x.reshape(g * g, D)[perm].reshape(g, g, D), w1, ones, zeros, w2, ones, zeros)
    np.testing.assert_allclose(b.reshape(g * g, C), a.reshape(g * g, C)[perm], rtol=1e-6, atol=1e-6)
