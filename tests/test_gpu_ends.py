"""Parity of the encoder ends (patch embedding + position embedding, neck) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from helpers import announce, assert_close, to_np
from paper_2605_17633_amd import binding as B
from paper_2605_17633_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev_bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV).to(torch.bfloat16).contiguous()


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


@pytest.mark.parametrize("Bn,H,W,P,D", [(2, 128, 160, 16, 256), (1, 1024, 1024, 16, 1280), (3, 64, 64, 8, 128)])
def test_patch_embed(Bn, H, W, P, D):
    announce("patch embed", Bn, H, W, P, D)
    rng = np.random.default_rng(H + D)
    img = inputs.bf16_round(rng.normal(size=(Bn, 3, H, W)).astype(np.float32))
    w = inputs.bf16_round((rng.normal(size=(D, 3, P, P)) * 0.05).astype(np.float32))
    b = (rng.normal(size=D) * 0.1).astype(np.float32)
    N = (H // P) * (W // P)
    pos = inputs.bf16_round(rng.normal(size=(N, D)).astype(np.float32))
    x = B.ssam_patch_embed(dev_bf16(img), dev_bf16(w.reshape(D, -1)), dev_f32(b), dev_bf16(pos), P)
    got = to_np(x)
    for bi in range(Bn):
        ref = oracle.patch_embed(img[bi], w, b, pos, P).reshape(N, D)
        assert_close(got[bi] - pos, ref - pos, f"patch embedding image {bi}", stored=ref)


@pytest.mark.parametrize("Bn,g,D,C", [(2, 12, 256, 128), (1, 64, 1280, 256), (3, 9, 64, 128)])
def test_neck(Bn, g, D, C):
    announce("neck", Bn, g, D, C)
    rng = np.random.default_rng(g + D)
    x = inputs.bf16_round(rng.normal(size=(Bn, g, g, D)).astype(np.float32))
    w1 = inputs.bf16_round((rng.normal(size=(C, D)) / np.sqrt(D)).astype(np.float32))
    w2 = inputs.bf16_round((rng.normal(size=(C, C, 3, 3)) / np.sqrt(9 * C)).astype(np.float32))
    g1, b1, g2, b2 = (1.0 + 0.1 * rng.normal(size=C)).astype(np.float32), (0.1 * rng.normal(size=C)).astype(np.float32), \
                     (1.0 + 0.1 * rng.normal(size=C)).astype(np.float32), (0.1 * rng.normal(size=C)).astype(np.float32)
    w2d = B.neck_conv3_weight(dev_bf16(w2))
    out = B.ssam_neck(dev_bf16(x.reshape(Bn, g * g, D)), dev_bf16(w1), dev_f32(g1), dev_f32(b1), w2d, dev_f32(g2), dev_f32(b2), g)
    got = to_np(out).reshape(Bn, g, g, C)
    for bi in range(Bn):
        ref = oracle.neck(x[bi], w1, g1, b1, w2, g2, b2)
        # four bf16 roundings (two contractions, two normalisations) on values of order one
        assert_close(got[bi], ref, f"neck image {bi}", stored=ref, updates=1, rms_updates=4)
