"""Parity at the benchmark's full size and launch configuration (SAM ViT-H, batch 8, 64x64 tokens,
window 14; densities 0.4, 0.3 and the dense block 1.0), through the same entry points bench.py times and
on the tables the library itself builds.  The oracle computes one image of the batch (the images are
independent); the other images are covered by properties."""
import numpy as np
import pytest
import torch

import oracle
from helpers import announce, assert_close, assert_keep_set, to_np
from stack_check import check_stack, library_tables
from paper_2605_17633_amd import binding as B
from paper_2605_17633_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"
SHAPE = inputs.VIT_H
G, BATCH = 64, 8


@pytest.mark.parametrize("R", [0.4, 0.3, 1.0])
@pytest.mark.parametrize("ws,Bm,img", [(14, 32, 5), (0, 128, 2)])
def test_vit_h_block_full_size(ws, Bm, img, R):
    """One windowed / one global block at B = 8, attention density = MLP keep ratio = R (K = 1638, 1228,
    4096): the oracle checks image `img` in full."""
    announce("ViT-H full-size block", ws, Bm, img, R)
    n = G * G
    rng = np.random.default_rng(100 + ws)
    w = ws if ws > 0 else G
    wt = inputs.block_weights(rng, SHAPE.D, SHAPE.heads, SHAPE.Dm, w)
    x = inputs.token_field(rng, BATCH, G, SHAPE.D)
    K = B.ssam_keep_count(n, R)
    assert K == oracle.keep_count(n, R)
    xd = torch.from_numpy(x.reshape(BATCH, n, SHAPE.D)).to(DEV).to(torch.bfloat16).contiguous()
    scores = B.ssam_score_tokens(xd.view(BATCH, G, G, SHAPE.D))
    keep = B.ssam_select_tokens(scores, K)
    sc_ref = oracle.score_tokens(x[img])
    keep_gpu = keep.cpu().numpy()
    assert_keep_set(keep_gpu[img], oracle.select_tokens(sc_ref, K), sc_ref, f"keep-set of image {img}")
    wtab, wsig, gtab = library_tables(G, SHAPE.ws)                # the library's own builders, checked against the oracle's
    table, sigma = (wtab, wsig) if ws > 0 else (gtab, gtab)
    wd = B.upload_block_weights(wt)
    cfg = B.make_cfg(BATCH, G, SHAPE.D, SHAPE.heads, SHAPE.Dm, ws, Bm, K, R)
    B.ssam_encoder_block(xd, B.block_weights_struct(wd), cfg, table, sigma, keep)
    torch.cuda.synchronize()
    got = to_np(xd[img]).reshape(G, G, SHAPE.D)
    mid, ref = oracle.encoder_block_halves(x[img], oracle.BlockWeights(**wt), SHAPE.heads, ws, 4, Bm, R, keep_gpu[img])
    assert_close(got - x[img], ref - x[img], f"ViT-H B=8 block ws={ws} r={R} image {img}", stored=(x[img], mid, ref), updates=2)
    # the same block with packed weights, LN1 folded into the qkv contraction and LN2 into fc1 (the form bench.py times)
    xf = torch.from_numpy(x.reshape(BATCH, n, SHAPE.D)).to(DEV).to(torch.bfloat16).contiguous()
    wf = B.pack_block_weights(wd, fold_ln1=True, fold_kv_bias=True, fold_ln2=True)
    B.ssam_encoder_block(xf, B.block_weights_struct(wf), cfg, table, sigma, keep)
    torch.cuda.synchronize()
    gotf = to_np(xf[img]).reshape(G, G, SHAPE.D)
    assert_close(gotf - x[img], ref - x[img], f"ViT-H B=8 block ws={ws} r={R} image {img}, folded", stored=(x[img], mid, ref), updates=2)
    del xf
    # every image was processed: finite and changed; rows outside an image's keep-set were written once (by the
    # attention half) and rows inside it twice
    allx = to_np(xd)
    assert np.isfinite(allx).all()
    assert all(np.abs(allx[b] - x[b].reshape(n, -1)).max() > 1e-3 for b in range(BATCH))


def test_vit_h_encoder_full_depth():
    """All 32 blocks at B = 8, density 0.4: ssam_encoder_forward against the loop of blocks bit for bit; every
    block of image 0 teacher-forced against the oracle at the 2e-2 bar, in the form bench.py times (packed
    weights; LN1, the key / value biases and LN2 folded) and with plain row-major weights; drift of the free-running
    stack reported apart.  (About a minute of oracle time on 16 cores.)"""
    rng = np.random.default_rng(7)
    x = inputs.token_field(rng, BATCH, G, SHAPE.D)
    wts = inputs.encoder_weights(8, SHAPE, G)
    check_stack("ViT-H B=8 encoder r=0.4", SHAPE, G, x, wts, 0.4, 0.4,
                [("packed, LN1, k/v biases and LN2 folded", dict(pack=True, fold_ln1=True, fold_kv_bias=True, fold_ln2=True)), ("row-major", dict())])
