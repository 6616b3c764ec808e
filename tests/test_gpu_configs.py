"""Parity at the full sizes of the other benchmark configurations: the ViT-B and ViT-L encoders at
batch 1 (full depth, densities 0.4 and 0.3) and the isolated ViT-H-dim kernels at batch 16 swept over
densities {0.2, 0.3, 0.4, 0.6, 1.0}.  Where the oracle cannot do the whole tensor in seconds it checks
sampled (image, head) problems / sampled kept rows in full."""
import numpy as np
import pytest
import torch

import oracle
from helpers import announce, assert_close, to_np
from stack_check import check_stack
from paper_2605_17633_amd import binding as B
from paper_2605_17633_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"
G = 64


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(DEV)


def dev_bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV).to(torch.bfloat16).contiguous()


@pytest.mark.parametrize("model,r", [("vit_b", 0.4), ("vit_l", 0.3), ("vit_l", 0.4)])
def test_encoder_full_depth_batch1(model, r):
    """Whole encoder stack of the named shape on one 64x64 image, packed weights with LN1 folded into the qkv
    contraction (the form bench.py times) and plain row-major weights: ssam_encoder_forward against the loop of
    blocks bit for bit, every block teacher-forced against the oracle at the 2e-2 bar, drift reported apart."""
    shape = inputs.SHAPES[model]
    x = inputs.token_field(np.random.default_rng(11), 1, G, shape.D)
    wts = inputs.encoder_weights(12, shape, G)
    check_stack(f"{model} encoder r={r}", shape, G, x, wts, r, r,
                [("packed, LN1, k/v biases and LN2 folded", dict(pack=True, fold_ln1=True, fold_kv_bias=True, fold_ln2=True)), ("row-major", dict())])


@pytest.mark.parametrize("r", [0.2, 0.3, 0.4, 0.6, 1.0])
def test_global_attention_batch16(r):
    """Isolated global Stripe-Sort attention, 16 images x 16 heads x 4096 tokens x 80: the launch the
    sweep times; three (image, head) problems checked in full by the oracle."""
    announce("global attention b16", r)
    Bn, h, d, w = 16, 16, 80, G
    S = w * w
    gen = torch.Generator(device=DEV)
    gen.manual_seed(100 + int(r * 10))
    qkv = (torch.randn((Bn, S, 3, h, d), generator=gen, device=DEV) * 0.7).to(torch.bfloat16)
    rel_h = (torch.randn((2 * w - 1, d), generator=gen, device=DEV) * 0.02).to(torch.bfloat16)
    rel_w = (torch.randn((2 * w - 1, d), generator=gen, device=DEV) * 0.02).to(torch.bfloat16)
    sig = oracle.grid_sigma(w, 4)[0]
    sig_lib = B.ssam_build_perm_device(w, w, 4)[0]                      # the GPU side runs on the library's own table
    assert np.array_equal(sig_lib.cpu().numpy(), sig)
    out = B.ssam_sparse_attention(qkv, rel_h, rel_w, sig_lib, w, 128, r)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    inv = np.empty(S, np.int64)
    inv[sig] = np.arange(S)
    for b, head in [(0, 0), (7, 5), (15, 15)]:
        scan = qkv[b, :, :, head, :].float().cpu().numpy()           # [S(scan), 3, d]
        spatial = scan[inv]                                         # row s = the token at spatial cell s
        ref = oracle.attention(spatial[None, :, 0], spatial[None, :, 1], spatial[None, :, 2],
                               to_np(rel_h), to_np(rel_w), w, 4, 128, r)[0]          # [S(spatial), d]
        got = to_np(out[b].reshape(S, h, d)[:, head, :])
        assert_close(got, ref[sig], f"global attention r={r} image {b} head {head}")


@pytest.mark.parametrize("rho", [0.2, 0.3, 0.4, 0.6, 1.0])
def test_routed_mlp_batch16(rho):
    """Isolated routed MLP 1280 -> 5120 -> 1280 over 16 x 4096 tokens with lognormal scores; the oracle
    recomputes a sample of kept rows of two images; every bypass row must be bit-identical."""
    announce("routed mlp b16", rho)
    Bn, n, D, Dm = 16, G * G, 1280, 5120
    rng = np.random.default_rng(200 + int(rho * 10))
    wt = inputs.block_weights(rng, D, 16, Dm, 14)
    for kname in ("w1", "w2"):
        wt[kname] = inputs.bf16_round(wt[kname] * 4)                # make the update comparable to x
    x = inputs.bf16_round(rng.normal(size=(Bn, n, D)).astype(np.float32))
    scores = inputs.lognormal_scores(rng, Bn, n)
    K = oracle.keep_count(n, rho)
    wd = B.upload_block_weights(wt)
    sd = torch.from_numpy(scores).to(DEV)
    keep = B.ssam_select_tokens(sd, K)
    keep_np = keep.cpu().numpy()
    for b in (0, 9):
        assert np.array_equal(keep_np[b], oracle.select_tokens(scores[b], K))      # integer work: bit-exact
    xd = dev_bf16(x)
    B.ssam_routed_mlp(xd, keep, wd["ln2_g"], wd["ln2_b"], 1e-6, wd["w1"], wd["b1"], wd["w2"], wd["b2"])
    torch.cuda.synchronize()
    got = to_np(xd)
    for b in (0, 9):
        rest = np.setdiff1d(np.arange(n), keep_np[b])
        assert np.array_equal(got[b][rest].view(np.uint32), x[b][rest].view(np.uint32))
        sample = np.sort(rng.choice(keep_np[b], size=96, replace=False)).astype(np.int32)
        ref = oracle.routed_mlp(x[b], sample, wt["ln2_g"], wt["ln2_b"], wt["w1"], wt["b1"], wt["w2"], wt["b2"])
        assert_close(got[b][sample] - x[b][sample], ref[sample] - x[b][sample], f"routed mlp rho={rho} image {b}",
                     stored=ref[sample])
    touched = np.abs(got - x).max(axis=2) > 0
    assert np.all(touched.sum(axis=1) <= K)
    # the form the encoder runs: packed weights, gather and LN2 folded into fc1
    Wf, colsum1, b1f = B.ssam_fold_ln_weight(wd["w1"], wd["b1"], wd["ln2_g"], wd["ln2_b"])
    xf = dev_bf16(x)
    B.ssam_routed_mlp_folded(xf, keep, 1e-6, B.ssam_pack_weight(Wf), colsum1, b1f, B.ssam_pack_weight(wd["w2"]), wd["b2"])
    torch.cuda.synchronize()
    gotf = to_np(xf)
    for b in (0, 9):
        rest = np.setdiff1d(np.arange(n), keep_np[b])
        assert np.array_equal(gotf[b][rest].view(np.uint32), x[b][rest].view(np.uint32))
        sample = np.sort(rng.choice(keep_np[b], size=96, replace=False)).astype(np.int32)
        ref = oracle.routed_mlp(x[b], sample, wt["ln2_g"], wt["ln2_b"], wt["w1"], wt["b1"], wt["w2"], wt["b2"])
        assert_close(gotf[b][sample] - x[b][sample], ref[sample] - x[b][sample], f"folded routed mlp rho={rho} image {b}",
                     stored=ref[sample])
