"""The allocation-free entry point (ssam_score_tokens_static: its scratch is a device array inside the library)
against the entry point it is a variant of (ssam_score_tokens, caller workspace), through the C ABI: same
kernels, so the scores must agree bit for bit -- on two calls in a row, the second on a smaller input, whose
result must not see what the first call left in the shared array."""
import numpy as np
import pytest
import torch

from helpers import announce
from paper_2605_17633_amd import binding as B
from paper_2605_17633_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _tokens(seed, Bn, g, D):
    x = inputs.token_field(np.random.default_rng(seed), Bn, g, D)
    return torch.from_numpy(x).to(DEV).to(torch.bfloat16).contiguous()


def test_score_tokens_static_matches_workspace_form():
    announce("no-alloc score_tokens: 8x64x64x1280, then 3x28x28x768")
    for seed, (Bn, g, D) in enumerate([(8, 64, 1280), (3, 28, 768)]):
        x = _tokens(seed, Bn, g, D)
        want = B.ssam_score_tokens(x)                                   # caller-owned workspace (torch allocates it)
        got = torch.full((Bn, g * g), -1.0, dtype=torch.float32, device=DEV)
        B.ssam_score_tokens_static(x, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"call {seed}: static-scratch scores differ from the workspace form"
        assert bool((got >= 0).all())


def test_score_tokens_static_rejects_oversize_without_launching():
    announce("no-alloc score_tokens: size limit")
    lim = 1 << 18
    x = torch.zeros((1, 8, 8, 64), dtype=torch.bfloat16, device=DEV)
    scores = torch.zeros((1, 64), dtype=torch.float32, device=DEV)
    # the check is on the sizes alone and comes before anything is enqueued: the tensors can stay small
    rc = B.lib().ssam_score_tokens_static(B._bf(x, "x"), B._f32(scores, "scores"), 65, 64, 64, 64, B._stream())
    assert 65 * 64 * 64 > lim and rc == B.EWORKSPACE
    rc = B.lib().ssam_score_tokens_static(B._bf(x, "x"), B._f32(scores, "scores"), 1, 8, 8, 60, B._stream())
    assert rc == B.EINVAL
