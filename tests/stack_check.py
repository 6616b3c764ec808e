"""Checks of a stack of encoder blocks on the GPU against the CPU oracle (helper of the GPU tests; holds
none of the method's arithmetic).

A stack is checked three ways, and the three are kept apart:

1. composition   -- ssam_encoder_forward (scores, keep-set, tables, every block) gives bit for bit what a
                    loop of ssam_encoder_block calls gives on the same keep-set and tables (GPU against
                    GPU: the same kernels in the same order), and its scores / keep-set / tables match
                    the oracle's (integer work bit-exact, keep-set up to fp32 ties at the threshold).
2. teacher-forced parity, per block, at the 2e-2 bar -- block i is given the ORACLE's block-i input
                    (rounded to bf16, which both sides then start from) and its update is compared
                    element by element with the oracle's update of the same input.  No error is
                    carried from block to block, so the bar does not depend on the depth.
3. drift report  -- the free-running GPU stack against the free-running fp64 oracle stack.  This mixes
                    the kernels' error with the 2*depth in-place bf16 roundings of the residual stream,
                    which the oracle does not have; it has a bar of its own (assert_drift) and is
                    printed as "[drift]".
"""
import numpy as np
import torch

import oracle
from helpers import announce, assert_close, assert_drift, assert_keep_set, to_np
from paper_2605_17633_amd import binding as B
from paper_2605_17633_amd import inputs

DEV = "cuda"


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(DEV)


def dev_bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV).to(torch.bfloat16).contiguous()


def library_tables(g, ws, G=4):
    """The position-only tables from the library's own builders (host and device forms), checked
    bit for bit against the oracle's.  Returns device tensors (window_table, sigma_window,
    global_table)."""
    wtab = B.ssam_build_window_table(g, ws, G)
    wsig = B.ssam_build_perm(ws, ws, G)[0]
    gtab, _ = B.ssam_build_perm_device(g, g, G)
    torch.cuda.synchronize()
    assert np.array_equal(wtab, oracle.window_table(g, ws, G))
    assert np.array_equal(wsig, oracle.grid_sigma(ws, G)[0])
    assert np.array_equal(gtab.cpu().numpy(), oracle.grid_sigma(g, G)[0])
    return dev_i32(wtab), dev_i32(wsig), gtab[: g * g].contiguous()


def check_stack(name, shape, g, x, wts, r, rho, variants, img=0, content_order=False, forced_blocks=None):
    """x [B,g,g,D] (bf16-representable fp32), wts: one numpy weight dict per block.
    variants: list of (label, dict(pack=, fold_ln1=, fold_kv_bias=, fold_ln2=)); the first one also runs the
    composition check and the drift report.  forced_blocks: indices of the blocks checked teacher-forced
    (default: all).  Returns {label: worst teacher-forced max-rel error}."""
    B_, n, depth = x.shape[0], g * g, len(wts)
    D = shape.D
    K = oracle.keep_count(n, rho)
    flags = [i in shape.global_blocks for i in range(depth)]
    cfg_l = B.make_cfg(B_, g, D, shape.heads, shape.Dm, shape.ws, 32, K, r, content_order=content_order)
    cfg_g = B.make_cfg(B_, g, D, shape.heads, shape.Dm, 0, 128, K, r, content_order=content_order)
    nW = (-(-g // shape.ws)) ** 2
    S_w = shape.ws * shape.ws
    if content_order:
        wtab = torch.empty((B_, nW * S_w), dtype=torch.int32, device=DEV)
        wsig = torch.empty((B_ * nW, S_w), dtype=torch.int32, device=DEV)
        gtab = torch.empty((B_, n), dtype=torch.int32, device=DEV)
        gsig = torch.empty((B_, n), dtype=torch.int32, device=DEV)
    else:
        wtab, wsig, gtab = library_tables(g, shape.ws)
        gsig = gtab
    scores = torch.empty((B_, n), dtype=torch.float32, device=DEV)
    keep = torch.empty((B_, K), dtype=torch.int32, device=DEV)
    ws_buf = torch.empty(B.ssam_encoder_workspace_bytes(cfg_l, cfg_g), dtype=torch.uint8, device=DEV)
    base = [B.upload_block_weights(w) for w in wts]                      # row-major device weights

    def structs_for(opts):
        if opts.get("pack") or opts.get("fold_ln1"):
            held = [B.pack_block_weights(w, fold_ln1=opts.get("fold_ln1", False), fold_kv_bias=opts.get("fold_kv_bias", False),
                                         fold_ln2=opts.get("fold_ln2", False)) for w in base]
        else:
            held = base
        return held, [B.block_weights_struct(w) for w in held]            # `held` keeps the tensors alive

    built = [(label,) + structs_for(opts) for label, opts in variants]

    # ---- 1. the whole stack through ssam_encoder_forward (first variant), free-running
    label0, _, structs0 = built[0]
    announce(name, "forward", label0)
    xd = dev_bf16(x.reshape(B_, n, D))
    B.ssam_encoder_forward(xd, structs0, flags, cfg_l, cfg_g, wtab, wsig, gtab, gsig, scores, keep, ws_buf)
    torch.cuda.synchronize()
    got_free = to_np(xd).reshape(x.shape)
    assert np.isfinite(got_free).all()
    keep_gpu = keep.cpu().numpy()
    sc_gpu = to_np(scores)
    for b in range(B_):
        sc_ref = oracle.score_tokens(x[b]).reshape(-1)
        np.testing.assert_allclose(sc_gpu[b], sc_ref, rtol=2e-5, atol=2e-5 * sc_ref.max())
        assert_keep_set(keep_gpu[b], oracle.select_tokens(sc_ref, K), sc_ref, f"{name}: keep-set of image {b}")
    if content_order:
        # the order is an integer decision on fp32 scores: both sides rank the SAME scores (the GPU's, which
        # match the oracle's to 2e-5 relative: checked above), so near-ties cannot flip it
        for b in range(B_):
            t_ref, s_ref = oracle.content_tables(sc_gpu[b].reshape(g, g), g, shape.ws, 4)
            assert np.array_equal(wtab[b].cpu().numpy(), t_ref)
            assert np.array_equal(wsig[b * nW:(b + 1) * nW].cpu().numpy(), s_ref)
            t_ref, s_ref = oracle.content_tables(sc_gpu[b].reshape(g, g), g, 0, 4)
            assert np.array_equal(gtab[b].cpu().numpy(), t_ref)
            assert np.array_equal(gsig[b:b + 1].cpu().numpy(), s_ref)
    order_scores = sc_gpu[img].reshape(g, g) if content_order else None

    def run_block(xt, structs, i):
        if flags[i]:
            B.ssam_encoder_block(xt, structs[i], cfg_g, gtab, gsig, keep)
        else:
            B.ssam_encoder_block(xt, structs[i], cfg_l, wtab, wsig, keep)

    # composition: the same stack as a loop of single-block calls, bit for bit
    xb = dev_bf16(x.reshape(B_, n, D))
    for i in range(depth):
        run_block(xb, structs0, i)
    torch.cuda.synchronize()
    assert torch.equal(xb, xd), f"{name}: ssam_encoder_forward differs from the loop over ssam_encoder_block"
    # determinism: a second forward on the same input gives the same bits
    xb.copy_(dev_bf16(x.reshape(B_, n, D)))
    B.ssam_encoder_forward(xb, structs0, flags, cfg_l, cfg_g, wtab, wsig, gtab, gsig, scores, keep, ws_buf)
    torch.cuda.synchronize()
    assert torch.equal(xb, xd), f"{name}: two runs differ"
    del xb

    # ---- 2. teacher-forced parity per block, and the oracle's own free-running stack for 3.
    ows = [oracle.BlockWeights(**w) for w in wts]

    def oracle_block(y, i, halves=False):
        f = oracle.encoder_block_halves if halves else oracle.encoder_block
        return f(y, ows[i], shape.heads, 0 if flags[i] else shape.ws, 4, 128 if flags[i] else 32, r,
                 keep_gpu[img], order_scores=order_scores)

    worst = {label: 0.0 for label, _, _ in built}
    xt = dev_bf16(x.reshape(B_, n, D))              # the other images of the batch keep whatever the last block left
    y = x[img]
    for i in range(depth):
        if forced_blocks is None or i in forced_blocks:
            y_in = inputs.bf16_round(y)              # the oracle's block-i input, representable on both sides
            mid, ref = oracle_block(y_in, i, halves=True)     # mid: the stream between the two halves
            for label, _, structs in built:
                xt[img].copy_(dev_bf16(y_in.reshape(n, D)))
                run_block(xt, structs, i)
                torch.cuda.synchronize()
                got = to_np(xt[img]).reshape(g, g, D)
                e = assert_close(got - y_in, ref - y_in, f"{name}: block {i} ({'global' if flags[i] else 'windowed'}) "
                                 f"teacher-forced, {label}", stored=(y_in, mid, ref), updates=2)
                worst[label] = max(worst[label], e)
        y = oracle_block(y, i)                       # the oracle's free-running stack (never rounded)
        print(f"[oracle] {name}: block {i} done", flush=True)

    # ---- 3. drift of the free-running stack (own bar)
    assert_drift(got_free[img], y, x[img], f"{name}: free-running stack, {label0}", depth)
    return worst
