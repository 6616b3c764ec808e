#!/usr/bin/env python3
"""Benchmark of the structured-sparse SAM ViT encoder hot path on one MI355X.

A step = one pass of the whole hot path over one batch: token scores (Eq. 1),
keep-set selection, then every encoder block (LN1+gather, qkv, Stripe-Sort
attention, proj+scatter+residual, routed MLP) through ``ssam_encoder_forward``.
Inputs are seeded synthetic tensors with SAM ViT-H shapes, resident in HBM
before the timed region.  Prints ONE JSON line.

Extra legs (run after the timed region, reported inside the same JSON line):
  roofline      the dominant kernel (qkv contraction) timed with HIP events
                recorded around every launch of it INSIDE the timed region
  cpu_baseline  the CPU oracle on a bounded sample of the same workload
  dense         the same kernels at density 1.0 (the "dense GPU block")
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--model", default="vit_h", choices=["vit_b", "vit_l", "vit_h"])
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--density", type=float, default=0.4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain row copy of known size (identity ssam_permute over the input batch), "
                         "the reference kernel that scales the FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


class Hip:
    """The few HIP runtime calls the benchmark itself needs (events on the caller's stream)."""

    def __init__(self):
        self.lib = C.CDLL("libamdhip64.so")

    def event(self):
        ev = C.c_void_p()
        assert self.lib.hipEventCreate(C.byref(ev)) == 0
        return ev

    def elapsed_ms(self, a, b):
        ms = C.c_float()
        rc = self.lib.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b))
        assert rc == 0, rc
        return ms.value


def device_weights(torch, seed, shape, g, dev):
    """Random-init weights of the whole stack, drawn on the GPU from a seeded generator:
    N(0, 0.02) Linear weights/biases and rel-pos tables, LayerNorm gamma = 1 + N(0, 0.02)."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    d = shape.D // shape.heads

    def n(*s, dtype=torch.float32):
        return (torch.randn(*s, generator=gen, device=dev) * 0.02).to(dtype).contiguous()

    blocks = []
    for i in range(shape.depth):
        w = g if i in shape.global_blocks else shape.ws
        bf = torch.bfloat16
        blocks.append({
            "ln1_g": 1.0 + n(shape.D), "ln1_b": n(shape.D),
            "wqkv": n(3 * shape.D, shape.D, dtype=bf), "bqkv": n(3 * shape.D),
            "rel_h": n(2 * w - 1, d, dtype=bf), "rel_w": n(2 * w - 1, d, dtype=bf),
            "wproj": n(shape.D, shape.D, dtype=bf), "bproj": n(shape.D),
            "ln2_g": 1.0 + n(shape.D), "ln2_b": n(shape.D),
            "w1": n(shape.Dm, shape.D, dtype=bf), "b1": n(shape.Dm),
            "w2": n(shape.D, shape.Dm, dtype=bf), "b2": n(shape.D),
        })
    return blocks


def profile_traffic(model):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size); None when no summary exists."""
    path = os.path.join(ROOT, "profiles", f"gemm_qkv_{model}_b8_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def encoder_flops(shape, g, B, r, rho, K):
    """Algorithmic FLOPs of one step (per batch), on real tokens for the MLP and on padded
    window slots for qkv/proj of local blocks (the rows the kernels really multiply)."""
    import math
    D, Dm, h, d = shape.D, shape.Dm, shape.heads, shape.D // shape.heads
    n = g * g
    nws = -(-g // shape.ws)
    rows_local = nws * nws * shape.ws ** 2
    total = 0.0
    qkv_flops = []
    for i in range(shape.depth):
        glob = i in shape.global_blocks
        rows = n if glob else rows_local
        S = n if glob else shape.ws ** 2
        Bm = 128 if glob else 32
        T = -(-S // Bm)
        n_pre = min(T, int(math.floor(r * T + 1e-6)))
        tiles = n_pre * T + (T - n_pre)
        groups = 1 if glob else nws * nws
        qkv = 2.0 * rows * D * 3 * D
        proj = 2.0 * rows * D * D
        attn = 4.0 * Bm * Bm * d * tiles * h * groups
        mlp = 4.0 * K * D * Dm
        total += qkv + proj + attn + mlp
        qkv_flops.append(qkv * B)
    return total * B, qkv_flops


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2605_17633_amd import binding as B
    from paper_2605_17633_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    hip = Hip()
    shape = inputs.SHAPES[args.model]
    g, Bn, r, rho = 64, args.batch, args.density, args.density
    n = g * g
    K = B.ssam_keep_count(n, rho)

    rng = np.random.default_rng(args.seed)
    x_host = inputs.token_field(rng, Bn, g, shape.D)
    x0 = torch.from_numpy(x_host.reshape(Bn, n, shape.D)).to(dev).to(torch.bfloat16).contiguous()
    wts = device_weights(torch, args.seed + 1, shape, g, dev)
    structs = [B.block_weights_struct(w) for w in wts]
    flags = [i in shape.global_blocks for i in range(shape.depth)]
    plan = B.EncoderPlan(structs, flags)
    wtab = torch.from_numpy(B.ssam_build_window_table(g, shape.ws, 4)).to(dev)
    wsig = torch.from_numpy(B.ssam_build_perm(shape.ws, shape.ws, 4)[0]).to(dev)
    gtab = torch.from_numpy(B.ssam_build_perm(g, g, 4)[0]).to(dev)
    scores = torch.empty((Bn, n), dtype=torch.float32, device=dev)
    keep = torch.empty((Bn, K), dtype=torch.int32, device=dev)
    x = torch.empty_like(x0)

    def make_cfgs(rr, kk):
        return (B.make_cfg(Bn, g, shape.D, shape.heads, shape.Dm, shape.ws, 32, kk, rr),
                B.make_cfg(Bn, g, shape.D, shape.heads, shape.Dm, 0, 128, kk, rr))

    cfg_l, cfg_g = make_cfgs(r, K)
    cfg_ld, cfg_gd = make_cfgs(1.0, n)
    ws_bytes = max(B.ssam_encoder_workspace_bytes(cfg_l, cfg_g), B.ssam_encoder_workspace_bytes(cfg_ld, cfg_gd))
    ws_buf = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    keep_dense = torch.empty((Bn, n), dtype=torch.int32, device=dev)

    def step(cl, cg, kp, events=None):
        x.copy_(x0)                      # every step sees the same input (one 2*B*N*D-byte device copy)
        B.ssam_encoder_forward(x, structs, flags, cl, cg, wtab, wsig, gtab, gtab, scores, kp, ws_buf,
                               qkv_events=events, plan=plan)

    def timed(cl, cg, kp, steps, warmup, with_events):
        for _ in range(warmup):
            step(cl, cg, kp)
        evs = None
        if with_events:
            evs = [(C.c_void_p * (2 * shape.depth))(*[hip.event() for _ in range(2 * shape.depth)]) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            step(cl, cg, kp, evs[s] if evs else None)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt, evs

    if args.calibrate_copy:
        ident = torch.arange(n, dtype=torch.int32, device=dev)
        ycopy = torch.empty_like(x0)
        for _ in range(3):
            B.ssam_permute(x0, ident, ycopy)           # reads and writes B*N*D*2 bytes each
        torch.cuda.synchronize()

    dt, evs = timed(cfg_l, cfg_g, keep, args.steps, args.warmup, True)
    ms_per_step = dt / args.steps * 1e3
    images_per_s = Bn * args.steps / dt
    assert torch.isfinite(x.float()).all().item(), "non-finite encoder output"

    # ---- roofline of the dominant kernel: the qkv contraction, from the events recorded in the timed region
    flops_step, qkv_flops = encoder_flops(shape, g, Bn, r, rho, K)
    qkv_ms = [[hip.elapsed_ms(e[2 * i], e[2 * i + 1]) for i in range(shape.depth)] for e in evs]
    qkv_ms = np.array(qkv_ms)                                            # [steps, depth]
    avg_ms = float(qkv_ms.mean())
    avg_flops = float(np.mean(qkv_flops))
    achieved = avg_flops / (avg_ms * 1e-3) / 1e12
    rows_local = (-(-g // shape.ws)) ** 2 * shape.ws ** 2
    roofline = {
        "kernel": "gemm_bf16_nt_kernel (qkv contraction, bias epilogue)",
        "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": profile_traffic(shape.name),
        "avg_launch_ms": round(avg_ms, 4), "launches_per_step": shape.depth,
        "flops_per_launch": avg_flops,
        "shape": f"M={Bn * rows_local} (local) / {Bn * n} (global), N={3 * shape.D}, K={shape.D}",
        "qkv_share_of_step": round(float(qkv_ms.sum(axis=1).mean()) / ms_per_step, 4),
    }

    out = {
        "metric": "ViT-H encoder images/sec at density 0.4 (1 GPU); sparse-attn/MLP MFMA util %",
        "value": round(images_per_s, 3), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"SAM {shape.name} encoder blocks, batch {Bn}, 64x64 tokens, window 14, "
                               f"global blocks {list(shape.global_blocks)}, density {r} (attention and MLP)",
                   "global_batch": Bn, "tokens": n, "depth": shape.depth, "keep": K, "density": r},
        "step_tflops": round(flops_step / (ms_per_step * 1e-3) / 1e12, 2),
        "step_mfma_frac": round(flops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
    }

    # ---- dense GPU block: the same kernels at r = rho = 1
    if not args.no_dense:
        keep_dense.copy_(torch.arange(n, dtype=torch.int32, device=dev).expand(Bn, n))
        dsteps = max(2, args.steps // 2)
        ddt, _ = timed(cfg_ld, cfg_gd, keep_dense, dsteps, 1, False)
        d_ms = ddt / dsteps * 1e3
        out["dense"] = {"ms_per_step": round(d_ms, 3), "images_per_s": round(Bn * dsteps / ddt, 3),
                        "speedup_sparse_over_dense": round(d_ms / ms_per_step, 3)}

    # ---- CPU oracle on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        import oracle
        wl = {k: v.float().cpu().numpy() for k, v in wts[0].items()}
        xi = x_host[0]
        t0 = time.perf_counter()
        keep_o = oracle.select_tokens(oracle.score_tokens(xi), oracle.keep_count(n, rho))
        oracle.encoder_block(xi, oracle.BlockWeights(**wl), shape.heads, shape.ws, 4, 32, r, keep_o)
        t_local = time.perf_counter() - t0
        gi = shape.global_blocks[0]
        wg = {k: v.float().cpu().numpy() for k, v in wts[gi].items()}
        t0 = time.perf_counter()
        oracle.encoder_block(xi, oracle.BlockWeights(**wg), shape.heads, 0, 4, 128, r, keep_o)
        t_global = time.perf_counter() - t0
        n_glob = len(shape.global_blocks)
        t_image = t_local * (shape.depth - n_glob) + t_global * n_glob
        out["cpu_baseline"] = {
            "value": round(1.0 / t_image, 6), "unit": "images/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
            "kind": "oracle",
            "sample": f"one image: scores + keep-set + 1 windowed block ({t_local:.2f} s) and 1 global block "
                      f"({t_global:.2f} s) at full {shape.name} size; images/s extrapolated as "
                      f"1/({shape.depth - n_glob}*t_local + {n_glob}*t_global)",
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
