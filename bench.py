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
  parts         the other entry points of the path timed one by one with HIP
                events (attention, routed MLP, LN+gather, scores, selection),
                each against the roofline that bounds it
  dense, density_0.3, content_order   the same kernels at density 1.0 (the "dense GPU block"), at 0.3,
                and at 0.4 with the content-aware order of Sec. 4.1 (per-image tables)
  pixels_to_embedding  the whole image encoder: patch embedding, the blocks, the neck
  other_models  SAM ViT-B and ViT-L shaped encoders at batch 1 (sparse and dense)
  kernels_batch16  isolated global attention and routed MLP at batch 16 over densities 0.2 .. 1.0
  hiera_l_routed_mlp  the routed MLP on the stage shapes of SAM2's Hiera-L encoder (shape-only)
  measured_peaks  what this machine sustains: MFMA-only loops (both bf16 MFMA shapes), a plain row copy (identity
                ssam_permute), and the vendor library's contraction on the qkv shape (torch.matmul, a yardstick
                only: it is not part of the product); every fraction is also given against these
  memory        bytes the calls require at density 1.0 / 0.4 / 0.3 (residual stream + workspace) and the part of the
                workspace a step actually touches
  cpu_baseline  the CPU oracle on a bounded sample of the same workload
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--model", default="vit_h", choices=["vit_b", "vit_l", "vit_h"])
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--density", type=float, default=0.4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the density 1.0 and 0.3 legs")
    ap.add_argument("--no-parts", action="store_true", help="skip the per-entry-point timings")
    ap.add_argument("--no-fold-ln1", action="store_true",
                    help="keep LN1 a pass of its own (by default it is folded into the qkv contraction)")
    ap.add_argument("--no-fold-ln2", action="store_true",
                    help="keep gather + LN2 a pass of its own (by default they are folded into fc1)")
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

    def record(self, ev, stream):
        assert self.lib.hipEventRecord(ev, C.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        ms = C.c_float()
        a, b = (e if isinstance(e, C.c_void_p) else C.c_void_p(e) for e in (a, b))
        rc = self.lib.hipEventElapsedTime(C.byref(ms), a, b)
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
    """Algorithmic FLOPs of one step (per batch): qkv, proj and the MLP on real tokens (the
    padding slots of the windows are not multiplied: their qkv rows are the bias), attention on
    the active tiles of every window / of the grid."""
    import math
    D, Dm, h, d = shape.D, shape.Dm, shape.heads, shape.D // shape.heads
    n = g * g
    nws = -(-g // shape.ws)
    rows_local = nws * nws * shape.ws ** 2
    total = 0.0
    qkv_flops = []
    for i in range(shape.depth):
        glob = i in shape.global_blocks
        rows = n
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


def measured_peaks(torch, hip, B, x0, shape, Bn, n):
    """The box's own peaks, each a sustained run of a few tens of milliseconds (the chip is power limited: the clock,
    and with it the rate, settles within a few milliseconds of sustained load)."""
    dev = x0.device
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = hip.event(), hip.event()

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        hip.record(e0, stream)
        for _ in range(reps):
            fn()
        hip.record(e1, stream)
        torch.cuda.synchronize()
        return hip.elapsed_ms(e0, e1) / reps

    out = {}
    sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    for shp, name in ((0, "mfma_bf16_32x32x16_tflops"), (1, "mfma_bf16_16x16x32_tflops")):
        # two waves per SIMD, ~60 ms a launch; two launches to let the clock settle, the third is timed
        for _ in range(2):
            flops = B.ssam_probe_mfma(shp, 512, 250000, sink)
        hip.record(e0, stream)
        B.ssam_probe_mfma(shp, 512, 250000, sink)
        hip.record(e1, stream)
        torch.cuda.synchronize()
        out[name] = round(flops / (hip.elapsed_ms(e0, e1) * 1e-3) / 1e12, 1)
    # a plain row copy larger than the 256 MB memory-side cache: 4 x the input batch in, as much out
    big = x0.repeat(4, 1, 1)
    ident = torch.arange(n, dtype=torch.int32, device=dev)
    ycopy = torch.empty_like(big)
    ms = timed(lambda: B.ssam_permute(big, ident, ycopy), 20)
    out["copy_gbs"] = round(2.0 * big.numel() * 2 / (ms * 1e-3) / 1e9, 1)
    out["copy_note"] = f"identity ssam_permute, {big.numel() * 2 >> 20} MiB read + as much written"
    del big, ycopy
    # the vendor library on the dominant contraction's shape: a yardstick beside the product, never inside it
    A = torch.randn((Bn * n, shape.D), device=dev).to(torch.bfloat16)
    W = (torch.randn((3 * shape.D, shape.D), device=dev) * 0.02).to(torch.bfloat16)
    Cm = torch.empty((Bn * n, 3 * shape.D), dtype=torch.bfloat16, device=dev)
    ms = timed(lambda: torch.matmul(A, W.t(), out=Cm), 100)
    out["vendor_library_qkv_tflops"] = round(2.0 * Bn * n * shape.D * 3 * shape.D / (ms * 1e-3) / 1e12, 1)
    out["vendor_library_note"] = "torch.matmul (hipBLASLt) on M x 3D x D, no bias, plain store; 100 back-to-back calls"
    del A, W, Cm
    # the four contraction shapes of a block, like for like: this library's kernel with packed weights and the plain
    # bias epilogue against the vendor library's plain product (no bias); each 100 back-to-back calls
    K_ = B.ssam_keep_count(n, 0.4)
    by_shape = {}
    ws_lin = torch.empty(B.ssam_linear_workspace_bytes(), dtype=torch.uint8, device=dev)
    for name, (M_, N_, Kd) in (("qkv", (Bn * n, 3 * shape.D, shape.D)), ("proj", (Bn * n, shape.D, shape.D)),
                               ("fc1", (Bn * K_, shape.Dm, shape.D)), ("fc2", (Bn * K_, shape.D, shape.Dm))):
        A = torch.randn((M_, Kd), device=dev).to(torch.bfloat16)
        W = (torch.randn((N_, Kd), device=dev) * 0.02).to(torch.bfloat16)
        Wp = B.ssam_pack_weight(W)
        bias = torch.zeros(N_, dtype=torch.float32, device=dev)
        Cm = torch.empty((M_, N_), dtype=torch.bfloat16, device=dev)
        fl = 2.0 * M_ * N_ * Kd
        ms_v = timed(lambda: torch.matmul(A, W.t(), out=Cm), 100)
        ms_o = timed(lambda: B.ssam_linear_ld(A, Wp, bias, Cm, workspace=ws_lin, w_packed=True), 100)
        by_shape[name] = {"shape": [M_, N_, Kd], "ours_tflops": round(fl / (ms_o * 1e-3) / 1e12, 1),
                          "vendor_library_tflops": round(fl / (ms_v * 1e-3) / 1e12, 1), "ratio": round(ms_v / ms_o, 3)}
        del A, W, Wp, Cm
    out["contractions_vs_vendor_library"] = by_shape
    out["mfma_tflops"] = max(out["mfma_bf16_32x32x16_tflops"], out["mfma_bf16_16x16x32_tflops"])
    return out


def memory_leg(torch, B, shape, g, Bn, n, step_fn, make_cfgs, ws_buf, weights_bytes):
    """Bytes the calls require per density (residual stream + the workspace ssam_encoder_workspace_bytes asks for;
    weights are the same for every density) and what a step at that density actually touches of the workspace:
    it is filled with a byte pattern, one step runs, and the bytes that changed are counted."""
    out = {"weights_bytes": int(weights_bytes), "residual_stream_bytes": int(Bn * n * shape.D * 2)}
    dens = {}
    for r in (1.0, 0.4, 0.3):
        K = B.ssam_keep_count(n, r)
        cl, cg = make_cfgs(r, K)
        need = int(B.ssam_encoder_workspace_bytes(cl, cg))
        keep = torch.empty((Bn, K), dtype=torch.int32, device=ws_buf.device)
        ws_buf.fill_(0xA5)
        step_fn(cl, cg, keep)
        torch.cuda.synchronize()
        changed = ws_buf[:need] != 0xA5
        touched = int(changed.sum().item())
        idx = torch.nonzero(changed)
        high = int(idx[-1].item()) + 1 if idx.numel() else 0
        del changed, idx
        dens[str(r)] = {"keep": K, "workspace_bytes_required": need, "workspace_bytes_touched": touched,
                        "workspace_high_water_offset": high,
                        "stream_plus_workspace_bytes": need + out["residual_stream_bytes"],
                        "stream_plus_touched_bytes": touched + out["residual_stream_bytes"]}
    out["by_density"] = dens
    for r in ("0.4", "0.3"):
        dens[r]["dense_over_sparse_required"] = round(dens["1.0"]["stream_plus_workspace_bytes"] / dens[r]["stream_plus_workspace_bytes"], 3)
        dens[r]["dense_over_sparse_touched"] = round(dens["1.0"]["stream_plus_touched_bytes"] / dens[r]["stream_plus_touched_bytes"], 3)
    out["note"] = ("activation memory of one step at batch %d: the in-place residual stream plus the caller's workspace (qkv, attention "
                   "output, gathered rows, hidden activations, K-split scratch, tables); a byte that happens to be rewritten with the "
                   "fill pattern is not counted as touched (1 in 256).  The paper's 2.8x memory figure (abstract, conclusion) was "
                   "measured on an NVIDIA A100 with its own implementation and is context only.") % Bn
    return out


def time_parts(torch, np, hip, B, shape, g, Bn, r, K, x0, wts, wtab, wsig, gtab, keep, scores, ws_buf, reps=10):
    """Each remaining entry point of the path on the benchmark's shapes, against its own roofline:
    algorithmic bytes (rows read + rows written, bf16) over HBM peak, or algorithmic flops over the
    bf16 MFMA peak.  Outputs are discarded; inputs are the benchmark's tensors."""
    import math
    dev = x0.device
    D, Dm, h, d = shape.D, shape.Dm, shape.heads, shape.D // shape.heads
    n = g * g
    nws = -(-g // shape.ws)
    nW, S = nws * nws, shape.ws ** 2
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = hip.event(), hip.event()

    def run(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        hip.record(e0, stream)
        for _ in range(reps):
            fn()
        hip.record(e1, stream)
        torch.cuda.synchronize()
        return hip.elapsed_ms(e0, e1) / reps

    def hbm(ms, nbytes):
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"us": round(ms * 1e3, 1), "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes": int(nbytes)}

    def mfma(ms, flops, extra=None):
        tf = flops / (ms * 1e-3) / 1e12
        o = {"us": round(ms * 1e3, 1), "bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
             "frac": round(tf / PEAK_BF16_TFLOPS, 4), "flops": float(flops)}
        if extra:
            o.update(extra)
        return o

    def tiles(Sx, Bm):
        T = -(-Sx // Bm)
        n_pre = min(T, int(math.floor(r * T + 1e-6)))
        return n_pre * T + (T - n_pre)

    parts = {}
    w0 = wts[0]
    wg_ = wts[shape.global_blocks[0]]
    bf = torch.bfloat16
    # LN1 + gather into window-major scan order, and LN2 + gather of the keep-set
    u = torch.empty((Bn, nW * S, D), dtype=bf, device=dev)
    ms = run(lambda: B.ssam_ln_gather(x0, wtab, 0, w0["ln1_g"], w0["ln1_b"], 1e-6, nW * S, y=u))
    parts["ln1_gather_windows"] = hbm(ms, 2.0 * Bn * (n + nW * S) * D)
    ms = run(lambda: B.ssam_ln_stats(x0, 1e-6))      # what is left of LN1 as a pass when it is folded into the qkv contraction
    parts["ln1_stats"] = hbm(ms, 2.0 * Bn * n * D)
    a2 = torch.empty((Bn, K, D), dtype=bf, device=dev)
    ms = run(lambda: B.ssam_ln_gather(x0, keep, K, w0["ln2_g"], w0["ln2_b"], 1e-6, K, y=a2))
    parts["ln2_gather_keep"] = hbm(ms, 2.0 * Bn * 2 * K * D)
    # windowed and global Stripe-Sort attention on a packed qkv tensor
    qkv = (torch.randn((Bn * nW, S, 3, h, d), device=dev) * 0.7).to(bf)
    o = torch.empty((Bn * nW, S, D), dtype=bf, device=dev)
    ms = run(lambda: B.ssam_sparse_attention(qkv, w0["rel_h"], w0["rel_w"], wsig, shape.ws, 32, r, out=o))
    win = hbm(ms, 2.0 * Bn * nW * S * 4 * D)
    fl = 4.0 * 32 * 32 * d * tiles(S, 32) * h * Bn * nW
    win["mfma_tflops"] = round(fl / (ms * 1e-3) / 1e12, 1)
    parts["attention_windows"] = win
    del qkv, o
    qkv = (torch.randn((Bn, n, 3, h, d), device=dev) * 0.7).to(bf)
    o = torch.empty((Bn, n, D), dtype=bf, device=dev)
    ms = run(lambda: B.ssam_sparse_attention(qkv, wg_["rel_h"], wg_["rel_w"], gtab, g, 128, r, out=o))
    parts["attention_global"] = mfma(ms, 4.0 * 128 * 128 * d * tiles(n, 128) * h * Bn,
                                     {"hbm_gbs": round(2.0 * Bn * n * 4 * D / (ms * 1e-3) / 1e9, 1)})
    del qkv, o
    # routed MLP (LN2 + gather, fc1 + GELU, fc2 + scatter-add), in place on a scratch copy
    xs = x0.clone()
    w1p, w2p = B.ssam_pack_weight(w0["w1"]), B.ssam_pack_weight(w0["w2"])      # the form the encoder uses
    ms = run(lambda: B.ssam_routed_mlp_packed(xs, keep, w0["ln2_g"], w0["ln2_b"], 1e-6, w1p, w0["b1"], w2p, w0["b2"],
                                              workspace=ws_buf))
    parts["routed_mlp_ln2_apart"] = mfma(ms, 4.0 * Bn * K * D * Dm)
    # the form the encoder runs: gather and LN2 folded into fc1 (statistics of the kept rows, then fc1 on x itself)
    Wf, colsum1, b1f = B.ssam_fold_ln_weight(w0["w1"], w0["b1"], w0["ln2_g"], w0["ln2_b"])
    w1fp = B.ssam_pack_weight(Wf)
    ms = run(lambda: B.ssam_routed_mlp_folded(xs, keep, 1e-6, w1fp, colsum1, b1f, w2p, w0["b2"], workspace=ws_buf))
    parts["routed_mlp"] = mfma(ms, 4.0 * Bn * K * D * Dm)
    del Wf, w1fp
    # scores (one read of x) and keep-set selection (latency bound: microseconds, once per image for all blocks)
    ms = run(lambda: B.ssam_score_tokens(x0.view(Bn, g, g, D), scores=scores, workspace=ws_buf))
    parts["score_tokens"] = hbm(ms, 2.0 * Bn * n * D)
    ms = run(lambda: B.ssam_select_tokens(scores, K, keep_idx=keep))
    parts["select_tokens"] = {"us": round(ms * 1e3, 1), "bound": "latency", "once_per": "image, shared by all blocks"}
    return parts


def sweep_leg(torch, hip, B, inputs, seed, reps=5):
    """The isolated ViT-H-dim kernels at batch 16 swept over densities (global Stripe-Sort attention over
    4096 tokens x 16 heads x 80; routed MLP 1280 -> 5120 -> 1280 with lognormal scores), each against the
    bf16 MFMA peak on its algorithmic FLOPs."""
    import math
    dev = "cuda:0"
    Bn, g, h, d, D, Dm = 16, 64, 16, 80, 1280, 5120
    n = g * g
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    bf = torch.bfloat16
    qkv = (torch.randn((Bn, n, 3, h, d), generator=gen, device=dev) * 0.7).to(bf)
    rel_h = (torch.randn((2 * g - 1, d), generator=gen, device=dev) * 0.02).to(bf)
    rel_w = (torch.randn((2 * g - 1, d), generator=gen, device=dev) * 0.02).to(bf)
    sig = torch.from_numpy(B.ssam_build_perm(g, g, 4)[0]).to(dev)
    o = torch.empty((Bn, n, D), dtype=bf, device=dev)
    x = (torch.randn((Bn, n, D), generator=gen, device=dev)).to(bf)
    scores = torch.exp(torch.randn((Bn, n), generator=gen, device=dev))
    w = {"ln2_g": 1.0 + torch.randn(D, generator=gen, device=dev) * 0.02, "ln2_b": torch.randn(D, generator=gen, device=dev) * 0.02,
         "w1": (torch.randn((Dm, D), generator=gen, device=dev) * 0.02).to(bf), "b1": torch.randn(Dm, generator=gen, device=dev) * 0.02,
         "w2": (torch.randn((D, Dm), generator=gen, device=dev) * 0.02).to(bf), "b2": torch.randn(D, generator=gen, device=dev) * 0.02}
    ws_buf = torch.empty(B.ssam_routed_mlp_workspace_bytes(Bn, n, D, Dm), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = hip.event(), hip.event()

    def run(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        hip.record(e0, stream)
        for _ in range(reps):
            fn()
        hip.record(e1, stream)
        torch.cuda.synchronize()
        return hip.elapsed_ms(e0, e1) / reps

    out = {"batch": Bn}
    w1p, w2p = B.ssam_pack_weight(w["w1"]), B.ssam_pack_weight(w["w2"])
    for r in (0.2, 0.3, 0.4, 0.6, 1.0):
        T = n // 128
        n_pre = min(T, int(math.floor(r * T + 1e-6)))
        tiles = n_pre * T + (T - n_pre)
        ms_a = run(lambda: B.ssam_sparse_attention(qkv, rel_h, rel_w, sig, g, 128, r, out=o))
        fl_a = 4.0 * 128 * 128 * d * tiles * h * Bn
        K = B.ssam_keep_count(n, r)
        keep = B.ssam_select_tokens(scores, K)
        ms_m = run(lambda: B.ssam_routed_mlp_packed(x, keep, w["ln2_g"], w["ln2_b"], 1e-6, w1p, w["b1"], w2p, w["b2"], workspace=ws_buf))
        fl_m = 4.0 * Bn * K * D * Dm
        out[f"density_{r}"] = {
            "attention_global": {"us": round(ms_a * 1e3, 1), "tflops": round(fl_a / ms_a / 1e9, 1),
                                 "frac": round(fl_a / ms_a / 1e9 / PEAK_BF16_TFLOPS, 4), "active_tiles": tiles},
            "routed_mlp": {"us": round(ms_m * 1e3, 1), "tflops": round(fl_m / ms_m / 1e9, 1),
                           "frac": round(fl_m / ms_m / 1e9 / PEAK_BF16_TFLOPS, 4), "keep": K}}
    return out


def hiera_leg(torch, hip, B, seed, Bn=4, reps=5):
    """Residual-Consistency MLP on a second backbone (Sec. 5, SAM2 with the Hiera-L encoder): a shape-only leg.
    Stage widths / token grids / block counts of Hiera-L on a 1024x1024 input (144, 288, 576, 1152 channels on
    256^2, 128^2, 64^2, 32^2 tokens; 2, 6, 36, 4 blocks; MLP ratio 4) are the public architecture, not the paper's;
    weights and tokens are random.  Per keep ratio r: the routed-MLP time of one image summed over all 48 blocks."""
    dev = "cuda:0"
    stages = [(256, 144, 2), (128, 288, 6), (64, 576, 36), (32, 1152, 4)]
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    bf = torch.bfloat16
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = hip.event(), hip.event()
    out = {"batch": Bn}
    per_r = {}
    for (g, D, blocks) in stages:
        n, Dm = g * g, 4 * D
        x = torch.randn((Bn, n, D), generator=gen, device=dev).to(bf)
        scores = torch.exp(torch.randn((Bn, n), generator=gen, device=dev))
        w = {"ln2_g": 1.0 + torch.randn(D, generator=gen, device=dev) * 0.02, "ln2_b": torch.randn(D, generator=gen, device=dev) * 0.02,
             "w1": (torch.randn((Dm, D), generator=gen, device=dev) * 0.02).to(bf), "b1": torch.randn(Dm, generator=gen, device=dev) * 0.02,
             "w2": (torch.randn((D, Dm), generator=gen, device=dev) * 0.02).to(bf), "b2": torch.randn(D, generator=gen, device=dev) * 0.02}
        ws_buf = torch.empty(B.ssam_routed_mlp_workspace_bytes(Bn, n, D, Dm), dtype=torch.uint8, device=dev)
        wp1, wp2 = (B.ssam_pack_weight(w["w1"]), B.ssam_pack_weight(w["w2"])) if D % 128 == 0 else (None, None)
        for r in (1.0, 0.7, 0.5, 0.3):
            K = B.ssam_keep_count(n, r)
            keep = B.ssam_select_tokens(scores, K)
            if D % 128 == 0:          # packed weights need widths that are multiples of 128 (only the last stage)
                fn = lambda: B.ssam_routed_mlp_packed(x, keep, w["ln2_g"], w["ln2_b"], 1e-6, wp1, w["b1"], wp2, w["b2"], workspace=ws_buf)
            else:
                fn = lambda: B.ssam_routed_mlp(x, keep, w["ln2_g"], w["ln2_b"], 1e-6, w["w1"], w["b1"], w["w2"], w["b2"], workspace=ws_buf)
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            hip.record(e0, stream)
            for _ in range(reps):
                fn()
            hip.record(e1, stream)
            torch.cuda.synchronize()
            ms = hip.elapsed_ms(e0, e1) / reps
            d = per_r.setdefault(r, {"ms_per_image": 0.0, "stages_us": []})
            d["ms_per_image"] += ms * blocks / Bn
            d["stages_us"].append(round(ms * 1e3, 1))
        del x, scores, ws_buf
    for r, d in per_r.items():
        out["dense" if r == 1.0 else f"keep_{r}"] = {"mlp_ms_per_image": round(d["ms_per_image"], 3), "stage_call_us": d["stages_us"],
                                                     "speedup_over_dense": round(per_r[1.0]["ms_per_image"] / d["ms_per_image"], 3)}
    return out


def model_leg(torch, B, inputs, name, Bn, densities, steps, seed):
    """The other encoder shapes the workload family names (SAM ViT-B / ViT-L, batch 1): images/s of the same
    path at each density and at density 1.0, packed weights, position-only order."""
    dev = "cuda:0"
    shape = inputs.SHAPES[name]
    g = 64
    n = g * g
    wts = [B.pack_block_weights(w, fold_ln1=True, fold_kv_bias=True, fold_ln2=True) for w in device_weights(torch, seed, shape, g, dev)]
    structs = [B.block_weights_struct(w) for w in wts]
    flags = [i in shape.global_blocks for i in range(shape.depth)]
    plan = B.EncoderPlan(structs, flags)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed + 7)
    x0 = torch.randn((Bn, n, shape.D), generator=gen, device=dev).to(torch.bfloat16)
    x = torch.empty_like(x0)
    wtab = torch.from_numpy(B.ssam_build_window_table(g, shape.ws, 4)).to(dev)
    wsig = torch.from_numpy(B.ssam_build_perm(shape.ws, shape.ws, 4)[0]).to(dev)
    gtab = torch.from_numpy(B.ssam_build_perm(g, g, 4)[0]).to(dev)
    scores = torch.empty((Bn, n), dtype=torch.float32, device=dev)
    out = {"batch": Bn, "depth": shape.depth, "width": shape.D}
    for r in list(densities) + [1.0]:
        K = B.ssam_keep_count(n, r)
        cl = B.make_cfg(Bn, g, shape.D, shape.heads, shape.Dm, shape.ws, 32, K, r)
        cg = B.make_cfg(Bn, g, shape.D, shape.heads, shape.Dm, 0, 128, K, r)
        keep = torch.empty((Bn, K), dtype=torch.int32, device=dev)
        ws_buf = torch.empty(B.ssam_encoder_workspace_bytes(cl, cg), dtype=torch.uint8, device=dev)

        def step():
            x.copy_(x0)
            B.ssam_encoder_forward(x, structs, flags, cl, cg, wtab, wsig, gtab, gtab, scores, keep, ws_buf, plan=plan)

        for _ in range(3):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        leg = {"ms_per_step": round(dt / steps * 1e3, 3), "images_per_s": round(Bn * steps / dt, 2)}
        # at batch 1 the ~10 launches per block are not covered by their own run time: the same step captured
        # once into a HIP graph (the library only enqueues on the caller's stream, so it can be captured as is)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        gdt = time.perf_counter() - t0
        leg["hip_graph"] = {"ms_per_step": round(gdt / steps * 1e3, 3), "images_per_s": round(Bn * steps / gdt, 2)}
        out["dense" if r == 1.0 else f"density_{r}"] = leg
    dense_flops = encoder_flops(shape, g, Bn, 1.0, 1.0, n)[0]
    for r in densities:
        out[f"density_{r}"]["speedup_over_dense"] = round(out["dense"]["ms_per_step"] / out[f"density_{r}"]["ms_per_step"], 3)
        # what the speed-up would be if time were proportional to the algorithmic FLOPs
        out[f"density_{r}"]["flop_ratio_dense_over_sparse"] = round(
            dense_flops / encoder_flops(shape, g, Bn, r, r, B.ssam_keep_count(n, r))[0], 3)
    return out


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
    # the four Linear weights of every block go into MFMA fragment order once, at load time (ssam_pack_weight)
    wts_packed = [B.pack_block_weights(w, fold_ln1=not args.no_fold_ln1, fold_kv_bias=not args.no_fold_ln1,
                                       fold_ln2=not args.no_fold_ln2) for w in wts]
    structs = [B.block_weights_struct(w) for w in wts_packed]
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

    # A recorded event costs the stream about 6 us (measured: 64 of them took 1.1 % off the step), so the qkv
    # contraction is timed in every fourth windowed block and in one global block, not in all 32.
    win_blocks = [i for i in range(shape.depth) if i not in shape.global_blocks]
    timed_win = win_blocks[1::4]
    timed_glob = list(shape.global_blocks)[:1]
    timed_blocks = set(timed_win + timed_glob)

    def timed(cl, cg, kp, steps, warmup, with_events):
        for _ in range(warmup):
            step(cl, cg, kp)
        evs = None
        if with_events:      # events only around the sampled blocks' contractions (NULL entries are skipped)
            evs = [(C.c_void_p * (2 * shape.depth))(*[hip.event() if i // 2 in timed_blocks else None
                                                     for i in range(2 * shape.depth)]) for _ in range(steps)]
        marks = [hip.event() for _ in range(steps + 1)]
        stream = torch.cuda.current_stream().cuda_stream
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        hip.record(marks[0], stream)
        for s in range(steps):
            step(cl, cg, kp, evs[s] if evs else None)
            hip.record(marks[s + 1], stream)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        per_step = [hip.elapsed_ms(marks[s], marks[s + 1]) for s in range(steps)]
        return dt, evs, per_step

    if args.calibrate_copy:
        ident = torch.arange(n, dtype=torch.int32, device=dev)
        ycopy = torch.empty_like(x0)
        for _ in range(3):
            B.ssam_permute(x0, ident, ycopy)           # reads and writes B*N*D*2 bytes each
        torch.cuda.synchronize()

    dt, evs, per_step = timed(cfg_l, cfg_g, keep, args.steps, args.warmup, True)
    ms_per_step = dt / args.steps * 1e3
    images_per_s = Bn * args.steps / dt
    assert torch.isfinite(x.float()).all().item(), "non-finite encoder output"

    # ---- roofline of the dominant kernel: the qkv contraction, from the events recorded in the timed region
    flops_step, qkv_flops = encoder_flops(shape, g, Bn, r, rho, K)
    t_win = np.array([[hip.elapsed_ms(e[2 * i], e[2 * i + 1]) for i in timed_win] for e in evs])      # [steps, sampled]
    t_glob = np.array([[hip.elapsed_ms(e[2 * i], e[2 * i + 1]) for i in timed_glob] for e in evs])
    n_win, n_glob = len(win_blocks), len(shape.global_blocks)
    # average launch duration over the step's launches: windowed and global blocks weighted by their counts
    avg_ms = float((n_win * t_win.mean() + n_glob * (t_glob.mean() if t_glob.size else 0.0)) / (n_win + n_glob))
    avg_flops = float(np.mean(qkv_flops))
    achieved = avg_flops / (avg_ms * 1e-3) / 1e12
    rows_local = (-(-g // shape.ws)) ** 2 * shape.ws ** 2
    roofline = {
        "kernel": ("gemm_bf16_nt_kernel (qkv contraction, bias epilogue)" if args.no_fold_ln1 else
                   "gemm_bf16_nt_lnf_kernel (qkv contraction with LN1 folded in, mapped store)"),
        "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": profile_traffic(shape.name),
        "traffic_source": f"profiles/gemm_qkv_{shape.name}_b8_hbm_traffic.txt (two rocprofv3 --pmc runs of this kernel, scaled by a copy)",
        "avg_launch_ms": round(avg_ms, 4), "launches_per_step": shape.depth,
        "launches_timed_per_step": len(timed_blocks),
        "timed_blocks": {"windowed": timed_win, "global": timed_glob,
                         "avg_ms_windowed": round(float(t_win.mean()), 4),
                         "avg_ms_global": round(float(t_glob.mean()), 4) if t_glob.size else None},
        "flops_per_launch": avg_flops,
        "shape": f"M={Bn * n} (real tokens; the {Bn * (rows_local - n)} padding slots of the windows are filled with the bias), "
                 f"N={3 * shape.D}, K={shape.D}",
        "qkv_share_of_step": round(avg_ms * shape.depth / ms_per_step, 4),
    }

    out = {
        "metric": "ViT-H encoder images/sec at density 0.4 (1 GPU); sparse-attn/MLP MFMA util %",
        "value": round(images_per_s, 3), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "ms_per_step_median": round(float(np.median(per_step)), 3),
        "ms_per_step_min": round(float(np.min(per_step)), 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"SAM {shape.name} encoder blocks, batch {Bn}, 64x64 tokens, window 14, "
                               f"global blocks {list(shape.global_blocks)}, density {r} (attention and MLP)",
                   "global_batch": Bn, "tokens": n, "depth": shape.depth, "keep": K, "density": r},
        "step_tflops": round(flops_step / (ms_per_step * 1e-3) / 1e12, 2),
        "step_mfma_frac": round(flops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
    }

    # ---- the other entry points, one by one (HIP events around `reps` back-to-back calls)
    if not args.no_parts:
        out["parts"] = time_parts(torch, np, hip, B, shape, g, Bn, r, K, x0, wts, wtab, wsig, gtab, keep, scores, ws_buf)
        # ---- what this machine sustains; every fraction also against that
        mp = measured_peaks(torch, hip, B, x0, shape, Bn, n)
        out["measured_peaks"] = mp
        roofline["peak_measured"] = mp["mfma_tflops"]
        roofline["frac_measured"] = round(roofline["achieved"] / mp["mfma_tflops"], 4)
        roofline["vs_vendor_library"] = round(roofline["achieved"] / mp["vendor_library_qkv_tflops"], 3)
        out["step_mfma_frac_measured"] = round(out["step_tflops"] / mp["mfma_tflops"], 4)
        for pv in out["parts"].values():
            if pv.get("bound") == "mfma":
                pv["frac_measured"] = round(pv["achieved"] / mp["mfma_tflops"], 4)
            elif pv.get("bound") == "hbm":
                pv["frac_measured"] = round(pv["achieved"] / mp["copy_gbs"], 4)

    # ---- dense GPU block (the same kernels at r = rho = 1) and density 0.3
    if not args.no_dense:
        keep_dense.copy_(torch.arange(n, dtype=torch.int32, device=dev).expand(Bn, n))
        dsteps = max(2, args.steps // 2)
        ddt, _, _ = timed(cfg_ld, cfg_gd, keep_dense, dsteps, 1, False)
        d_ms = ddt / dsteps * 1e3
        out["dense"] = {"ms_per_step": round(d_ms, 3), "images_per_s": round(Bn * dsteps / ddt, 3),
                        "speedup_sparse_over_dense": round(d_ms / ms_per_step, 3),
                        # what the speed-up would be if time were proportional to the algorithmic FLOPs
                        "flop_ratio_dense_over_sparse": round(encoder_flops(shape, g, Bn, 1.0, 1.0, n)[0] /
                                                              encoder_flops(shape, g, Bn, r, r, K)[0], 3)}
        # content-aware Stripe-Sort order (Sec. 4.1): per-image tables built from the scores inside the step
        nW_, S_ = (-(-g // shape.ws)) ** 2, shape.ws ** 2
        cl_c = B.make_cfg(Bn, g, shape.D, shape.heads, shape.Dm, shape.ws, 32, K, r, content_order=True)
        cg_c = B.make_cfg(Bn, g, shape.D, shape.heads, shape.Dm, 0, 128, K, r, content_order=True)
        ctab = [torch.empty((Bn, nW_ * S_), dtype=torch.int32, device=dev), torch.empty((Bn * nW_, S_), dtype=torch.int32, device=dev),
                torch.empty((Bn, n), dtype=torch.int32, device=dev), torch.empty((Bn, n), dtype=torch.int32, device=dev)]

        def step_content():
            x.copy_(x0)
            B.ssam_encoder_forward(x, structs, flags, cl_c, cg_c, ctab[0], ctab[1], ctab[2], ctab[3], scores, keep, ws_buf, plan=plan)

        for _ in range(2):
            step_content()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(dsteps):
            step_content()
        torch.cuda.synchronize()
        cdt = time.perf_counter() - t0
        out["content_order"] = {"ms_per_step": round(cdt / dsteps * 1e3, 3), "images_per_s": round(Bn * dsteps / cdt, 3),
                                "note": "tokens of every window / image ranked by the Sobel score, tables rebuilt every step"}
        if abs(r - 0.3) > 1e-9:
            K3 = B.ssam_keep_count(n, 0.3)
            cfg_l3, cfg_g3 = make_cfgs(0.3, K3)
            keep3 = torch.empty((Bn, K3), dtype=torch.int32, device=dev)
            tdt, _, _ = timed(cfg_l3, cfg_g3, keep3, dsteps, 1, False)
            out["density_0.3"] = {"ms_per_step": round(tdt / dsteps * 1e3, 3), "images_per_s": round(Bn * dsteps / tdt, 3),
                                  "keep": K3, "speedup_over_dense": round(d_ms / (tdt / dsteps * 1e3), 3),
                                  "flop_ratio_dense_over_sparse": round(encoder_flops(shape, g, Bn, 1.0, 1.0, n)[0] /
                                                                        encoder_flops(shape, g, Bn, 0.3, 0.3, K3)[0], 3)}

    # ---- activation memory per density
    if not args.no_dense:
        wbytes = sum(t.numel() * t.element_size() for w in wts_packed for t in w.values() if hasattr(t, "numel"))
        out["memory"] = memory_leg(torch, B, shape, g, Bn, n, lambda cl, cg, kp: step(cl, cg, kp), make_cfgs, ws_buf, wbytes)

    # ---- pixels in -> embedding out: patch embedding + position embedding, the blocks, the neck
    if not args.no_dense:
        gen = torch.Generator(device=dev)
        gen.manual_seed(args.seed + 400)
        bf = torch.bfloat16
        P_, C_ = 16, 256
        img = torch.randn((Bn, 3, g * P_, g * P_), generator=gen, device=dev).to(bf)
        w_pe = (torch.randn((shape.D, 3 * P_ * P_), generator=gen, device=dev) * 0.02).to(bf)
        b_pe = torch.randn(shape.D, generator=gen, device=dev) * 0.02
        pos = (torch.randn((n, shape.D), generator=gen, device=dev) * 0.02).to(bf)
        w_n1 = (torch.randn((C_, shape.D), generator=gen, device=dev) * 0.02).to(bf)
        w_n2 = (torch.randn((C_, 9 * C_), generator=gen, device=dev) * 0.02).to(bf)
        ln_g, ln_b = 1.0 + torch.randn(C_, generator=gen, device=dev) * 0.02, torch.randn(C_, generator=gen, device=dev) * 0.02
        emb = torch.empty((Bn, n, C_), dtype=bf, device=dev)
        ws_pe = torch.empty(B.ssam_patch_embed_workspace_bytes(Bn, g * P_, g * P_, P_), dtype=torch.uint8, device=dev)
        ws_nk = torch.empty(B.ssam_neck_workspace_bytes(Bn, g, shape.D, C_), dtype=torch.uint8, device=dev)

        def step_full():
            B.ssam_patch_embed(img, w_pe, b_pe, pos, P_, x=x, workspace=ws_pe)
            B.ssam_encoder_forward(x, structs, flags, cfg_l, cfg_g, wtab, wsig, gtab, gtab, scores, keep, ws_buf, plan=plan)
            B.ssam_neck(x, w_n1, ln_g, ln_b, w_n2, ln_g, ln_b, g, out=emb, workspace=ws_nk)

        for _ in range(2):
            step_full()
        torch.cuda.synchronize()
        fsteps = max(2, args.steps // 2)
        t0 = time.perf_counter()
        for _ in range(fsteps):
            step_full()
        torch.cuda.synchronize()
        fdt = time.perf_counter() - t0
        out["pixels_to_embedding"] = {"ms_per_step": round(fdt / fsteps * 1e3, 3), "images_per_s": round(Bn * fsteps / fdt, 3),
                                      "note": "1024x1024 bf16 images: patch embedding + position embedding, the 32 blocks at "
                                              f"density {r}, neck to {C_} channels"}

    # ---- the smaller encoder shapes of the workload family, batch 1
    if not args.no_dense and not args.no_parts and shape.name == "vit_h":
        out["other_models"] = {"vit_b": model_leg(torch, B, inputs, "vit_b", 1, [0.4], 10, args.seed + 100),
                               "vit_l": model_leg(torch, B, inputs, "vit_l", 1, [0.3, 0.4], 10, args.seed + 200)}
        out["kernels_batch16"] = sweep_leg(torch, hip, B, inputs, args.seed + 300)
        out["hiera_l_routed_mlp"] = hiera_leg(torch, hip, B, args.seed + 600)

    # ---- CPU oracle on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        import oracle
        xi = x_host[0]
        n_glob = len(shape.global_blocks)
        loc = [i for i in range(shape.depth) if i not in shape.global_blocks][:10]
        glo = list(shape.global_blocks)[:3]
        t0 = time.perf_counter()
        keep_o = oracle.select_tokens(oracle.score_tokens(xi), oracle.keep_count(n, rho))
        t_sel = time.perf_counter() - t0
        y = xi
        t0 = time.perf_counter()
        for i in loc:
            wl = {k: v.float().cpu().numpy() for k, v in wts[i].items()}
            y = oracle.encoder_block(y, oracle.BlockWeights(**wl), shape.heads, shape.ws, 4, 32, r, keep_o)
        t_local = (time.perf_counter() - t0) / len(loc)
        t0 = time.perf_counter()
        for i in glo:
            wg = {k: v.float().cpu().numpy() for k, v in wts[i].items()}
            y = oracle.encoder_block(y, oracle.BlockWeights(**wg), shape.heads, 0, 4, 128, r, keep_o)
        t_global = (time.perf_counter() - t0) / len(glo)
        t_image = t_sel + t_local * (shape.depth - n_glob) + t_global * n_glob
        out["cpu_baseline"] = {
            "value": round(1.0 / t_image, 6), "unit": "images/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
            "kind": "oracle",
            "sample": f"one image at full {shape.name} size: scores + keep-set ({t_sel:.2f} s), {len(loc)} windowed blocks "
                      f"({t_local:.2f} s each) and {len(glo)} global blocks ({t_global:.2f} s each), host-to-numpy weight "
                      f"conversion included; images/s extrapolated as 1/(t_sel + {shape.depth - n_glob}*t_local + {n_glob}*t_global)",
        }
        # the whole ViT-B encoder on one image (the smallest full configuration), timed in full
        if "other_models" in out:
            sb = inputs.SHAPES["vit_b"]
            rng_b = np.random.default_rng(args.seed + 500)
            xb = inputs.token_field(rng_b, 1, g, sb.D)[0]
            wb = inputs.encoder_weights(args.seed + 501, sb, g)
            t0 = time.perf_counter()
            oracle.encoder(xb, [oracle.BlockWeights(**w) for w in wb], sb.heads, sb.ws, sb.global_blocks, 4, r, rho)
            tb = time.perf_counter() - t0
            out["other_models"]["vit_b"]["cpu_oracle"] = {"images_per_s": round(1.0 / tb, 4), "seconds_per_image": round(tb, 2),
                                                          "cores": out["cpu_baseline"]["cores"],
                                                          "sample": "the whole encoder on one image, not extrapolated"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
