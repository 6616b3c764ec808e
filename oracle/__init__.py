"""CPU oracle for the structured-sparse SAM encoder block -- TEST INFRASTRUCTURE.

Thin ctypes/numpy marshalling over ``libssam_oracle.so`` (built from
``ssam_oracle.c`` in this folder with gcc).  Nothing here is a product path and
nothing here imports the HIP library or its binding.  Only tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package.

Every function cites the passage of the paper (arXiv 2605.17633) it follows in
the C source; this file only moves arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libssam_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle's C source with gcc (``make`` in this folder)."""
    src = os.path.join(_HERE, "ssam_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.run(["make", "-B", "-C", _HERE], check=True, capture_output=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name} failed with code {rc}")


def morton_order(gh: int, gw: int) -> np.ndarray:
    pi = np.empty(gh * gw, np.int32)
    _check(lib().oracle_morton_order(C.c_int(gh), C.c_int(gw), _p(pi)), "oracle_morton_order")
    return pi


def stripe_sort(pi: np.ndarray, G: int):
    pi = _i32(pi)
    sigma = np.empty_like(pi)
    sinv = np.empty_like(pi)
    _check(lib().oracle_stripe_sort(_p(pi), C.c_int(pi.size), C.c_int(G), _p(sigma), _p(sinv)),
           "oracle_stripe_sort")
    return sigma, sinv


def grid_sigma(w: int, G: int):
    return stripe_sort(morton_order(w, w), G)


def content_order(scores, G: int):
    """Content-aware order of one attention group (Sec. 4.1): cells ranked by score descending
    (ties: lower index), then the stripe interleave.  Returns (sigma, sigma_inv)."""
    sc = _f32(scores).reshape(-1)
    n = sc.size
    sigma = np.empty(n, np.int32)
    sinv = np.empty(n, np.int32)
    _check(lib().oracle_content_order(_p(sc), C.c_int(n), C.c_int(G), _p(sigma), _p(sinv)), "oracle_content_order")
    return sigma, sinv


def content_tables(scores, g: int, ws: int, G: int):
    """Per-image tables of the content-aware order: for every window (ws = 0: the whole grid) the
    scan position -> spatial index gather table (-1 = padding) and scan position -> cell-in-window
    sigma.  scores [g,g] of one image.  Returns (table [nW*S], sigma [nW,S])."""
    sc = _f32(scores).reshape(g, g)
    w = ws if ws > 0 else g
    nws = -(-g // w)
    S = w * w
    table = np.empty((nws * nws, S), np.int32)
    sig = np.empty((nws * nws, S), np.int32)
    for wr in range(nws):
        for wc in range(nws):
            ms = np.full((w, w), -np.inf, np.float32)
            rows, cols = min(w, g - wr * w), min(w, g - wc * w)
            ms[:rows, :cols] = sc[wr * w:wr * w + rows, wc * w:wc * w + cols]
            sigma, _ = content_order(ms, G)
            row, col = wr * w + sigma // w, wc * w + sigma % w
            sig[wr * nws + wc] = sigma
            table[wr * nws + wc] = np.where((row < g) & (col < g), row * g + col, -1)
    return table.reshape(-1), sig


def window_table(g: int, ws: int, G: int) -> np.ndarray:
    nws = (g + ws - 1) // ws
    t = np.empty(nws * nws * ws * ws, np.int32)
    _check(lib().oracle_window_table(C.c_int(g), C.c_int(ws), C.c_int(G), _p(t)), "oracle_window_table")
    return t


def block_mask(S: int, Bm: int, r: float):
    T = (S + Bm - 1) // Bm
    m = np.empty((T, T), np.uint8)
    n_pre = C.c_int(0)
    _check(lib().oracle_block_mask(C.c_int(S), C.c_int(Bm), C.c_double(r), _p(m), C.byref(n_pre)),
           "oracle_block_mask")
    return m, n_pre.value


def attention(q, k, v, rel_h, rel_w, w: int, G: int, Bm: int, r: float, sinv=None) -> np.ndarray:
    """q,k,v [h,S,d] in spatial order, S = w*w; returns [h,S,d] in spatial order."""
    q, k, v, rel_h, rel_w = map(_f32, (q, k, v, rel_h, rel_w))
    h, S, d = q.shape
    assert S == w * w and k.shape == q.shape and v.shape == q.shape
    assert rel_h.shape == (2 * w - 1, d) and rel_w.shape == (2 * w - 1, d)
    out = np.empty_like(q)
    if sinv is None:
        rc = lib().oracle_attention(_p(q), _p(k), _p(v), _p(rel_h), _p(rel_w), C.c_int(h), C.c_int(w),
                                    C.c_int(d), C.c_int(G), C.c_int(Bm), C.c_double(r), _p(out))
    else:
        sinv = _i32(sinv)
        assert sinv.size == S
        rc = lib().oracle_attention_ordered(_p(q), _p(k), _p(v), _p(rel_h), _p(rel_w), C.c_int(h),
                                            C.c_int(w), C.c_int(d), _p(sinv), C.c_int(Bm),
                                            C.c_double(r), _p(out))
    _check(rc, "oracle_attention")
    return out


def score_tokens(x) -> np.ndarray:
    """x [gh,gw,D] -> M [gh,gw] (Eq. 1)."""
    x = _f32(x)
    gh, gw, D = x.shape
    M = np.empty((gh, gw), np.float32)
    _check(lib().oracle_score_tokens(_p(x), C.c_int(gh), C.c_int(gw), C.c_int(D), _p(M)),
           "oracle_score_tokens")
    return M


def keep_count(n: int, rho: float) -> int:
    K = lib().oracle_keep_count(C.c_int(n), C.c_double(rho))
    if K < 0:
        raise ValueError("oracle_keep_count: bad argument")
    return K


def select_tokens(scores, K: int) -> np.ndarray:
    scores = _f32(scores).reshape(-1)
    keep = np.empty(K, np.int32)
    _check(lib().oracle_select_tokens(_p(scores), C.c_int(scores.size), C.c_int(K), _p(keep)),
           "oracle_select_tokens")
    return keep


def routed_mlp(x, keep, ln_g, ln_b, w1, b1, w2, b2, eps: float = 1e-6) -> np.ndarray:
    """x [n,D]; returns the updated copy."""
    x = _f32(x).copy()
    n, D = x.shape
    keep = _i32(keep)
    ln_g, ln_b, w1, b1, w2, b2 = map(_f32, (ln_g, ln_b, w1, b1, w2, b2))
    Dm = w1.shape[0]
    assert w1.shape == (Dm, D) and w2.shape == (D, Dm)
    _check(lib().oracle_routed_mlp(_p(x), C.c_int(n), C.c_int(D), C.c_int(Dm), _p(keep), C.c_int(keep.size),
                                   _p(ln_g), _p(ln_b), C.c_double(eps), _p(w1), _p(b1), _p(w2), _p(b2)),
           "oracle_routed_mlp")
    return x


@dataclass
class BlockWeights:
    """fp32 arrays (values already rounded to bf16 by the generator)."""
    ln1_g: np.ndarray
    ln1_b: np.ndarray
    wqkv: np.ndarray     # [3D, D]
    bqkv: np.ndarray     # [3D]
    rel_h: np.ndarray    # [2w-1, d]
    rel_w: np.ndarray    # [2w-1, d]
    wproj: np.ndarray    # [D, D]
    bproj: np.ndarray    # [D]
    ln2_g: np.ndarray
    ln2_b: np.ndarray
    w1: np.ndarray       # [Dm, D]
    b1: np.ndarray
    w2: np.ndarray       # [D, Dm]
    b2: np.ndarray


def encoder_block(x, wt, h: int, ws: int, G: int, Bm: int, r: float, keep, eps: float = 1e-6,
                  order_scores=None) -> np.ndarray:
    """x [g,g,D] one image; ws = 0 for a global block.  order_scores [g,g]: rank every attention
    group's tokens by these scores (content-aware order) instead of by position.  Returns the block output."""
    x = _f32(x).copy()
    g, g2, D = x.shape
    assert g == g2
    keep = _i32(keep)
    a = {f: _f32(getattr(wt, f)) for f in wt.__dataclass_fields__}
    Dm = a["w1"].shape[0]
    w = ws if ws > 0 else g
    d = D // h
    assert a["rel_h"].shape == (2 * w - 1, d), (a["rel_h"].shape, w, d)
    osc = np.ascontiguousarray(_f32(order_scores).reshape(g, g)) if order_scores is not None else None
    rc = lib().oracle_encoder_block(
        _p(x), C.c_int(g), C.c_int(D), C.c_int(h), C.c_int(Dm), C.c_int(ws), C.c_int(G), C.c_int(Bm),
        C.c_double(r), _p(keep), C.c_int(keep.size), C.c_double(eps),
        _p(osc),
        _p(a["ln1_g"]), _p(a["ln1_b"]), _p(a["wqkv"]), _p(a["bqkv"]), _p(a["rel_h"]), _p(a["rel_w"]),
        _p(a["wproj"]), _p(a["bproj"]), _p(a["ln2_g"]), _p(a["ln2_b"]),
        _p(a["w1"]), _p(a["b1"]), _p(a["w2"]), _p(a["b2"]))
    _check(rc, "oracle_encoder_block")
    return x


def encoder_block_halves(x, wt, h: int, ws: int, G: int, Bm: int, r: float, keep, eps: float = 1e-6, order_scores=None):
    """The block as its two halves, for tests that need the residual stream between them: returns
    (x1, y), x1 = x + attention half (the C routine with an empty keep-set), y = routed MLP applied to
    x1.  This is the composition the C routine itself makes, so y equals encoder_block's result bit
    for bit (checked in the oracle's tests)."""
    x1 = encoder_block(x, wt, h, ws, G, Bm, r, np.zeros(0, np.int32), eps, order_scores=order_scores)
    g, _, D = x1.shape
    y = routed_mlp(x1.reshape(g * g, D), keep, wt.ln2_g, wt.ln2_b, wt.w1, wt.b1, wt.w2, wt.b2, eps).reshape(g, g, D)
    return x1, y


def encoder(x, blocks, h: int, ws: int, global_blocks, G: int, r: float, rho: float,
            Bm_window: int = 32, Bm_global: int = 128, eps: float = 1e-6, content_order: bool = False):
    """One image through a stack of blocks (Sec. 4: scores and keep-set are taken
    once, from the encoder input, and reused by every block).  Returns (y, keep)."""
    x = _f32(x)
    g = x.shape[0]
    K = keep_count(g * g, rho)
    scores = score_tokens(x)
    keep = select_tokens(scores, K)
    for i, wt in enumerate(blocks):
        is_global = i in global_blocks
        x = encoder_block(x, wt, h, 0 if is_global else ws, G, Bm_global if is_global else Bm_window,
                          r, keep, eps, order_scores=scores if content_order else None)
    return x, keep


def patch_embed(img, w, b, pos, P: int) -> np.ndarray:
    """img [3,H,W], w [D,3,P,P], b [D], pos [gh*gw,D] -> tokens [gh,gw,D] (SAM's patch embedding plus the
    absolute position embedding)."""
    img, w, b, pos = map(_f32, (img, w, b, pos))
    _, H, W = img.shape
    D = w.shape[0]
    assert w.shape == (D, 3, P, P) and pos.shape == ((H // P) * (W // P), D)
    x = np.empty(((H // P) * (W // P), D), np.float32)
    _check(lib().oracle_patch_embed(_p(img), C.c_int(H), C.c_int(W), C.c_int(P), _p(w), _p(b), _p(pos), C.c_int(D), _p(x)),
           "oracle_patch_embed")
    return x.reshape(H // P, W // P, D)


def neck(x, w1, ln1_g, ln1_b, w2, ln2_g, ln2_b, eps: float = 1e-6) -> np.ndarray:
    """x [g,g,D]; w1 [C,D]; w2 [C,C,3,3] -> [g,g,C] (SAM's neck: 1x1 conv, LayerNorm over channels, 3x3 conv
    with zero padding, LayerNorm over channels; no conv biases)."""
    x, w1, ln1_g, ln1_b, w2, ln2_g, ln2_b = map(_f32, (x, w1, ln1_g, ln1_b, w2, ln2_g, ln2_b))
    g, _, D = x.shape
    Cn = w1.shape[0]
    assert w1.shape == (Cn, D) and w2.shape == (Cn, Cn, 3, 3)
    out = np.empty((g * g, Cn), np.float32)
    _check(lib().oracle_neck(_p(x), C.c_int(g), C.c_int(D), C.c_int(Cn), _p(w1), _p(ln1_g), _p(ln1_b), _p(w2), _p(ln2_g),
                             _p(ln2_b), C.c_double(eps), _p(out)), "oracle_neck")
    return out.reshape(g, g, Cn)
