"""Python binding of libssam (argument marshalling only).

Every function has the name of the C entry point in ``include/ssam.h`` and does
nothing but check dtypes, pull raw pointers out of torch tensors and forward
them with the current torch stream.  No step of the method runs in Python or in
PyTorch ops.  If the HIP library has not been built the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssam.so")
_lib = None

EPI_BIAS, EPI_BIAS_GELU, EPI_BIAS_SCATTER_ADD, EPI_BIAS_SCATTER = 0, 1, 2, 3
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4


class SsamError(RuntimeError):
    def __init__(self, name, code):
        self.code = code
        super().__init__(f"{name}: {status_string(code)} ({code})")


_WEIGHT_POINTERS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "rel_h", "rel_w", "wproj", "bproj",
                    "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class BlockWeights(C.Structure):
    _fields_ = ([(n, C.c_void_p) for n in _WEIGHT_POINTERS] + [("packed", C.c_int), ("fold_ln1", C.c_int),
                ("qkv_colsum", C.c_void_p), ("bqkv_folded", C.c_void_p), ("fold_kv_bias", C.c_int),
                ("bproj_folded", C.c_void_p), ("fold_ln2", C.c_int), ("fc1_colsum", C.c_void_p),
                ("b1_folded", C.c_void_p)])


class BlockCfg(C.Structure):
    _fields_ = [("B", C.c_int), ("g", C.c_int), ("D", C.c_int), ("heads", C.c_int), ("Dm", C.c_int),
                ("ws", C.c_int), ("mask_block", C.c_int), ("K", C.c_int), ("r", C.c_double), ("eps", C.c_float),
                ("content_order", C.c_int), ("stripe", C.c_int)]


def lib():
    """Load libssam.so; fail loudly if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        L.ssam_status_string.restype = C.c_char_p
        for n in ("ssam_score_tokens_workspace_bytes", "ssam_routed_mlp_workspace_bytes",
                  "ssam_encoder_block_workspace_bytes", "ssam_encoder_workspace_bytes", "ssam_linear_workspace_bytes",
                  "ssam_patch_embed_workspace_bytes", "ssam_neck_workspace_bytes"):
            getattr(L, n).restype = C.c_size_t
        L.ssam_probe_mfma_flops.restype = C.c_double
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().ssam_status_string(C.c_int(code)).decode()


def _check(name, rc):
    if rc != 0:
        raise SsamError(name, rc)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if t is None:
        return C.c_void_p(0)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous device tensor of {dtype}")
    return C.c_void_p(t.data_ptr())


_bf = lambda t, n: _dev(t, torch.bfloat16, n)
_f32 = lambda t, n: _dev(t, torch.float32, n)
_i32 = lambda t, n: _dev(t, torch.int32, n)


# ------------------------------------------------------------------ integer layer (host)
def ssam_build_perm(gh: int, gw: int, G: int):
    perm = np.empty(gh * gw, np.int32)
    inv = np.empty(gh * gw, np.int32)
    _check("ssam_build_perm", lib().ssam_build_perm(C.c_int(gh), C.c_int(gw), C.c_int(G),
                                                    perm.ctypes.data_as(C.c_void_p), inv.ctypes.data_as(C.c_void_p)))
    return perm, inv


def ssam_build_perm_device(gh: int, gw: int, G: int, device="cuda"):
    perm = torch.empty(max(gh * gw, 1), dtype=torch.int32, device=device)
    inv = torch.empty_like(perm)
    _check("ssam_build_perm_device", lib().ssam_build_perm_device(C.c_int(gh), C.c_int(gw), C.c_int(G),
                                                                  _i32(perm, "perm"), _i32(inv, "inv"), _stream()))
    return perm, inv


def ssam_build_window_table(g: int, ws: int, G: int):
    nws = (g + ws - 1) // ws
    t = np.empty(nws * nws * ws * ws, np.int32)
    _check("ssam_build_window_table", lib().ssam_build_window_table(C.c_int(g), C.c_int(ws), C.c_int(G),
                                                                    t.ctypes.data_as(C.c_void_p)))
    return t


def ssam_build_block_mask(S: int, mask_block: int, r: float):
    T = (S + mask_block - 1) // mask_block
    row_ptr = np.empty(T + 1, np.int32)
    col_idx = np.empty(T * T, np.int32)
    n_pre = C.c_int(0)
    _check("ssam_build_block_mask", lib().ssam_build_block_mask(
        C.c_int(S), C.c_int(mask_block), C.c_double(r), row_ptr.ctypes.data_as(C.c_void_p),
        col_idx.ctypes.data_as(C.c_void_p), C.byref(n_pre)))
    return row_ptr, col_idx[: row_ptr[-1]].copy(), n_pre.value


def ssam_keep_count(N: int, rho: float) -> int:
    K = lib().ssam_keep_count(C.c_int(N), C.c_double(rho))
    if K < 0:
        raise SsamError("ssam_keep_count", K)
    return K


# ------------------------------------------------------------------ movers
def ssam_permute(x, idx, y=None):
    B, Nin, D = x.shape
    Nout = idx.numel()
    if y is None:
        y = torch.empty((B, Nout, D), dtype=torch.bfloat16, device=x.device)
    _check("ssam_permute", lib().ssam_permute(_bf(x, "x"), _i32(idx, "idx"), _bf(y, "y"), C.c_int(B), C.c_int(Nin),
                                              C.c_int(Nout), C.c_int(D), _stream()))
    return y


def ssam_unpermute(y, idx, x, residual=None):
    B, Ny, D = y.shape
    Nx = x.shape[1]
    _check("ssam_unpermute", lib().ssam_unpermute(_bf(y, "y"), _i32(idx, "idx"), _bf(x, "x"), _bf(residual, "residual"),
                                                  C.c_int(B), C.c_int(Nx), C.c_int(Ny), C.c_int(D), _stream()))
    return x


def ssam_ln_gather(x, idx, idx_batch_stride, gamma, beta, eps, Nout, y=None):
    B, Nin, D = x.shape
    if y is None:
        y = torch.empty((B, Nout, D), dtype=torch.bfloat16, device=x.device)
    _check("ssam_ln_gather", lib().ssam_ln_gather(_bf(x, "x"), _i32(idx, "idx"), C.c_int(idx_batch_stride),
                                                  _f32(gamma, "gamma"), _f32(beta, "beta"), C.c_float(eps), _bf(y, "y"),
                                                  C.c_int(B), C.c_int(Nin), C.c_int(Nout), C.c_int(D), _stream()))
    return y


def ssam_build_content_tables(scores, g, ws, G=4, gather_table=None, sigma=None):
    """scores [B, g*g] fp32 -> (gather_table [B, nW*S], sigma [B*nW, S]) of the content-aware order."""
    Bn = scores.shape[0]
    w = ws if ws > 0 else g
    nW, S = (-(-g // w)) ** 2, w * w
    if gather_table is None:
        gather_table = torch.empty((Bn, nW * S), dtype=torch.int32, device=scores.device)
    if sigma is None:
        sigma = torch.empty((Bn * nW, S), dtype=torch.int32, device=scores.device)
    _check("ssam_build_content_tables", lib().ssam_build_content_tables(
        _f32(scores, "scores"), C.c_int(Bn), C.c_int(g), C.c_int(ws), C.c_int(G),
        _i32(gather_table, "gather_table"), _i32(sigma, "sigma"), _stream()))
    return gather_table, sigma


# ------------------------------------------------------------------ GEMM
def ssam_linear(A, W, bias, C_out=None, epilogue=EPI_BIAS, row_map=None, rows_per_batch=1, map_batch_stride=0,
                dst_rows_per_batch=1, tile=0):
    M, K = A.shape
    N = W.shape[0]
    assert W.shape[1] == K
    if C_out is None:
        C_out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    _check("ssam_linear", lib().ssam_linear_tiled(
        _bf(A, "A"), _bf(W, "W"), _f32(bias, "bias"), _bf(C_out, "C"), C.c_int(M), C.c_int(N), C.c_int(K),
        C.c_int(epilogue), _i32(row_map, "row_map"), C.c_int(rows_per_batch), C.c_int(map_batch_stride),
        C.c_int(dst_rows_per_batch), C.c_int(tile), _stream()))
    return C_out


def ssam_linear_workspace_bytes():
    return int(lib().ssam_linear_workspace_bytes())


def _rows(t, dtype, name):
    """Pointer and row stride of a 2-D device tensor whose rows are contiguous (a column slice is fine)."""
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.dim() == 2 and t.stride(1) == 1):
        raise TypeError(f"{name}: expected a 2-D device tensor of {dtype} with contiguous rows")
    return C.c_void_p(t.data_ptr()), C.c_int(t.stride(0))


def ssam_linear_ld(A, W, bias, C_out=None, epilogue=EPI_BIAS, row_map=None, rows_per_batch=1, map_batch_stride=0,
                   dst_rows_per_batch=1, tile=0, workspace=None, w_packed=False):
    """ssam_linear on operands with their own row strides, with an optional scratch workspace (uint8);
    w_packed: W is the output of ssam_pack_weight."""
    M, K = A.shape
    N = W.shape[0]
    assert W.shape[1] == K
    if C_out is None:
        C_out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    (pa, lda), (pw, ldw), (pc, ldc) = _rows(A, torch.bfloat16, "A"), _rows(W, torch.bfloat16, "W"), _rows(C_out, torch.bfloat16, "C")
    _check("ssam_linear_ld", lib().ssam_linear_ld(
        pa, lda, pw, ldw, C.c_int(1 if w_packed else 0), _f32(bias, "bias"), pc, ldc, C.c_int(M), C.c_int(N), C.c_int(K),
        C.c_int(epilogue), _i32(row_map, "row_map"), C.c_int(rows_per_batch), C.c_int(map_batch_stride),
        C.c_int(dst_rows_per_batch), C.c_int(tile), _dev(workspace, torch.uint8, "workspace"),
        C.c_size_t(0 if workspace is None else workspace.numel()), _stream()))
    return C_out


# ------------------------------------------------------------------ attention
def ssam_sparse_attention(qkv, rel_h, rel_w, sigma, w, mask_block, r, scale=None, out=None, out_rows=None):
    """qkv: packed [groups, S, 3, h, d] bf16; sigma [S] shared, or [groups, S] per group.  Returns [groups, S, h*d]."""
    groups, S, three, h, d = qkv.shape
    assert three == 3
    if out is None:
        out = torch.empty((groups, S, h * d), dtype=torch.bfloat16, device=qkv.device)
    if scale is None:
        scale = d ** -0.5
    base = qkv.data_ptr()
    _bf(qkv, "qkv")
    esz = 2
    _check("ssam_sparse_attention", lib().ssam_sparse_attention(
        C.c_void_p(base), C.c_void_p(base + h * d * esz), C.c_void_p(base + 2 * h * d * esz), C.c_long(3 * h * d),
        _bf(rel_h, "rel_h"), _bf(rel_w, "rel_w"), _i32(sigma, "sigma"), C.c_long(S if sigma.dim() == 2 else 0),
        _bf(out, "out"), _i32(out_rows, "out_rows"),
        C.c_int(groups), C.c_int(S), C.c_int(w), C.c_int(h), C.c_int(d), C.c_int(mask_block), C.c_double(r),
        C.c_float(scale), _stream()))
    return out


# ------------------------------------------------------------------ routed MLP
def ssam_score_tokens(x, scores=None, workspace=None):
    B, gh, gw, D = x.shape
    if scores is None:
        scores = torch.empty((B, gh * gw), dtype=torch.float32, device=x.device)
    need = lib().ssam_score_tokens_workspace_bytes(C.c_int(B), C.c_int(gh), C.c_int(gw))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check("ssam_score_tokens", lib().ssam_score_tokens(_bf(x, "x"), _f32(scores, "scores"), C.c_int(B), C.c_int(gh),
                                                        C.c_int(gw), C.c_int(D), C.c_void_p(workspace.data_ptr()),
                                                        C.c_size_t(workspace.numel()), _stream()))
    return scores


def ssam_score_tokens_static(x, scores):
    """The allocation-free entry point: `scores` [B, gh*gw] fp32 is the caller's; no workspace."""
    B, gh, gw, D = x.shape
    _check("ssam_score_tokens_static", lib().ssam_score_tokens_static(_bf(x, "x"), _f32(scores, "scores"), C.c_int(B),
                                                                      C.c_int(gh), C.c_int(gw), C.c_int(D), _stream()))
    return scores


def ssam_select_tokens(scores, K, keep_idx=None):
    B, N = scores.shape
    if keep_idx is None:
        keep_idx = torch.empty((B, K), dtype=torch.int32, device=scores.device)
    _check("ssam_select_tokens", lib().ssam_select_tokens(_f32(scores, "scores"), _i32(keep_idx, "keep_idx"),
                                                          C.c_int(B), C.c_int(N), C.c_int(K), _stream()))
    return keep_idx


def ssam_routed_mlp_workspace_bytes(B, K, D, Dm) -> int:
    return lib().ssam_routed_mlp_workspace_bytes(C.c_int(B), C.c_int(K), C.c_int(D), C.c_int(Dm))


def ssam_routed_mlp(x, keep_idx, ln_g, ln_b, eps, w1, b1, w2, b2, workspace=None, w_packed=False):
    """w_packed: w1 and w2 are outputs of ssam_pack_weight (ssam_routed_mlp_packed)."""
    B, N, D = x.shape
    Dm = w1.shape[0]
    K = keep_idx.shape[1]
    if workspace is None:
        workspace = torch.empty(ssam_routed_mlp_workspace_bytes(B, K, D, Dm), dtype=torch.uint8, device=x.device)
    name = "ssam_routed_mlp_packed" if w_packed else "ssam_routed_mlp"
    _check(name, getattr(lib(), name)(
        _bf(x, "x"), _i32(keep_idx, "keep_idx"), _f32(ln_g, "ln_g"), _f32(ln_b, "ln_b"), C.c_float(eps),
        _bf(w1, "w1"), _f32(b1, "b1"), _bf(w2, "w2"), _f32(b2, "b2"),
        C.c_int(B), C.c_int(N), C.c_int(D), C.c_int(Dm), C.c_int(K),
        C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream()))
    return x


def ssam_routed_mlp_packed(x, keep_idx, ln_g, ln_b, eps, w1p, b1, w2p, b2, workspace=None):
    return ssam_routed_mlp(x, keep_idx, ln_g, ln_b, eps, w1p, b1, w2p, b2, workspace=workspace, w_packed=True)


def ssam_routed_mlp_folded(x, keep_idx, eps, w1fp, colsum1, b1f, w2p, b2, workspace=None):
    """Gather and LN2 folded into fc1: w1fp = ssam_pack_weight(Wf), (Wf, colsum1, b1f) = ssam_fold_ln_weight(w1, b1,
    ln_g, ln_b); w2p = ssam_pack_weight(w2)."""
    B, N, D = x.shape
    Dm = w1fp.shape[0]
    K = keep_idx.shape[1]
    if workspace is None:
        workspace = torch.empty(ssam_routed_mlp_workspace_bytes(B, K, D, Dm), dtype=torch.uint8, device=x.device)
    _check("ssam_routed_mlp_folded", lib().ssam_routed_mlp_folded(
        _bf(x, "x"), _i32(keep_idx, "keep_idx"), C.c_float(eps),
        _bf(w1fp, "w1fp"), _f32(colsum1, "colsum1"), _f32(b1f, "b1f"), _bf(w2p, "w2p"), _f32(b2, "b2"),
        C.c_int(B), C.c_int(N), C.c_int(D), C.c_int(Dm), C.c_int(K),
        C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream()))
    return x


# ------------------------------------------------------------------ block / encoder
_BF16_FIELDS = ("wqkv", "rel_h", "rel_w", "wproj", "w1", "w2")


_PACKABLE = ("wqkv", "wproj", "w1", "w2")


def ssam_pack_weight(W, Wp=None):
    """Row-major [N][K] bf16 weight -> MFMA fragment order (same shape and bytes, different order)."""
    N, K = W.shape
    pw, ldw = _rows(W, torch.bfloat16, "W")
    if Wp is None:
        Wp = torch.empty((N, K), dtype=torch.bfloat16, device=W.device)
    _check("ssam_pack_weight", lib().ssam_pack_weight(pw, ldw, _bf(Wp, "Wp"), C.c_int(N), C.c_int(K), _stream()))
    return Wp


def ssam_ln_stats(x, eps=1e-6):
    """x: [..., D] bf16 contiguous -> [rows, 2] fp32 {rstd, -rstd*mean}."""
    _dev(x, torch.bfloat16, "x")
    D = x.shape[-1]
    rows = x.numel() // D
    stats = torch.empty((rows, 2), dtype=torch.float32, device=x.device)
    _check("ssam_ln_stats", lib().ssam_ln_stats(_bf(x, "x"), _f32(stats, "stats"), C.c_long(rows), C.c_int(D),
                                                  C.c_float(eps), _stream()))
    return stats


def ssam_fold_ln_weight(W, bias, gamma, beta):
    """-> (Wf [N,K] bf16, colsum [N] fp32, bias_f [N] fp32), see the header."""
    _dev(W, torch.bfloat16, "W")
    N, K = W.shape
    Wf = torch.empty((N, K), dtype=torch.bfloat16, device=W.device)
    colsum = torch.empty(N, dtype=torch.float32, device=W.device)
    bias_f = torch.empty(N, dtype=torch.float32, device=W.device)
    _check("ssam_fold_ln_weight", lib().ssam_fold_ln_weight(
        _bf(W, "W"), C.c_int(K), _f32(bias, "bias"), _f32(gamma, "gamma"), _f32(beta, "beta"), _bf(Wf, "Wf"),
        _f32(colsum, "colsum"), _f32(bias_f, "bias_f"), C.c_int(N), C.c_int(K), _stream()))
    return Wf, colsum, bias_f


def ssam_linear_ln(x, stats, Wfp, colsum, bias_f, out, row_map, rows_per_batch, map_batch_stride, dst_rows_per_batch):
    """out[dst(m)] = Linear(LN(x[m])) with the LayerNorm folded in; x [M,K], Wfp packed [N,K], out [rows,N]."""
    _dev(x, torch.bfloat16, "x"); _dev(out, torch.bfloat16, "out")
    M, K = x.shape
    N = Wfp.shape[0]
    _check("ssam_linear_ln", lib().ssam_linear_ln(
        _bf(x, "x"), C.c_int(K), _f32(stats, "stats"), _bf(Wfp, "Wfp"), _f32(colsum, "colsum"), _f32(bias_f, "bias_f"),
        _bf(out, "out"), C.c_int(out.shape[-1]), C.c_int(M), C.c_int(N), C.c_int(K), _i32(row_map, "row_map"),
        C.c_int(rows_per_batch), C.c_int(map_batch_stride), C.c_int(dst_rows_per_batch), _stream()))
    return out


def ssam_fold_kv_bias(bias_in, bqkv, wproj, bproj):
    """-> (bias_out [3D], bproj_out [D]) fp32, see the header; wproj row-major."""
    D = bproj.numel()
    _dev(wproj, torch.bfloat16, "wproj")
    bias_out = torch.empty(3 * D, dtype=torch.float32, device=bproj.device)
    bproj_out = torch.empty(D, dtype=torch.float32, device=bproj.device)
    _check("ssam_fold_kv_bias", lib().ssam_fold_kv_bias(
        _f32(bias_in, "bias_in"), _f32(bqkv, "bqkv"), _bf(wproj, "wproj"), _f32(bproj, "bproj"), _f32(bias_out, "bias_out"),
        _f32(bproj_out, "bproj_out"), C.c_int(D), _stream()))
    return bias_out, bproj_out


def pack_block_weights(wt: dict, fold_ln1=False, fold_kv_bias=False, fold_ln2=False) -> dict:
    """Device weight dict (row-major weights) -> the same with the four Linear weights in fragment order (flagged
    'packed').  fold_ln1: wqkv becomes the packed LN1-folded weight (ssam_fold_ln_weight), with its column sums
    and bias; fold_kv_bias (with fold_ln1): the key and value biases move out of the contraction (ssam_fold_kv_bias);
    fold_ln2: w1 becomes the packed LN2-folded weight, with its column sums and bias."""
    out = dict(wt)
    for k in _PACKABLE:
        out[k] = ssam_pack_weight(wt[k])
    out["packed"] = True
    if fold_ln1:
        Wf, colsum, bias_f = ssam_fold_ln_weight(wt["wqkv"], wt["bqkv"], wt["ln1_g"], wt["ln1_b"])
        out["wqkv"] = ssam_pack_weight(Wf)
        out["qkv_colsum"], out["bqkv_folded"], out["fold_ln1"] = colsum, bias_f, True
        if fold_kv_bias:
            out["bqkv_folded"], out["bproj_folded"] = ssam_fold_kv_bias(bias_f, wt["bqkv"], wt["wproj"], wt["bproj"])
            out["fold_kv_bias"] = True
    elif fold_kv_bias:
        raise ValueError("fold_kv_bias needs fold_ln1")
    if fold_ln2:
        Wf, colsum, bias_f = ssam_fold_ln_weight(wt["w1"], wt["b1"], wt["ln2_g"], wt["ln2_b"])
        out["w1"] = ssam_pack_weight(Wf)
        out["fc1_colsum"], out["b1_folded"], out["fold_ln2"] = colsum, bias_f, True
    return out


def upload_block_weights(wdict: dict, device="cuda", pack=False, fold_ln1=False, fold_kv_bias=False, fold_ln2=False) -> dict:
    """numpy fp32 dict (bf16-representable values) -> device tensors in the ABI's dtypes."""
    out = {}
    for k, v in wdict.items():
        t = torch.from_numpy(np.ascontiguousarray(v))
        out[k] = t.to(device=device, dtype=torch.bfloat16 if k in _BF16_FIELDS else torch.float32).contiguous()
    if not pack:
        if fold_ln2:
            raise ValueError("fold_ln2 needs pack")
        return out
    return pack_block_weights(out, fold_ln1=fold_ln1, fold_kv_bias=fold_kv_bias, fold_ln2=fold_ln2)


def block_weights_struct(wt: dict) -> BlockWeights:
    s = BlockWeights()
    for name in _WEIGHT_POINTERS:
        t = wt[name]
        want = torch.bfloat16 if name in _BF16_FIELDS else torch.float32
        _dev(t, want, name)
        setattr(s, name, t.data_ptr())
    s.packed = 1 if wt.get("packed") else 0
    s.fold_ln1 = 1 if wt.get("fold_ln1") else 0
    if s.fold_ln1:
        for name in ("qkv_colsum", "bqkv_folded"):
            _dev(wt[name], torch.float32, name)
            setattr(s, name, wt[name].data_ptr())
    s.fold_kv_bias = 1 if wt.get("fold_kv_bias") else 0
    if s.fold_kv_bias:
        _dev(wt["bproj_folded"], torch.float32, "bproj_folded")
        s.bproj_folded = wt["bproj_folded"].data_ptr()
    s.fold_ln2 = 1 if wt.get("fold_ln2") else 0
    if s.fold_ln2:
        for name in ("fc1_colsum", "b1_folded"):
            _dev(wt[name], torch.float32, name)
            setattr(s, name, wt[name].data_ptr())
    return s


def make_cfg(B, g, D, heads, Dm, ws, mask_block, K, r, eps=1e-6, content_order=False, stripe=4) -> BlockCfg:
    return BlockCfg(B, g, D, heads, Dm, ws, mask_block, K, r, eps, 1 if content_order else 0, stripe)


def ssam_encoder_block_workspace_bytes(cfg: BlockCfg) -> int:
    return lib().ssam_encoder_block_workspace_bytes(C.byref(cfg))


def ssam_encoder_block(x, wstruct: BlockWeights, cfg: BlockCfg, gather_table, sigma, keep_idx, workspace=None):
    if workspace is None:
        workspace = torch.empty(ssam_encoder_block_workspace_bytes(cfg), dtype=torch.uint8, device=x.device)
    _check("ssam_encoder_block", lib().ssam_encoder_block(
        _bf(x, "x"), C.byref(wstruct), C.byref(cfg), _i32(gather_table, "gather_table"), _i32(sigma, "sigma"),
        _i32(keep_idx, "keep_idx"), C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream()))
    return x


def ssam_encoder_workspace_bytes(cfg_local, cfg_global) -> int:
    return lib().ssam_encoder_workspace_bytes(C.byref(cfg_local) if cfg_local is not None else None,
                                              C.byref(cfg_global) if cfg_global is not None else None)


class EncoderPlan:
    """Host-side argument block of ssam_encoder_forward, marshalled once and reused."""

    def __init__(self, wstructs, is_global):
        self.n = len(wstructs)
        self.weights = (BlockWeights * self.n)(*wstructs)
        self.flags = (C.c_uint8 * self.n)(*[1 if f else 0 for f in is_global])


def ssam_encoder_forward(x, wstructs, is_global, cfg_local, cfg_global, window_table, sigma_window,
                         global_table, sigma_global, scores, keep_idx, workspace, qkv_events=None, plan=None):
    """qkv_events: optional ctypes array of 2*n_blocks hipEvent_t handles (c_void_p)."""
    if plan is None:
        plan = EncoderPlan(wstructs, is_global)
    n, arr, flags = plan.n, plan.weights, plan.flags
    _check("ssam_encoder_forward", lib().ssam_encoder_forward(
        _bf(x, "x"), arr, flags, C.c_int(n),
        C.byref(cfg_local) if cfg_local is not None else None,
        C.byref(cfg_global) if cfg_global is not None else None,
        _i32(window_table, "window_table"), _i32(sigma_window, "sigma_window"),
        _i32(global_table, "global_table"), _i32(sigma_global, "sigma_global"),
        _f32(scores, "scores"), _i32(keep_idx, "keep_idx"),
        C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), qkv_events, _stream()))
    return x


# ------------------------------------------------------------------ encoder ends
def ssam_patch_embed_workspace_bytes(B, H, W, P) -> int:
    return lib().ssam_patch_embed_workspace_bytes(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(P))


def ssam_patch_embed(img, w, bias, pos, P, x=None, workspace=None):
    """img [B,3,H,W] bf16; w [D,3*P*P] bf16; bias [D] fp32; pos [N,D] bf16 -> tokens [B,N,D] bf16."""
    Bn, three, H, W = img.shape
    D = w.shape[0]
    N = (H // P) * (W // P)
    assert three == 3 and w.shape[1] == 3 * P * P
    if x is None:
        x = torch.empty((Bn, N, D), dtype=torch.bfloat16, device=img.device)
    if workspace is None:
        workspace = torch.empty(ssam_patch_embed_workspace_bytes(Bn, H, W, P), dtype=torch.uint8, device=img.device)
    _check("ssam_patch_embed", lib().ssam_patch_embed(
        _bf(img, "img"), _bf(w, "w"), _f32(bias, "bias"), _bf(pos, "pos"), _bf(x, "x"), C.c_int(Bn), C.c_int(H), C.c_int(W),
        C.c_int(P), C.c_int(D), C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream()))
    return x


def ssam_neck_workspace_bytes(B, g, D, Cn) -> int:
    return lib().ssam_neck_workspace_bytes(C.c_int(B), C.c_int(g), C.c_int(D), C.c_int(Cn))


def neck_conv3_weight(w2):
    """[C,C,3,3] convolution weight (out, in, ky, kx) -> the [C, 9*C] layout of ssam_neck (out; ky, kx, in)."""
    Cn = w2.shape[0]
    return w2.permute(0, 2, 3, 1).reshape(Cn, 9 * Cn).contiguous()


def ssam_neck(x, w1, ln1_g, ln1_b, w2, ln2_g, ln2_b, g, eps=1e-6, out=None, workspace=None):
    """x [B,g*g,D] bf16; w1 [C,D]; w2 [C,9*C] (see neck_conv3_weight) -> [B,g*g,C] bf16."""
    Bn, N, D = x.shape
    Cn = w1.shape[0]
    assert N == g * g and w2.shape == (Cn, 9 * Cn)
    if out is None:
        out = torch.empty((Bn, N, Cn), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty(ssam_neck_workspace_bytes(Bn, g, D, Cn), dtype=torch.uint8, device=x.device)
    _check("ssam_neck", lib().ssam_neck(
        _bf(x, "x"), _bf(w1, "w1"), _f32(ln1_g, "ln1_g"), _f32(ln1_b, "ln1_b"), _bf(w2, "w2"), _f32(ln2_g, "ln2_g"),
        _f32(ln2_b, "ln2_b"), C.c_float(eps), _bf(out, "out"), C.c_int(Bn), C.c_int(g), C.c_int(D), C.c_int(Cn),
        C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream()))
    return out


# ------------------------------------------------------------------ instrumentation
def ssam_probe_mfma_flops(workgroups: int, iters: int) -> float:
    return float(lib().ssam_probe_mfma_flops(C.c_int(workgroups), C.c_int(iters)))


def ssam_probe_mfma(shape: int, workgroups: int, iters: int, sink=None):
    """Enqueue the MFMA-only loop (see the header); returns the flops of the launch.  The caller times it."""
    if sink is None:
        sink = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    _check("ssam_probe_mfma", lib().ssam_probe_mfma(C.c_int(shape), C.c_int(workgroups), C.c_int(iters), _f32(sink, "sink"), _stream()))
    return ssam_probe_mfma_flops(workgroups, iters)
