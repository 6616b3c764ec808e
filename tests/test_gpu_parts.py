"""GPU parity of the individual entry points against the CPU oracle (or, for the
pure data movers and the dense contraction, against the definition written with
numpy on the oracle's tables).  Every call goes through the C ABI."""
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


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(DEV)


# ------------------------------------------------------------------ integer layer
@pytest.mark.parametrize("gh,gw,G", [(14, 14, 4), (28, 28, 4), (64, 64, 4), (70, 70, 4), (5, 9, 1), (14, 14, 1), (128, 128, 4)])
def test_perm_device_bit_exact(gh, gw, G):
    announce("perm_device", gh, gw, G)
    perm, inv = B.ssam_build_perm_device(gh, gw, G)
    torch.cuda.synchronize()
    sigma, sinv = oracle.stripe_sort(oracle.morton_order(gh, gw), G)
    assert np.array_equal(perm.cpu().numpy(), sigma)
    assert np.array_equal(inv.cpu().numpy(), sinv)


# ------------------------------------------------------------------ movers
@pytest.mark.parametrize("B_,g,ws,D", [(2, 28, 14, 768), (1, 64, 14, 1280), (3, 16, 6, 64)])
def test_permute_unpermute_roundtrip(B_, g, ws, D):
    announce("permute", B_, g, ws, D)
    rng = np.random.default_rng(0)
    x = inputs.bf16_round(rng.normal(size=(B_, g * g, D)).astype(np.float32))
    table = oracle.window_table(g, ws, 4)
    xd, td = dev_bf16(x), dev_i32(B.ssam_build_window_table(g, ws, 4))     # GPU side: the library's own table
    y = B.ssam_permute(xd, td)
    expect = np.where(table[None, :, None] >= 0, x[:, np.maximum(table, 0)], 0.0)
    assert np.array_equal(to_np(y), expect)                       # pure copy: bit exact
    back = torch.full_like(xd, 7.0)
    B.ssam_unpermute(y, td, back)
    assert np.array_equal(to_np(back), x)                          # inverse restores the input bit for bit
    res = inputs.bf16_round(rng.normal(size=x.shape).astype(np.float32))
    out = torch.zeros_like(xd)
    B.ssam_unpermute(y, td, out, dev_bf16(res))
    assert np.array_equal(to_np(out), inputs.bf16_round(x + res))  # one fp32 add, one rounding
    # global order
    sigma, sinv = oracle.grid_sigma(g, 4)
    sig_lib, inv_lib = B.ssam_build_perm_device(g, g, 4)
    y2 = B.ssam_permute(xd, sig_lib)
    assert np.array_equal(to_np(y2), x[:, sigma])
    assert np.array_equal(to_np(B.ssam_permute(y2, inv_lib)), x)


@pytest.mark.parametrize("B_,n,D,K", [(2, 784, 768, 313), (1, 300, 1280, 300), (2, 100, 1024, 7), (1, 50, 2048, 50), (1, 64, 64, 64)])
def test_ln_gather(B_, n, D, K):
    announce("ln_gather", B_, n, D, K)
    rng = np.random.default_rng(1)
    x = inputs.bf16_round((rng.normal(size=(B_, n, D)) * 2 + 0.5).astype(np.float32))
    g = (1 + 0.1 * rng.normal(size=D)).astype(np.float32)
    b = (0.1 * rng.normal(size=D)).astype(np.float32)
    idx = np.stack([rng.permutation(n)[:K] for _ in range(B_)]).astype(np.int32)
    idx[:, 0] = -1                                                 # a padding slot
    y = B.ssam_ln_gather(dev_bf16(x), dev_i32(idx), K, dev_f32(g), dev_f32(b), 1e-6, K)
    xd = torch.from_numpy(x).double()
    ref = torch.nn.functional.layer_norm(xd, (D,), torch.from_numpy(g).double(), torch.from_numpy(b).double(), 1e-6).numpy()
    ref = np.stack([ref[i, np.maximum(idx[i], 0)] for i in range(B_)])
    ref[:, 0] = 0.0
    assert_close(to_np(y), ref, "ln_gather", tol=1e-2)
    assert np.all(to_np(y)[:, 0] == 0.0)


# ------------------------------------------------------------------ scores / select
@pytest.mark.parametrize("B_,g,D", [(2, 28, 768), (1, 64, 1280), (3, 9, 64)])
def test_score_tokens(B_, g, D):
    announce("score_tokens", B_, g, D)
    rng = np.random.default_rng(2)
    x = inputs.token_field(rng, B_, g, D)
    s = to_np(B.ssam_score_tokens(dev_bf16(x)))
    ref = np.stack([oracle.score_tokens(x[b]).reshape(-1) for b in range(B_)])
    np.testing.assert_allclose(s, ref, rtol=2e-5, atol=2e-5 * np.abs(ref).max())


def _check_select(scores, K):
    B_, n = scores.shape
    got = B.ssam_select_tokens(dev_f32(scores), K).cpu().numpy()
    for b in range(B_):
        assert np.array_equal(got[b], oracle.select_tokens(scores[b], K)), (b, n, K)


@pytest.mark.parametrize("n,rho", [(4096, 0.4), (4096, 0.3), (4096, 0.2), (4096, 0.6), (4096, 1.0), (784, 0.4), (100, 0.01), (5000, 0.5)])
def test_select_tokens_lognormal(n, rho):
    announce("select", n, rho)
    rng = np.random.default_rng(3)
    _check_select(inputs.lognormal_scores(rng, 4, n), oracle.keep_count(n, rho))


def test_select_tokens_ties_and_specials():
    announce("select ties")
    rng = np.random.default_rng(4)
    n = 4096
    s = inputs.lognormal_scores(rng, 5, n)
    s[0] = 1.0                                                      # all equal -> 0..K-1
    s[1] = np.round(s[1] * 2) / 2                                   # heavy ties at the threshold
    s[2, ::3] = 0.0
    s[2, 1::3] = -0.0
    s[2, 2::3] = -1.0                                               # signed zeros tie, negatives rank below
    s[3] = -s[3]                                                    # all negative
    s[4, :100] = np.nan
    s[4, 100:200] = -np.inf
    s[4, 200:300] = np.inf
    for K in (1, 37, 1638, 2800, 4096):
        _check_select(s, K)


# ------------------------------------------------------------------ dense contraction
def _gemm_ref(A, W, b):
    return A.astype(np.float64) @ W.astype(np.float64).T + b.astype(np.float64)


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
@pytest.mark.parametrize("M,N,K", [(300, 256, 64), (1000, 512, 192), (513, 768, 768), (64, 256, 128)])
def test_linear_bias_and_gelu(tile, M, N, K):
    announce("linear", tile, M, N, K)
    rng = np.random.default_rng(5)
    A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    ref = _gemm_ref(A, W, b)
    out = B.ssam_linear(dev_bf16(A), dev_bf16(W), dev_f32(b), tile=tile)
    assert_close(to_np(out), ref, f"linear bias tile{tile}", tol=1e-2)
    out = B.ssam_linear(dev_bf16(A), dev_bf16(W), dev_f32(b), epilogue=B.EPI_BIAS_GELU, tile=tile)
    gelu = torch.nn.functional.gelu(torch.from_numpy(ref)).numpy()
    assert_close(to_np(out), gelu, f"linear gelu tile{tile}", tol=1e-2)


@pytest.mark.parametrize("tile,M,N", [(1, 8400, 2048), (2, 8400, 1024), (3, 4200, 2048), (0, 8400, 2048)])
def test_linear_tail_launch(tile, M, N):
    """Shapes whose tiles fill one round of workgroups plus a few: whole rounds of the large tile and
    a second launch of smaller tiles for the rest (ragged last tile row included).  K is never split,
    so every tile choice gives the same bits."""
    announce("linear tail launch", tile, M, N)
    K = 128
    rng = np.random.default_rng(15)
    A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    Ad, Wd, bd = dev_bf16(A), dev_bf16(W), dev_f32(b)
    out = B.ssam_linear(Ad, Wd, bd, tile=tile)
    assert_close(to_np(out), _gemm_ref(A, W, b), f"linear tail tile{tile}", tol=1e-2)
    other = B.ssam_linear(Ad, Wd, bd, tile=3 if tile != 3 else 2)
    assert torch.equal(out, other)


@pytest.mark.parametrize("tile,M,N,epi", [(1, 8400, 2048, 0), (3, 4200, 2048, 1), (1, 8400, 2048, 2), (2, 8400, 1024, 2)])
def test_linear_tail_cut_along_k(tile, M, N, epi):
    """Few left-over tiles and a long K with a workspace: the left-over launch splits K, partial tiles
    are added in a fixed order.  Bias, GELU and scatter epilogues; reproducible bit for bit."""
    announce("linear K-split tail", tile, M, N, epi)
    K = 2048
    rng = np.random.default_rng(16)
    A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    ws = torch.empty(B.ssam_linear_workspace_bytes(), dtype=torch.uint8, device=DEV)
    Ad, Wd, bd = dev_bf16(A), dev_bf16(W), dev_f32(b)
    ref = _gemm_ref(A, W, b)
    if epi == 2:
        x = inputs.bf16_round(rng.normal(size=(M + 50, N)).astype(np.float32))
        rows = np.sort(rng.permutation(M + 50)[:M]).astype(np.int32)
        outs = []
        for _ in range(2):
            xd = dev_bf16(x)
            B.ssam_linear_ld(Ad, Wd, bd, xd, epilogue=B.EPI_BIAS_SCATTER_ADD, row_map=dev_i32(rows), rows_per_batch=M,
                             map_batch_stride=0, dst_rows_per_batch=M + 50, tile=tile, workspace=ws)
            outs.append(xd)
        assert torch.equal(outs[0], outs[1])
        got = to_np(outs[0])
        untouched = np.setdiff1d(np.arange(M + 50), rows)
        assert np.array_equal(got[untouched].view(np.uint32), x[untouched].view(np.uint32))
        assert_close(got[rows] - x[rows], ref, f"K-split scatter tile{tile}", stored=got[rows])
        return
    out = B.ssam_linear_ld(Ad, Wd, bd, epilogue=epi, tile=tile, workspace=ws)
    again = B.ssam_linear_ld(Ad, Wd, bd, epilogue=epi, tile=tile, workspace=ws)
    assert torch.equal(out, again)
    if epi == 1:
        ref = torch.nn.functional.gelu(torch.from_numpy(ref)).numpy()
    assert_close(to_np(out), ref, f"K-split tail tile{tile} epi{epi}", tol=1e-2)
    plain = B.ssam_linear(Ad, Wd, bd, epilogue=epi, tile=tile)
    assert_close(to_np(out), to_np(plain).astype(np.float64), "K-split against one-pass tail", tol=1e-2)


@pytest.mark.parametrize("tile,M,N,K,epi", [(1, 700, 512, 192, 0), (3, 333, 384, 64, 1), (0, 8400, 2048, 2048, 0),
                                            (1, 8400, 2048, 128, 2), (3, 4200, 2048, 2048, 0),
                                            (4, 8400, 2048, 2048, 2), (4, 700, 512, 192, 1),
                                            # widths that are multiples of 128 but not of the 256-wide tiles: the last
                                            # tile column has no W blocks past N to read
                                            (4, 700, 384, 192, 0), (1, 309, 1408, 1216, 0), (0, 5102, 1152, 704, 1)])
def test_linear_packed_weights(tile, M, N, K, epi):
    """Weights in MFMA fragment order (ssam_pack_weight): same bits as the row-major form, on the plain,
    left-over and K-split launches and with every epilogue."""
    announce("linear packed", tile, M, N, K, epi)
    rng = np.random.default_rng(18)
    A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    Ad, Wd, bd = dev_bf16(A), dev_bf16(W), dev_f32(b)
    Wp = B.ssam_pack_weight(Wd)
    # the packing itself, against its definition
    ref_p = to_np(Wd).reshape(N // 16, 16, K // 32, 4, 8).transpose(0, 2, 3, 1, 4).reshape(N, K)
    assert np.array_equal(to_np(Wp), ref_p)
    ws = torch.empty(B.ssam_linear_workspace_bytes(), dtype=torch.uint8, device=DEV)
    kw = {}
    if epi == 2:
        rows = np.sort(rng.permutation(M + 9)[:M]).astype(np.int32)
        kw = dict(row_map=dev_i32(rows), rows_per_batch=M, map_batch_stride=0, dst_rows_per_batch=M + 9)
        x = inputs.bf16_round(rng.normal(size=(M + 9, N)).astype(np.float32))
        o1, o2 = dev_bf16(x), dev_bf16(x)
    else:
        o1 = o2 = None
    o1 = B.ssam_linear_ld(Ad, Wd, bd, o1, epilogue=epi, tile=tile, workspace=ws, **kw)
    o2 = B.ssam_linear_ld(Ad, Wp, bd, o2, epilogue=epi, tile=tile, workspace=ws, w_packed=True, **kw)
    if tile != 0:
        assert torch.equal(o1, o2)             # the same (forced) tile: the same bits
    else:                                      # the automatic choice may differ between the layouts
        assert_close(to_np(o2), to_np(o1).astype(np.float64), "packed against row-major, automatic tile", tol=1e-2)
    if epi == 0:
        assert_close(to_np(o2), _gemm_ref(A, W, b), "packed linear", tol=1e-2)
    with pytest.raises(B.SsamError) as e:
        B.ssam_linear_ld(Ad, Wp, bd, epilogue=0, tile=2, w_packed=True)
    assert e.value.code == B.EUNSUPPORTED


@pytest.mark.parametrize("tile,M,N,K,packed", [(0, 500, 256, 128, False), (1, 8400, 2048, 2048, True), (3, 4200, 2048, 128, False),
                                                (4, 8400, 2048, 2048, True)])
def test_linear_mapped_store(tile, M, N, K, packed):
    """SSAM_EPI_BIAS_SCATTER: row m of the product is stored at the mapped row (negative: dropped), the rows
    the map does not name keep their bits; plain, left-over and K-split launches."""
    announce("linear mapped store", tile, M, N, K, packed)
    rng = np.random.default_rng(19)
    A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    rows_out = M + 77
    dst = rng.permutation(rows_out)[:M].astype(np.int32)
    dst[3] = -1
    Wd = dev_bf16(W)
    if packed:
        Wd = B.ssam_pack_weight(Wd)
    ws = torch.empty(B.ssam_linear_workspace_bytes(), dtype=torch.uint8, device=DEV)
    out = torch.full((rows_out, N), 5.0, dtype=torch.bfloat16, device=DEV)
    B.ssam_linear_ld(dev_bf16(A), Wd, dev_f32(b), out, epilogue=B.EPI_BIAS_SCATTER, row_map=dev_i32(dst), rows_per_batch=M,
                     map_batch_stride=0, dst_rows_per_batch=rows_out, tile=tile, workspace=ws, w_packed=packed)
    got = to_np(out)
    ref = _gemm_ref(A, W, b)
    ok = dst >= 0
    assert_close(got[dst[ok]], ref[ok], "mapped store", tol=1e-2)
    untouched = np.setdiff1d(np.arange(rows_out), dst[ok])
    assert np.all(got[untouched] == 5.0)


_SWEEP_REF = {}


def _sweep_case(M, N, K):
    key = (M, N, K)
    if key not in _SWEEP_REF:
        rng = np.random.default_rng(M + N + K)
        A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
        W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
        b = rng.normal(size=N).astype(np.float32)
        ref = (A @ W.T).astype(np.float64) + b                      # operands are bf16-exact; fp32 sums are ample here
        _SWEEP_REF.clear()                                          # one case resident at a time
        _SWEEP_REF[key] = (A, W, b, ref, dev_bf16(A), dev_bf16(W), dev_f32(b))
    return _SWEEP_REF[key]


@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("epi", [0, 1, 2, 3])
@pytest.mark.parametrize("tile,M,N,K", [(1, 8400, 2048, 256), (1, 8400, 2048, 1024), (2, 8400, 1024, 256), (2, 8400, 1024, 1024),
                                        (3, 4200, 2048, 256), (3, 4200, 2048, 1024), (3, 4150, 2048, 1024),
                                        (4, 8400, 2048, 256), (4, 8400, 2048, 1024), (4, 8350, 2048, 1024)])
def test_linear_every_instantiation(tile, M, N, K, epi, packed):
    """Every kernel instantiation the dispatcher can reach: large tile, its left-over launch (plain at K = 256,
    cut along K at K = 1024 with a workspace), each epilogue, row-major and packed weights, ragged last rows."""
    if packed and tile == 2:
        pytest.skip("the 256x128 tile has no packed-weight form")
    announce("linear instantiation", tile, M, N, K, epi, packed)
    A, W, b, ref, Ad, Wd, bd = _sweep_case(M, N, K)
    Wx = B.ssam_pack_weight(Wd) if packed else Wd
    ws = torch.empty(B.ssam_linear_workspace_bytes(), dtype=torch.uint8, device=DEV)
    if epi in (2, 3):
        rows_out = M + 13
        dst = np.random.default_rng(1).permutation(rows_out)[:M].astype(np.int32)
        x = inputs.bf16_round(np.random.default_rng(2).normal(size=(rows_out, N)).astype(np.float32))
        out = dev_bf16(x)
        B.ssam_linear_ld(Ad, Wx, bd, out, epilogue=epi, row_map=dev_i32(dst), rows_per_batch=M, map_batch_stride=0,
                         dst_rows_per_batch=rows_out, tile=tile, workspace=ws, w_packed=packed)
        got = to_np(out)
        want = ref + x[dst] if epi == 2 else ref
        assert_close(got[dst], want, f"tile{tile} epi{epi}", tol=1e-2)
        rest = np.setdiff1d(np.arange(rows_out), dst)
        assert np.array_equal(got[rest].view(np.uint32), x[rest].view(np.uint32))
    else:
        out = B.ssam_linear_ld(Ad, Wx, bd, epilogue=epi, tile=tile, workspace=ws, w_packed=packed)
        want = torch.nn.functional.gelu(torch.from_numpy(ref)).numpy() if epi == 1 else ref
        assert_close(to_np(out), want, f"tile{tile} epi{epi}", tol=1e-2)


@pytest.mark.parametrize("epi", [0, 1, 2, 3])
@pytest.mark.parametrize("tile,M,N,K", [(0, 500, 144, 576), (0, 1000, 576, 144), (3, 333, 288, 1152), (1, 700, 1160, 200),
                                        (0, 70000, 144, 576), (1, 8400, 2056, 1096), (3, 4200, 2056, 1096),
                                        (4, 8400, 2056, 1096)])
def test_linear_ragged_widths(tile, M, N, K, epi):
    """N and K that are multiples of 8 only (the stage widths of hierarchical encoders: 144, 288, 576):
    ragged last tile column and ragged last K slab, every epilogue, single, left-over and K-split launches."""
    announce("linear ragged", tile, M, N, K, epi)
    A, W, b, ref, Ad, Wd, bd = _sweep_case(M, N, K)
    ws = torch.empty(B.ssam_linear_workspace_bytes(), dtype=torch.uint8, device=DEV)
    if epi in (2, 3):
        rows_out = M + 5
        dst = np.random.default_rng(3).permutation(rows_out)[:M].astype(np.int32)
        x = inputs.bf16_round(np.random.default_rng(4).normal(size=(rows_out, N)).astype(np.float32))
        out = dev_bf16(x)
        B.ssam_linear_ld(Ad, Wd, bd, out, epilogue=epi, row_map=dev_i32(dst), rows_per_batch=M, map_batch_stride=0,
                         dst_rows_per_batch=rows_out, tile=tile, workspace=ws)
        got = to_np(out)
        want = ref + x[dst] if epi == 2 else ref
        assert_close(got[dst], want, f"ragged tile{tile} epi{epi}", tol=1e-2)
        rest = np.setdiff1d(np.arange(rows_out), dst)
        assert np.array_equal(got[rest].view(np.uint32), x[rest].view(np.uint32))
    else:
        # the result sits in a wider buffer: the columns past N must stay untouched
        buf = torch.full((M, N + 24), 3.0, dtype=torch.bfloat16, device=DEV)
        B.ssam_linear_ld(Ad, Wd, bd, buf[:, :N], epilogue=epi, tile=tile, workspace=ws)
        want = torch.nn.functional.gelu(torch.from_numpy(ref)).numpy() if epi == 1 else ref
        assert_close(to_np(buf[:, :N]), want, f"ragged tile{tile} epi{epi}", tol=1e-2)
        assert bool((buf[:, N:] == 3.0).all())


def test_linear_row_strides():
    """Operands and result as column slices of wider buffers: strides are honoured, padding untouched."""
    announce("linear strides")
    M, N, K = 700, 384, 192
    rng = np.random.default_rng(17)
    A = inputs.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    Ab = torch.full((M, K + 64), 7.0, dtype=torch.bfloat16, device=DEV)
    Wb = torch.full((N, K + 8), 7.0, dtype=torch.bfloat16, device=DEV)
    Cb = torch.full((M, N + 16), 3.0, dtype=torch.bfloat16, device=DEV)
    Ab[:, :K] = dev_bf16(A)
    Wb[:, :K] = dev_bf16(W)
    B.ssam_linear_ld(Ab[:, :K], Wb[:, :K], dev_f32(b), Cb[:, :N])
    assert_close(to_np(Cb[:, :N]), _gemm_ref(A, W, b), "linear with row strides", tol=1e-2)
    assert bool((Cb[:, N:] == 3.0).all())
    with pytest.raises(B.SsamError) as e:
        B.ssam_linear_ld(Ab[:, 4:K + 4], Wb[:, :K], dev_f32(b), Cb[:, :N])      # A not 16-byte aligned
    assert e.value.code == B.EINVAL


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
def test_linear_scatter_add(tile):
    announce("linear scatter", tile)
    rng = np.random.default_rng(6)
    B_, n, Kk, N, K = 2, 500, 210, 256, 128
    A = inputs.bf16_round(rng.normal(size=(B_ * Kk, K)).astype(np.float32))
    W = inputs.bf16_round((rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.normal(size=N).astype(np.float32)
    x = inputs.bf16_round(rng.normal(size=(B_, n, N)).astype(np.float32))
    idx = np.stack([np.sort(rng.permutation(n)[:Kk]) for _ in range(B_)]).astype(np.int32)
    idx[1, 5] = -1
    xd = dev_bf16(x)
    B.ssam_linear(dev_bf16(A), dev_bf16(W), dev_f32(b), xd, epilogue=B.EPI_BIAS_SCATTER_ADD, row_map=dev_i32(idx),
                  rows_per_batch=Kk, map_batch_stride=Kk, dst_rows_per_batch=n, tile=tile)
    got = to_np(xd)
    prod = _gemm_ref(A, W, b).reshape(B_, Kk, N)
    ref = x.astype(np.float64).copy()
    touched = np.zeros((B_, n), bool)
    for bi in range(B_):
        for j in range(Kk):
            if idx[bi, j] >= 0:
                ref[bi, idx[bi, j]] += prod[bi, j]
                touched[bi, idx[bi, j]] = True
    assert np.array_equal(got[~touched].view(np.uint32), x[~touched].view(np.uint32))   # untouched rows bit-identical
    assert_close(got[touched] - x[touched], ref[touched] - x[touched], f"scatter-add delta tile{tile}")


def test_linear_rejects_unsupported():
    A = torch.zeros((8, 64), dtype=torch.bfloat16, device=DEV)
    W = torch.zeros((100, 64), dtype=torch.bfloat16, device=DEV)          # N not a multiple of 8
    b = torch.zeros(100, device=DEV)
    with pytest.raises(B.SsamError) as e:
        B.ssam_linear(A, W, b)
    assert e.value.code == B.EUNSUPPORTED


# ------------------------------------------------------------------ LayerNorm folded into a contraction
def test_ln_fold_pieces():
    """ssam_ln_stats, ssam_fold_ln_weight and ssam_linear_ln against Linear(LN(x)) written out in fp64."""
    announce("ln fold pieces")
    rng = np.random.default_rng(70)
    M, K, N = 1024, 768, 2304
    x = inputs.bf16_round((rng.normal(size=(M, K)) * rng.uniform(0.3, 2.0, size=(M, 1)) + rng.normal(size=(M, 1))).astype(np.float32))
    W = inputs.bf16_round((0.02 * rng.normal(size=(N, K))).astype(np.float32))
    bias = (0.02 * rng.normal(size=N)).astype(np.float32)
    gamma = (1.0 + 0.3 * rng.normal(size=K)).astype(np.float32)
    beta = (0.2 * rng.normal(size=K)).astype(np.float32)
    xd, Wd = dev_bf16(x), dev_bf16(W)
    bd, gd, bed = (torch.from_numpy(a).to(DEV) for a in (bias, gamma, beta))
    x64 = x.astype(np.float64)
    mean, var = x64.mean(1), x64.var(1)
    rstd = 1.0 / np.sqrt(var + 1e-6)
    stats = B.ssam_ln_stats(xd, 1e-6)
    got = stats.cpu().numpy()
    np.testing.assert_allclose(got[:, 0], rstd, rtol=2e-6)
    np.testing.assert_allclose(got[:, 1], -rstd * mean, rtol=2e-5, atol=2e-6)
    Wf, colsum, bias_f = B.ssam_fold_ln_weight(Wd, bd, gd, bed)
    Wf_ref = inputs.bf16_round((W * gamma[None, :]).astype(np.float32))       # one fp32 product, rounded once
    assert np.array_equal(to_np(Wf), Wf_ref)
    np.testing.assert_allclose(colsum.cpu().numpy(), Wf_ref.astype(np.float64).sum(1), rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(bias_f.cpu().numpy(), bias + (W.astype(np.float64) * beta[None, :]).sum(1), rtol=1e-5, atol=1e-6)
    # rows stored through a map: two "images" of 512 rows, destination rows reversed within each image, 8 skipped
    rmap = np.tile(np.arange(511, -1, -1, dtype=np.int32), 1)
    rmap[:8] = -1
    out = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
    B.ssam_linear_ln(xd, stats, B.ssam_pack_weight(Wf), colsum, bias_f, out, dev_i32(rmap), 512, 0, 512)
    torch.cuda.synchronize()
    ref = ((x64 - mean[:, None]) * rstd[:, None] * gamma + beta) @ W.astype(np.float64).T + bias
    got = to_np(out)
    for b in range(2):
        rows = np.arange(8, 512)
        assert_close(got[b * 512 + rmap[rows]], ref[b * 512 + rows], f"folded linear image {b}")
        assert np.all(got[b * 512 + np.arange(512 - 8, 512)] == 7.0)          # skipped rows' destinations untouched


def test_fold_kv_bias():
    """ssam_fold_kv_bias against its definition in fp64."""
    announce("fold kv bias")
    rng = np.random.default_rng(71)
    D = 768
    bias_in = rng.normal(size=3 * D).astype(np.float32)
    bqkv = (0.5 * rng.normal(size=3 * D)).astype(np.float32)
    wproj = inputs.bf16_round((0.02 * rng.normal(size=(D, D))).astype(np.float32))
    bproj = (0.2 * rng.normal(size=D)).astype(np.float32)
    to_dev = lambda a: torch.from_numpy(a).to(DEV)
    bias_out, bproj_out = B.ssam_fold_kv_bias(to_dev(bias_in), to_dev(bqkv), dev_bf16(wproj), to_dev(bproj))
    ref_bias = bias_in.astype(np.float64).copy()
    ref_bias[D:] -= bqkv[D:]
    np.testing.assert_allclose(bias_out.cpu().numpy(), ref_bias, rtol=1e-6, atol=1e-6)       # the query part is untouched
    assert np.array_equal(bias_out.cpu().numpy()[:D], bias_in[:D])
    ref_proj = bproj + wproj.astype(np.float64) @ bqkv[2 * D:].astype(np.float64)
    np.testing.assert_allclose(bproj_out.cpu().numpy(), ref_proj, rtol=1e-5, atol=1e-5)
