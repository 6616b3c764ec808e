"""CPU-side checks of the HIP library: it loads, exports every symbol the header
declares, its host-side integer builders match the oracle bit for bit, and bad
arguments come back as error codes.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_17633_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ssam.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ssam_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = declared_symbols()
    assert len(syms) >= 20
    L = B.lib()
    for s in syms:
        assert hasattr(L, s), f"libssam.so does not export {s}"


def test_python_binding_has_the_same_names():
    skip = {"ssam_status_string", "ssam_score_tokens_workspace_bytes", "ssam_linear_tiled"}
    for s in declared_symbols():
        if s in skip:
            continue
        assert hasattr(B, s), f"binding lacks {s}"


@pytest.mark.parametrize("gh,gw,G", [(14, 14, 4), (28, 28, 4), (64, 64, 4), (70, 70, 4), (14, 14, 1), (5, 9, 1), (6, 4, 2)])
def test_build_perm_matches_oracle(gh, gw, G):
    perm, inv = B.ssam_build_perm(gh, gw, G)
    sigma, sinv = oracle.stripe_sort(oracle.morton_order(gh, gw), G)
    assert np.array_equal(perm, sigma) and np.array_equal(inv, sinv)


@pytest.mark.parametrize("g,ws", [(64, 14), (28, 14), (16, 6)])
def test_window_table_matches_oracle(g, ws):
    assert np.array_equal(B.ssam_build_window_table(g, ws, 4), oracle.window_table(g, ws, 4))


@pytest.mark.parametrize("S,Bm", [(196, 32), (4096, 128), (784, 128), (64, 32)])
@pytest.mark.parametrize("r", [0.2, 0.25, 0.3, 0.4, 0.5, 0.6, 1.0])
def test_block_mask_matches_oracle(S, Bm, r):
    row_ptr, col_idx, n_pre = B.ssam_build_block_mask(S, Bm, r)
    m, n_pre_o = oracle.block_mask(S, Bm, r)
    T = m.shape[0]
    dense = np.zeros((T, T), np.uint8)
    for i in range(T):
        cols = col_idx[row_ptr[i]:row_ptr[i + 1]]
        assert np.all(np.diff(cols) > 0)
        dense[i, cols] = 1
    assert n_pre == n_pre_o and np.array_equal(dense, m)


def test_keep_count_matches_oracle():
    for n in (784, 4096, 10):
        for rho in (0.01, 0.2, 0.3, 0.4, 0.6, 1.0):
            assert B.ssam_keep_count(n, rho) == oracle.keep_count(n, rho)


def test_error_codes():
    L = B.lib()
    buf = (C.c_int32 * 16)()
    assert L.ssam_build_perm(3, 3, 4, buf, None) == B.EINVAL           # 9 cells not divisible by 4
    assert L.ssam_build_perm(0, 3, 1, buf, None) == B.EINVAL
    assert L.ssam_build_perm(2, 2, 1, None, None) == B.EINVAL
    assert L.ssam_build_block_mask(196, 32, C.c_double(0.0), buf, buf, None) == B.EINVAL
    assert L.ssam_build_block_mask(196, 32, C.c_double(1.5), buf, buf, None) == B.EINVAL
    assert L.ssam_keep_count(10, C.c_double(0.0)) == B.EINVAL
    # null pointers / bad sizes are rejected before anything is enqueued
    assert L.ssam_permute(None, None, None, 1, 1, 1, 8, None) == B.EINVAL
    assert L.ssam_linear(None, None, None, None, 1, 128, 64, 0, None, 1, 0, 1, None) == B.EINVAL
    assert L.ssam_select_tokens(None, None, 1, 8, 4, None) == B.EINVAL
    assert L.ssam_build_content_tables(None, 1, 8, 4, 4, None, None, None) == B.EINVAL
    assert L.ssam_pack_weight(None, 64, None, 32, 64, None) == B.EINVAL
    assert L.ssam_routed_mlp_folded(None, None, C.c_float(1e-6), None, None, None, None, None, 1, 64, 128, 256, 16,
                                    None, C.c_size_t(0), None) == B.EINVAL
    assert L.ssam_probe_mfma(0, 4, 10, None, None) == B.EINVAL and L.ssam_probe_mfma(2, 4, 10, buf, None) == B.EINVAL
    assert B.ssam_probe_mfma_flops(2, 3) == 2 * 4 * 3 * 8 * 2.0 * 32 * 32 * 16
    assert L.ssam_sparse_attention(None, None, None, C.c_long(0), None, None, None, C.c_long(0), None, None,
                                   1, 196, 14, 1, 64, 32, C.c_double(0.4), C.c_float(1.0), None) == B.EINVAL
    assert B.status_string(B.EUNSUPPORTED) == "unsupported shape"
    cfg = B.make_cfg(1, 28, 768, 12, 3072, 14, 32, 313, 0.4)
    assert B.ssam_encoder_block_workspace_bytes(cfg) > 0
    assert L.ssam_encoder_block(None, None, C.byref(cfg), None, None, None, None, C.c_size_t(0), None) == B.EINVAL
