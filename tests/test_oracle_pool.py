"""Pins for the CPU oracle's flex-max-pool forward and backward (CPU only)."""
import numpy as np
from scipy.ndimage import maximum_filter

import oracle
from helpers import grid2d


def _brute_pool(feat, nbr):
    B, C, N = feat.shape
    K = nbr.shape[1]
    out = np.empty((B, C, N), np.float32)
    arg = np.empty((B, C, N), np.int32)
    for b in range(B):
        for l in range(N):
            ns = nbr[b, :, l]
            for c in range(C):
                vals = feat[b, c, ns]
                m = vals.max()
                winners = ns[vals == m]
                arg[b, c, l] = winners.min()          # lowest point index among the maxima
                out[b, c, l] = feat[b, c, arg[b, c, l]]
    return out, arg


def test_pool_fwd_bruteforce_with_ties():
    rng = np.random.default_rng(0)
    B, C, N, K = 2, 3, 23, 5
    feat = rng.integers(-2, 3, size=(B, C, N)).astype(np.float32)   # many ties
    feat[0, 0, :4] = [0.0, -0.0, 0.0, -0.0]                          # signed zeros tie
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    out, arg = oracle.flexpool_fwd(feat, nbr)
    ro, ra = _brute_pool(feat, nbr)
    assert np.array_equal(arg, ra)
    assert np.array_equal(out.view(np.uint32), ro.view(np.uint32))


def test_pool_fwd_invariants():
    rng = np.random.default_rng(1)
    B, C, N, K = 2, 4, 50, 6
    feat = rng.standard_normal((B, C, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    nbr[:, 0, :] = np.arange(N)
    out, arg = oracle.flexpool_fwd(feat, nbr)
    bi = np.arange(B)[:, None, None]
    ci = np.arange(C)[None, :, None]
    assert np.array_equal(out, feat[bi, ci, arg])                    # value is the winner's
    assert (out >= feat).all()                                       # self is a neighbour
    assert all((arg[b, c, l] in nbr[b, :, l]) for b in range(B) for c in range(C) for l in range(N))
    # slot order must not matter (this is what fixes the tie rule to point index)
    perm = rng.permutation(K)
    out2, arg2 = oracle.flexpool_fwd(feat, nbr[:, perm, :])
    assert np.array_equal(out, out2) and np.array_equal(arg, arg2)


def test_pool_fwd_k1_identity_and_constant_feature():
    N = 12
    rng = np.random.default_rng(2)
    feat = rng.standard_normal((1, 2, N)).astype(np.float32)
    self_only = np.arange(N, dtype=np.int32).reshape(1, 1, N)
    out, arg = oracle.flexpool_fwd(feat, self_only)
    assert np.array_equal(out, feat) and np.array_equal(arg[0, 0], np.arange(N))
    nbr = rng.integers(0, N, size=(1, 4, N)).astype(np.int32)
    out, arg = oracle.flexpool_fwd(np.full((1, 2, N), 3.5, np.float32), nbr)
    assert np.array_equal(arg[0, 0], nbr[0].min(0)) and (out == 3.5).all()


def test_pool_fwd_grid_is_3x3_maxpool_stride1():
    # Sec. 4.1: like grid max-pooling but without subsampling.
    H, W = 9, 11
    _, nbr, _ = grid2d(H, W, 1.0)
    rng = np.random.default_rng(3)
    feat = rng.standard_normal((1, 2, H * W)).astype(np.float32)
    out, _ = oracle.flexpool_fwd(feat, nbr)
    for c in range(2):
        ref = maximum_filter(feat[0, c].reshape(H, W), size=3, mode="nearest")
        assert np.array_equal(out[0, c].reshape(H, W)[1:-1, 1:-1], ref[1:-1, 1:-1])


def test_pool_bwd_bruteforce_and_mass():
    rng = np.random.default_rng(4)
    B, C, N, K = 2, 3, 31, 4
    feat = rng.integers(-1, 2, size=(B, C, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    g = rng.standard_normal((B, C, N)).astype(np.float32)
    _, arg = oracle.flexpool_fwd(feat, nbr)
    gf = oracle.flexpool_bwd(g, arg)
    ref = np.zeros((B, C, N))
    for b in range(B):
        for c in range(C):
            for l in range(N):
                ref[b, c, arg[b, c, l]] += float(g[b, c, l])
    np.testing.assert_allclose(gf, ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gf.sum(2), g.astype(np.float64).sum(2), rtol=1e-12, atol=1e-12)
    hit = np.zeros((B, C, N), bool)
    bi = np.arange(B)[:, None, None]
    ci = np.arange(C)[None, :, None]
    hit[bi, ci, arg] = True
    assert not gf[~hit].any()                                        # support within the argmax image


def test_pool_bwd_is_adjoint_of_selection():
    # With the winners fixed, pooling is the linear selection S; bwd must be S^T.
    rng = np.random.default_rng(5)
    B, C, N, K = 1, 2, 40, 5
    feat = rng.standard_normal((B, C, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    g = rng.standard_normal((B, C, N)).astype(np.float32)
    out, arg = oracle.flexpool_fwd(feat, nbr)
    gf = oracle.flexpool_bwd(g, arg)
    lhs = (out.astype(np.float64) * g.astype(np.float64)).sum()
    rhs = (gf * feat.astype(np.float64)).sum()
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_pool_range_arguments():
    rng = np.random.default_rng(6)
    B, C, N, K = 2, 3, 29, 4
    feat = rng.standard_normal((B, C, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    g = rng.standard_normal((B, C, N)).astype(np.float32)
    out, arg = oracle.flexpool_fwd(feat, nbr)
    po, pa = oracle.flexpool_fwd(feat, nbr, l_range=(7, 19))
    assert np.array_equal(po, out[:, :, 7:19]) and np.array_equal(pa, arg[:, :, 7:19])
    full = oracle.flexpool_bwd(g, arg)
    parts = oracle.flexpool_bwd(g, arg, l_range=(0, 7)) + oracle.flexpool_bwd(g, arg, l_range=(7, N))
    np.testing.assert_allclose(parts, full, rtol=1e-13, atol=1e-13)
