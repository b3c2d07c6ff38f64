"""Pins for the CPU oracle's flex-max-pooling with subsampling (Sec. 4.1 / Sec. 4.3), CPU only."""
import numpy as np
from scipy.ndimage import maximum_filter

import oracle
from helpers import grid2d


def _case(seed, B=2, C=3, N=37, K=5, Ns=11, ties=False):
    rng = np.random.default_rng(seed)
    if ties:
        feat = rng.integers(-2, 3, size=(B, C, N)).astype(np.float32)
    else:
        feat = rng.standard_normal((B, C, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    sel = np.stack([rng.permutation(N)[:Ns] for _ in range(B)]).astype(np.int32)
    g = rng.standard_normal((B, C, Ns)).astype(np.float32)
    return feat, nbr, sel, g


def test_pool_sub_fwd_bruteforce_with_ties():
    feat, nbr, sel, _ = _case(0, ties=True)
    B, C, N = feat.shape
    Ns = sel.shape[1]
    out, arg = oracle.flexpool_sub_fwd(feat, nbr, sel)
    for b in range(B):
        for j in range(Ns):
            ns = nbr[b, :, sel[b, j]]
            for c in range(C):
                vals = feat[b, c, ns]
                w = ns[vals == vals.max()].min()          # lowest point index among the maxima
                assert arg[b, c, j] == w
                assert out[b, c, j].view(np.uint32) == feat[b, c, w].view(np.uint32)


def test_pool_sub_fwd_grid_is_3x3_maxpool_stride2():
    # On a regular grid with the 3x3 offsets, keeping every second row and column is the ordinary
    # stride-2 max-pooling of image networks (Sec. 4.3 compares the layer with exactly that).
    H, W = 12, 14
    _, nbr, _ = grid2d(H, W, 1.0)
    rng = np.random.default_rng(1)
    feat = rng.standard_normal((1, 2, H * W)).astype(np.float32)
    ys, xs = np.meshgrid(np.arange(1, H - 1, 2), np.arange(1, W - 1, 2), indexing="ij")
    sel = (ys * W + xs).ravel().astype(np.int32)[None]
    out, arg = oracle.flexpool_sub_fwd(feat, nbr, sel)
    for c in range(2):
        ref = maximum_filter(feat[0, c].reshape(H, W), size=3, mode="nearest")[1:H - 1:2, 1:W - 1:2]
        assert np.array_equal(out[0, c].reshape(ref.shape), ref)
    assert np.array_equal(feat[0, 0][arg[0, 0]], out[0, 0])


def test_pool_sub_fwd_identity_selection_and_k1():
    feat, nbr, _, _ = _case(2)
    B, C, N = feat.shape
    ident = np.tile(np.arange(N, dtype=np.int32), (B, 1))
    out, arg = oracle.flexpool_sub_fwd(feat, nbr, ident)
    # every point kept: nothing but pooling is left; K = 1 with self neighbours: a plain row selection
    bi = np.arange(B)[:, None, None]
    ci = np.arange(C)[None, :, None]
    assert np.array_equal(out, feat[bi, ci, arg])
    assert (out >= np.take_along_axis(feat, np.broadcast_to(nbr[:, :1, :], (B, C, N)).astype(np.int64), 2)).all()
    self_only = ident[:, None, :].copy()
    sel = np.stack([np.random.default_rng(3 + b).permutation(N)[:9] for b in range(B)]).astype(np.int32)
    o2, a2 = oracle.flexpool_sub_fwd(feat, self_only, sel)
    assert np.array_equal(o2, np.take_along_axis(feat, np.broadcast_to(sel[:, None, :], (B, C, 9)).astype(np.int64), 2))
    assert np.array_equal(a2, np.broadcast_to(sel[:, None, :], (B, C, 9)))


def test_pool_sub_bwd_bruteforce_mass_and_repeats():
    feat, nbr, sel, g = _case(4, ties=True)
    B, C, N = feat.shape
    Ns = sel.shape[1]
    _, arg = oracle.flexpool_sub_fwd(feat, nbr, sel)
    gf = oracle.flexpool_sub_bwd(g, arg, sel, N)
    ref = np.zeros((B, C, N))
    for b in range(B):
        for c in range(C):
            for j in range(Ns):
                ref[b, c, arg[b, c, j]] += float(g[b, c, j])
    np.testing.assert_allclose(gf, ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gf.sum(2), g.astype(np.float64).sum(2), rtol=1e-12, atol=1e-12)


def test_pool_sub_bwd_is_directional_derivative():
    # Without ties the layer is linear around the input: d/dt sum(g * pool_sub(feat + t*d)) at t = 0
    # must equal <grad_feat, d>; a central difference with a step far below the value gaps is exact
    # up to rounding.
    feat, nbr, sel, g = _case(5, B=1, C=2, N=41, K=4, Ns=13)
    N = feat.shape[2]
    _, arg = oracle.flexpool_sub_fwd(feat, nbr, sel)
    gf = oracle.flexpool_sub_bwd(g, arg, sel, N)
    rng = np.random.default_rng(6)
    d = rng.standard_normal(feat.shape).astype(np.float32)
    t = np.float32(2.0 ** -12)
    op, ap = oracle.flexpool_sub_fwd(feat + t * d, nbr, sel)
    om, am = oracle.flexpool_sub_fwd(feat - t * d, nbr, sel)
    assert np.array_equal(ap, arg) and np.array_equal(am, arg)       # the step crossed no tie
    fd = ((op.astype(np.float64) - om.astype(np.float64)) * g.astype(np.float64)).sum() / (2.0 * float(t))
    an = (gf * d.astype(np.float64)).sum()
    assert abs(fd - an) <= 2e-4 * max(1.0, abs(an))


def test_pool_sub_matches_pool_then_select():
    # the two pooling oracles are separate code; restricted to the kept columns they must agree,
    # forward and backward (backward: the kept columns' gradients, zero for the dropped ones)
    feat, nbr, sel, g = _case(7, ties=True)
    B, C, N = feat.shape
    Ns = sel.shape[1]
    fo, fa = oracle.flexpool_fwd(feat, nbr)
    so, sa = oracle.flexpool_sub_fwd(feat, nbr, sel)
    idx = np.broadcast_to(sel[:, None, :], (B, C, Ns)).astype(np.int64)
    assert np.array_equal(so, np.take_along_axis(fo, idx, 2)) and np.array_equal(sa, np.take_along_axis(fa, idx, 2))
    gfull = np.zeros((B, C, N), np.float32)
    np.put_along_axis(gfull, idx, g, 2)
    np.testing.assert_allclose(oracle.flexpool_sub_bwd(g, sa, sel, N), oracle.flexpool_bwd(gfull, fa),
                               rtol=1e-13, atol=1e-13)
