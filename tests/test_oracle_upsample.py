"""Pins for the CPU oracle's flex-upsampling forward and backward (CPU only).

Flex-upsampling (Sec. 4.1) = copy the selected points' features into the larger layer, zero
elsewhere, then flex-max-pool.  The pins: brute force on tiny clouds, the composition
zero-fill (numpy) + pooling oracle (pinned on its own), the identity selection, zero-insertion
upsampling of an image followed by a 3x3 stride-1 max filter, and the backward pass against
brute force, mass conservation and the pooling oracle's backward gathered at the selection."""
import numpy as np
import pytest
from scipy.ndimage import maximum_filter

import oracle
from helpers import grid2d


def _problem(seed, B=2, C=3, Nf=29, Ns=9, K=5, ties=True):
    rng = np.random.default_rng(seed)
    feat = (rng.integers(-2, 3, size=(B, C, Ns)) if ties else rng.standard_normal((B, C, Ns))).astype(np.float32)
    sel = np.stack([rng.permutation(Nf)[:Ns] for _ in range(B)]).astype(np.int32)
    nbr = rng.integers(0, Nf, size=(B, K, Nf)).astype(np.int32)
    g = rng.standard_normal((B, C, Nf)).astype(np.float32)
    return feat, sel, nbr, g


def _zero_filled(feat, sel, Nf):
    B, C, Ns = feat.shape
    dense = np.zeros((B, C, Nf), np.float32)
    for b in range(B):
        dense[b][:, sel[b]] = feat[b]
    return dense


def _brute(feat, sel, nbr):
    B, C, Ns = feat.shape
    _, K, Nf = nbr.shape
    out = np.empty((B, C, Nf), np.float32)
    arg = np.empty((B, C, Nf), np.int32)
    for b in range(B):
        where = {int(m): j for j, m in enumerate(sel[b])}
        for l in range(Nf):
            for c in range(C):
                cand = [(float(feat[b, c, where[int(n)]]) if int(n) in where else 0.0, int(n)) for n in nbr[b, :, l]]
                top = max(v for v, _ in cand)
                arg[b, c, l] = min(n for v, n in cand if v == top)
                m = arg[b, c, l]
                out[b, c, l] = feat[b, c, where[m]] if m in where else 0.0
    return out, arg


def test_upsample_fwd_bruteforce_with_ties():
    feat, sel, nbr, _ = _problem(0)
    feat[0, 0, :2] = [-0.0, 0.0]
    out, arg = oracle.flexupsample_fwd(feat, sel, nbr)
    ro, ra = _brute(feat, sel, nbr)
    assert np.array_equal(arg, ra)
    assert np.array_equal(out.view(np.uint32), ro.view(np.uint32))


def test_upsample_fwd_is_zero_fill_then_pool():
    feat, sel, nbr, _ = _problem(1, B=3, C=4, Nf=64, Ns=16, K=8, ties=False)
    out, arg = oracle.flexupsample_fwd(feat, sel, nbr)
    po, pa = oracle.flexpool_fwd(_zero_filled(feat, sel, 64), nbr)
    assert np.array_equal(arg, pa)
    assert np.array_equal(out.view(np.uint32), po.view(np.uint32))
    # ranged call = its columns
    o2, a2 = oracle.flexupsample_fwd(feat, sel, nbr, l_range=(10, 37))
    assert np.array_equal(o2, out[:, :, 10:37]) and np.array_equal(a2, arg[:, :, 10:37])


def test_upsample_identity_selection_is_pooling():
    rng = np.random.default_rng(2)
    B, C, N, K = 2, 3, 40, 6
    feat = rng.standard_normal((B, C, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    sel = np.broadcast_to(np.arange(N, dtype=np.int32), (B, N)).copy()
    out, arg = oracle.flexupsample_fwd(feat, sel, nbr)
    po, pa = oracle.flexpool_fwd(feat, nbr)
    assert np.array_equal(arg, pa) and np.array_equal(out, po)
    # a permuted selection of all points only relabels the smaller layer
    perm = rng.permutation(N).astype(np.int32)
    o3, a3 = oracle.flexupsample_fwd(feat[:, :, perm], np.broadcast_to(perm, (B, N)).copy(), nbr)
    assert np.array_equal(a3, pa) and np.array_equal(o3, po)


def test_upsample_grid_is_zero_insertion_then_3x3_max():
    h, w = 7, 9
    H, W = 2 * h, 2 * w
    rng = np.random.default_rng(3)
    img = rng.standard_normal((2, h, w)).astype(np.float32)            # 2 channels
    _, nbr, _ = grid2d(H, W, 1.0)
    ys, xs = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    sel = ((2 * ys) * W + 2 * xs).ravel().astype(np.int32)[None]
    out, _ = oracle.flexupsample_fwd(img.reshape(1, 2, h * w), sel, nbr)
    big = np.zeros((2, H, W), np.float32)
    big[:, ::2, ::2] = img
    want = np.stack([maximum_filter(big[c], size=3, mode="nearest") for c in range(2)])
    got = out.reshape(2, H, W)
    assert np.array_equal(got[:, 1:-1, 1:-1], want[:, 1:-1, 1:-1])


def test_upsample_rejects_bad_selection():
    feat, sel, nbr, _ = _problem(4)
    bad = sel.copy(); bad[0, 1] = bad[0, 0]
    with pytest.raises(RuntimeError):
        oracle.flexupsample_fwd(feat, bad, nbr)
    bad = sel.copy(); bad[1, 0] = nbr.shape[2]
    with pytest.raises(RuntimeError):
        oracle.flexupsample_fwd(feat, bad, nbr)


def test_upsample_bwd_bruteforce_mass_and_composition():
    feat, sel, nbr, g = _problem(5, B=2, C=3, Nf=31, Ns=11, K=4)
    _, arg = oracle.flexupsample_fwd(feat, sel, nbr)
    gs = oracle.flexupsample_bwd(g, arg, sel)
    B, C, Ns = feat.shape
    want = np.zeros((B, C, Ns))
    for b in range(B):
        for j in range(Ns):
            for c in range(C):
                want[b, c, j] = g[b, c][arg[b, c] == sel[b, j]].astype(np.float64).sum()
    assert np.allclose(gs, want, rtol=0, atol=1e-12)
    # mass: exactly the gradient of the centres whose winner is a selected point arrives
    for b in range(B):
        chosen = np.isin(arg[b], sel[b])
        assert np.allclose(gs[b].sum(axis=1), (g[b].astype(np.float64) * chosen).sum(axis=1), atol=1e-12)
    # composition: pooling backward on the larger layer, read at the selection
    dense_grad = oracle.flexpool_bwd(g, arg)
    for b in range(B):
        assert np.allclose(gs[b], dense_grad[b][:, sel[b]], atol=1e-12)


def test_upsample_bwd_is_adjoint_of_the_selection_map():
    # with the winners frozen, out = S(feat) is linear: <g, S(v)> == <S^T g, v>
    feat, sel, nbr, g = _problem(6, B=1, C=2, Nf=37, Ns=13, K=5, ties=False)
    _, arg = oracle.flexupsample_fwd(feat, sel, nbr)
    rng = np.random.default_rng(7)
    v = rng.standard_normal(feat.shape).astype(np.float32)
    dense_v = _zero_filled(v, sel, 37)
    Sv = np.take_along_axis(dense_v, arg.astype(np.int64), axis=2)
    lhs = float((g.astype(np.float64) * Sv).sum())
    rhs = float((oracle.flexupsample_bwd(g, arg, sel) * v).sum())
    assert abs(lhs - rhs) <= 1e-9 * max(1.0, abs(lhs))
