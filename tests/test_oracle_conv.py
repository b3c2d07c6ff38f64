"""Pins for the CPU oracle's flex-conv forward and backward (CPU only)."""
import numpy as np
import pytest
from scipy.signal import correlate2d

import oracle
from helpers import (tiny_problem, dense_weights, gathered, grid2d, read_golden_kernels)
from workloads import CONFIGS, make_inputs


# ---- forward ---------------------------------------------------------------

@pytest.mark.parametrize("seed,B,N,K,Din,Dout", [(0, 2, 11, 3, 3, 2), (1, 1, 16, 4, 2, 3), (2, 3, 5, 5, 1, 1)])
def test_fwd_bruteforce_dense_weight_tensor(seed, B, N, K, Din, Dout):
    # Eq.(4) with Eq.(6), evaluated through an explicit W[b,l,k,c,o] tensor.
    pos, nbr, feat, theta, bias, _ = tiny_problem(seed, B, N, K, Din, Dout)
    W = dense_weights(pos, nbr, theta, bias)
    ref = np.einsum("blkco,blkc->bol", W, gathered(feat, nbr))
    got = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_fwd_sign_reading_neighbour_minus_centre():
    # Eq.(6) as printed uses (centre - neighbour); the reading used here
    # (neighbour - centre, Fig. 2 caption) is the same layer with theta negated.
    pos, nbr, feat, theta, bias, _ = tiny_problem(3)
    W = dense_weights(pos, nbr, -theta, bias, centre_minus_neighbour=True)
    ref = np.einsum("blkco,blkc->bol", W, gathered(feat, nbr))
    got = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
    # and the two readings really differ for this data
    W2 = dense_weights(pos, nbr, theta, bias, centre_minus_neighbour=True)
    assert np.abs(np.einsum("blkco,blkc->bol", W2, gathered(feat, nbr)) - got).max() > 1e-3


def _grid_case(H, W, h, Din, Dout, seed):
    rng = np.random.default_rng(seed)
    pos, nbr, offs = grid2d(H, W, h)
    feat = rng.standard_normal((1, Din, H * W)).astype(np.float32)
    theta = rng.standard_normal((3, Din, Dout)).astype(np.float32)
    bias = rng.standard_normal((Din, Dout)).astype(np.float32)
    return pos, nbr, offs, feat, theta, bias


def test_fwd_grid_reduces_to_2d_correlation():
    # Footnote to Eq.(4): on an image grid with the 9 fixed offsets the layer is
    # the ordinary 3x3 convolution of Eq.(1) with kernel w[tau] = <theta, h*tau> + bias.
    H, W, h, Din, Dout = 9, 12, 0.25, 3, 2
    pos, nbr, offs, feat, theta, bias = _grid_case(H, W, h, Din, Dout, 7)
    got = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)[0].reshape(Dout, H, W)
    img = feat[0].astype(np.float64).reshape(Din, H, W)
    for o in range(Dout):
        ref = np.zeros((H - 2, W - 2))
        for c in range(Din):
            kern = np.empty((3, 3))
            for (dy, dx) in offs:
                kern[dy + 1, dx + 1] = float(theta[0, c, o]) * (h * dx) + float(theta[1, c, o]) * (h * dy) + float(bias[c, o])
            ref += correlate2d(img[c], kern, mode="valid")
        np.testing.assert_allclose(got[o, 1:-1, 1:-1], ref, rtol=1e-10, atol=1e-10)


def test_fwd_grid_1d_correlation():
    n, h = 40, 0.5
    rng = np.random.default_rng(11)
    x = np.arange(n)
    pos = np.stack([x * h, np.zeros(n), np.zeros(n)], 0).astype(np.float32)[None]
    nbr = np.stack([np.clip(x + d, 0, n - 1) for d in (-1, 0, 1)], 0).astype(np.int32)[None]
    feat = rng.standard_normal((1, 1, n)).astype(np.float32)
    theta = np.array([0.7, -3.0, 5.0], np.float32).reshape(3, 1, 1)
    bias = np.array([[0.3]], np.float32)
    got = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)[0, 0]
    kern = np.array([float(theta[0, 0, 0]) * (h * d) + float(bias[0, 0]) for d in (-1, 0, 1)])
    ref = np.correlate(feat[0, 0].astype(np.float64), kern, mode="valid")
    np.testing.assert_allclose(got[1:-1], ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("name,th,b", [("prewitt_x", (1, 0, 0), 0.0), ("prewitt_y", (0, 1, 0), 0.0),
                                       ("blur", (0, 0, 0), 1.0 / 9.0)])
def test_fwd_named_image_operators(name, th, b):
    # Fig. 2: the weight theta_x (x-x0) + theta_y (y-y0) + theta_b reproduces Prewitt and Blur.
    kern = read_golden_kernels()[name]
    H, W = 8, 10
    pos, nbr, _ = grid2d(H, W, 1.0)
    rng = np.random.default_rng(5)
    feat = rng.standard_normal((1, 1, H * W)).astype(np.float32)
    theta = np.array(th, np.float32).reshape(3, 1, 1)
    bias = np.array([[b]], np.float32)
    got = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)[0, 0].reshape(H, W)
    ref = correlate2d(feat[0, 0].astype(np.float64).reshape(H, W), kern, mode="valid")
    np.testing.assert_allclose(got[1:-1, 1:-1], ref, rtol=1e-6, atol=1e-6)   # 1/9 is stored in fp32


def test_fwd_theta_zero_is_bias_weighted_neighbour_sum():
    pos, nbr, feat, theta, bias, _ = tiny_problem(4, B=2, N=20, K=4, Din=3, Dout=4)
    B, K, N = nbr.shape
    adj = np.zeros((B, N, N))
    for b in range(B):
        for k in range(K):
            for l in range(N):
                adj[b, l, nbr[b, k, l]] += 1.0
    s = np.einsum("bln,bcn->bcl", adj, feat.astype(np.float64))           # sum of neighbour features
    ref = np.einsum("co,bcl->bol", bias.astype(np.float64), s)
    got = oracle.flexconv_fwd(feat, pos, nbr, np.zeros_like(theta), bias)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_fwd_translation_invariance_exact():
    # Sec. 3.1: the weight depends on position differences only.  Dyadic
    # coordinates and a dyadic shift keep the float32 inputs exact.
    rng = np.random.default_rng(9)
    B, N, K, Din, Dout = 1, 30, 5, 2, 3
    pos = (rng.integers(-64, 64, size=(B, 3, N)) / 16.0).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    feat = rng.standard_normal((B, Din, N)).astype(np.float32)
    theta = rng.standard_normal((3, Din, Dout)).astype(np.float32)
    bias = rng.standard_normal((Din, Dout)).astype(np.float32)
    a = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    shift = np.array([8.0, -4.5, 2.25], np.float32).reshape(1, 3, 1)
    b = oracle.flexconv_fwd(feat, pos + shift, nbr, theta, bias)
    assert np.array_equal(a, b)


def test_fwd_slot_permutation_and_relabelling():
    pos, nbr, feat, theta, bias, _ = tiny_problem(12, B=1, N=17, K=4, Din=2, Dout=2)
    a = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    b = oracle.flexconv_fwd(feat, pos, nbr[:, ::-1, :], theta, bias)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-13)
    perm = np.random.default_rng(0).permutation(17)          # new label of old point i is inv[i]
    inv = np.argsort(perm)
    pos2, feat2 = pos[:, :, perm], feat[:, :, perm]
    nbr2 = inv[nbr[:, :, perm]].astype(np.int32)
    c = oracle.flexconv_fwd(feat2, pos2, nbr2, theta, bias)
    np.testing.assert_allclose(c, a[:, :, perm], rtol=1e-13, atol=1e-13)


def test_fwd_factored_form_matches_direct():
    # The weight is linear in the position difference, so the neighbour sum
    # factors into a per-point (4*Din) aggregate times a (4*Din x Dout) matrix.
    x = make_inputs(CONFIGS[0], n_override=512)
    got = oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias)
    F = gathered(x.feat, x.nbr)                                        # [B,N,K,C]
    pos = x.pos.astype(np.float64)
    bi = np.arange(x.cfg.B)[:, None, None]
    dp = pos[bi, :, x.nbr.transpose(0, 2, 1)] - pos.transpose(0, 2, 1)[:, :, None, :]   # [B,N,K,3]
    A = np.concatenate([np.einsum("blkd,blkc->bldc", dp, F), F.sum(2)[:, :, None, :]], 2)  # [B,N,4,C]
    Theta = np.concatenate([x.theta, x.bias[None]], 0).astype(np.float64)                   # [4,C,O]
    ref = np.einsum("bljc,jco->bol", A, Theta)
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_fwd_range_argument_returns_its_columns():
    pos, nbr, feat, theta, bias, _ = tiny_problem(13, B=2, N=19)
    full = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    part = oracle.flexconv_fwd(feat, pos, nbr, theta, bias, l_range=(5, 12))
    assert part.shape == (2, full.shape[1], 7)
    assert np.array_equal(part, full[:, :, 5:12])


# ---- backward --------------------------------------------------------------

def test_bwd_bruteforce_dense():
    pos, nbr, feat, theta, bias, g = tiny_problem(21, B=2, N=9, K=3, Din=3, Dout=2)
    B, K, N = nbr.shape
    W = dense_weights(pos, nbr, theta, bias)
    F = gathered(feat, nbr)
    g64 = g.astype(np.float64)
    gf_ref = np.zeros((B, feat.shape[1], N))
    contrib = np.einsum("blkco,bol->blkc", W, g64)
    for b in range(B):
        for l in range(N):
            for k in range(K):
                gf_ref[b, :, nbr[b, k, l]] += contrib[b, l, k]
    pos64 = pos.astype(np.float64)
    bi = np.arange(B)[:, None, None]
    dp = pos64[bi, :, nbr.transpose(0, 2, 1)] - pos64.transpose(0, 2, 1)[:, :, None, :]
    gt_ref = np.einsum("blkd,blkc,bol->dco", dp, F, g64)
    gb_ref = np.einsum("blkc,bol->co", F, g64)
    gf, gt, gb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    np.testing.assert_allclose(gf, gf_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gt, gt_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gb, gb_ref, rtol=1e-12, atol=1e-12)


def test_bwd_finite_differences_full_jacobian():
    # The forward map is bilinear in (feat, [theta;bias]), so central differences
    # are exact up to rounding for any step.
    pos, nbr, feat, theta, bias, g = tiny_problem(22, B=1, N=7, K=3, Din=2, Dout=2)
    g64 = g.astype(np.float64)
    gf, gt, gb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)

    def loss(f, t, b):
        return float((oracle.flexconv_fwd(f, pos, nbr, t, b) * g64).sum())

    step = np.float32(0.5)
    for arr, grad, which in ((feat, gf, 0), (theta, gt, 1), (bias, gb, 2)):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            plus, minus = arr.copy(), arr.copy()
            plus[i] += step
            minus[i] -= step
            args_p = [feat, theta, bias]
            args_m = [feat, theta, bias]
            args_p[which], args_m[which] = plus, minus
            fd = (loss(*args_p) - loss(*args_m)) / (float(plus[i]) - float(minus[i]))
            assert abs(fd - grad[i]) <= 1e-9 * max(1.0, abs(grad[i])), (which, i, fd, grad[i])


def test_bwd_adjoint_identities_cfg0():
    # <g, fwd(v; Theta)> = <grad_feat(g), v>  and  <g, fwd(feat; dTheta)> = <grad_Theta(g), dTheta>
    x = make_inputs(CONFIGS[0])
    rng = np.random.default_rng(77)
    gf, gt, gb = oracle.flexconv_bwd(x.feat, x.pos, x.nbr, x.theta, x.bias, x.grad_out)
    g64 = x.grad_out.astype(np.float64)
    v = rng.standard_normal(x.feat.shape).astype(np.float32)
    lhs = (oracle.flexconv_fwd(v, x.pos, x.nbr, x.theta, x.bias) * g64).sum()
    rhs = (gf * v.astype(np.float64)).sum()
    assert abs(lhs - rhs) <= 1e-10 * abs(lhs)
    dth = rng.standard_normal(x.theta.shape).astype(np.float32)
    db = rng.standard_normal(x.bias.shape).astype(np.float32)
    lhs = (oracle.flexconv_fwd(x.feat, x.pos, x.nbr, dth, db) * g64).sum()
    rhs = (gt * dth.astype(np.float64)).sum() + (gb * db.astype(np.float64)).sum()
    assert abs(lhs - rhs) <= 1e-10 * abs(lhs)


def test_bwd_bias_gradient_is_adjacency_feat_transpose_g():
    pos, nbr, feat, theta, bias, g = tiny_problem(23, B=2, N=13, K=4, Din=3, Dout=2)
    s = gathered(feat, nbr).sum(2)                         # [B,N,C] neighbour-feature sums
    ref = np.einsum("blc,bol->co", s, g.astype(np.float64))
    _, _, gb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    np.testing.assert_allclose(gb, ref, rtol=1e-12, atol=1e-12)


def test_bwd_grad_feat_at_matches_full():
    x = make_inputs(CONFIGS[0], n_override=700)
    gf, _, _ = oracle.flexconv_bwd(x.feat, x.pos, x.nbr, x.theta, x.bias, x.grad_out, want_params=False)
    targets = np.random.default_rng(1).choice(700, size=50, replace=False).astype(np.int64)
    rows = oracle.flexconv_grad_feat_at(x.pos, x.nbr, x.theta, x.bias, x.grad_out, targets)
    np.testing.assert_allclose(rows, gf[0][:, targets].T, rtol=1e-12, atol=1e-12)


def test_bwd_ranges_add_up():
    pos, nbr, feat, theta, bias, g = tiny_problem(24, B=2, N=15)
    full = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    a = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g, l_range=(0, 6))
    b = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g, l_range=(6, 15))
    for f, p, q in zip(full, a, b):
        np.testing.assert_allclose(f, p + q, rtol=1e-12, atol=1e-12)


# ---- gradient with respect to the point locations ---------------------------------------
def test_bwd_pos_finite_differences():
    # out is affine in pos, so a central difference of <g, fwd(pos)> is exact up to rounding
    pos, nbr, feat, theta, bias, g = tiny_problem(21, B=2, N=9, K=4, Din=3, Dout=2, self_first=True)
    gp = oracle.flexconv_bwd_pos(feat, nbr, theta, g)
    g64 = g.astype(np.float64)
    h = 0.25                                   # exactly representable steps on top of float32 inputs
    for b in range(2):
        for d in range(3):
            for m in range(9):
                pp, pm = pos.astype(np.float64).copy(), pos.astype(np.float64).copy()
                pp[b, d, m] += h
                pm[b, d, m] -= h
                # the oracle takes float32 positions: evaluate the definition in numpy on the float64 copies
                fd = (np.sum(g64 * _fwd_numpy(feat, pp, nbr, theta, bias)) - np.sum(g64 * _fwd_numpy(feat, pm, nbr, theta, bias))) / (2 * h)
                assert abs(gp[b, d, m] - fd) <= 1e-9 * max(1.0, abs(fd))


def _fwd_numpy(feat, pos64, nbr, theta, bias):
    W = dense_weights_f64(pos64, nbr, theta, bias)
    return np.einsum("blkco,blkc->bol", W, gathered(feat, nbr))


def dense_weights_f64(pos64, nbr, theta, bias):
    B, K, N = nbr.shape
    bi = np.arange(B)[:, None, None]
    pn = pos64[bi, :, nbr.transpose(0, 2, 1)]
    pl = pos64.transpose(0, 2, 1)[:, :, None, :]
    return np.einsum("dco,blkd->blkco", theta.astype(np.float64), pn - pl) + bias.astype(np.float64)


def test_bwd_pos_bruteforce_translation_and_self_edges():
    pos, nbr, feat, theta, bias, g = tiny_problem(22, B=2, N=12, K=3, Din=2, Dout=3)
    gp = oracle.flexconv_bwd_pos(feat, nbr, theta, g)
    # brute force: s[b,l,k,d] scattered with +/- signs
    F = gathered(feat, nbr)                                                  # [B,N,K,Din]
    s = np.einsum("dco,blkc,bol->blkd", theta.astype(np.float64), F, g.astype(np.float64))
    want = np.zeros_like(gp)
    for b in range(2):
        for l in range(12):
            for k in range(3):
                want[b, :, nbr[b, k, l]] += s[b, l, k]
                want[b, :, l] -= s[b, l, k]
    assert np.allclose(gp, want, rtol=0, atol=1e-12)
    # translation invariance of the layer: the location gradients of a cloud sum to zero
    assert np.abs(gp.sum(axis=2)).max() <= 1e-12 * max(1.0, np.abs(gp).max())
    # neighbourhoods made of the centre alone: no dependence on the locations at all
    self_only = np.broadcast_to(np.arange(12, dtype=np.int32), nbr.shape).copy()
    assert np.abs(oracle.flexconv_bwd_pos(feat, self_only, theta, g)).max() == 0.0
    # the gradient does not involve the bias nor the locations themselves (the map is affine in pos)
    assert np.array_equal(gp, oracle.flexconv_bwd_pos(feat, nbr, theta, g))
