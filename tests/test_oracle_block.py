"""Pins for the CPU oracle's 1x1-convolution + flex-convolution block (Sec. 4.3), CPU only."""
import numpy as np

import oracle


def _case(seed, B=2, N=19, K=4, Din0=3, Dmid=4, Dout=2):
    rng = np.random.default_rng(seed)
    feat = rng.standard_normal((B, Din0, N)).astype(np.float32)
    pos = rng.random((B, 3, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    nbr[:, 0, :] = np.arange(N)
    W = rng.standard_normal((Dmid, Din0)).astype(np.float32)
    theta = rng.standard_normal((3, Dmid, Dout)).astype(np.float32)
    bias = rng.standard_normal((Dmid, Dout)).astype(np.float32)
    g = rng.standard_normal((B, Dout, N)).astype(np.float32)
    return feat, pos, nbr, W, theta, bias, g


def test_block_fwd_bruteforce_dense():
    feat, pos, nbr, W, theta, bias, _ = _case(0)
    B, Din0, N = feat.shape
    K = nbr.shape[1]
    out = oracle.block_fwd(feat, pos, nbr, W, theta, bias)
    f64, p64 = feat.astype(np.float64), pos.astype(np.float64)
    mid = np.einsum("ce,ben->bcn", W.astype(np.float64), f64)
    ref = np.zeros_like(out)
    for b in range(B):
        for l in range(N):
            for k in range(K):
                n = nbr[b, k, l]
                dp = p64[b, :, n] - p64[b, :, l]
                w = np.einsum("dco,d->co", theta.astype(np.float64), dp) + bias.astype(np.float64)
                ref[b, :, l] += w.T @ mid[b, :, n]
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)


def test_block_identity_1x1_is_plain_flexconv():
    feat, pos, nbr, _, theta, bias, g = _case(1, Din0=4, Dmid=4)
    eye = np.eye(4, dtype=np.float32)
    np.testing.assert_allclose(oracle.block_fwd(feat, pos, nbr, eye, theta, bias),
                               oracle.flexconv_fwd(feat, pos, nbr, theta, bias), rtol=1e-13, atol=1e-13)
    gf, gW, gt, gb = oracle.block_bwd(feat, pos, nbr, eye, theta, bias, g)
    rf, rt, rb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    np.testing.assert_allclose(gf, rf, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gt, rt, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gb, rb, rtol=1e-12, atol=1e-12)


def test_block_fwd_is_flexconv_of_the_1x1_output():
    # the second step alone is the (separately pinned) flex-conv oracle; feeding it the 1x1 output rounded
    # to float32 can differ from the all-double block by that rounding only
    feat, pos, nbr, W, theta, bias, _ = _case(2)
    mid = np.einsum("ce,ben->bcn", W.astype(np.float64), feat.astype(np.float64)).astype(np.float32)
    a = oracle.block_fwd(feat, pos, nbr, W, theta, bias)
    b = oracle.flexconv_fwd(mid, pos, nbr, theta, bias)
    assert np.abs(a - b).max() <= 2e-6 * np.abs(a).max()


def test_block_bwd_finite_differences_full_jacobian():
    # the block is linear in feat, in W and in (theta, bias): a central difference is exact up to rounding
    feat, pos, nbr, W, theta, bias, g = _case(3, B=1, N=9, K=3, Din0=2, Dmid=3, Dout=2)
    gf, gW, gt, gb = oracle.block_bwd(feat, pos, nbr, W, theta, bias, g)
    g64 = g.astype(np.float64)
    h = np.float32(0.25)

    def loss(f, w, t, bb):
        return (oracle.block_fwd(f, pos, nbr, w, t, bb) * g64).sum()

    for name, arr, grad, idx_arg in (("feat", feat, gf, 0), ("W", W, gW, 1), ("theta", theta, gt, 2), ("bias", bias, gb, 3)):
        for idx in np.ndindex(arr.shape):
            args = [feat, W, theta, bias]
            plus, minus = arr.copy(), arr.copy()
            plus[idx] += h
            minus[idx] -= h
            args[idx_arg] = plus
            lp = loss(*args)
            args[idx_arg] = minus
            lm = loss(*args)
            fd = (lp - lm) / (float(plus[idx]) - float(minus[idx]))
            assert abs(fd - grad[idx]) <= 1e-9 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])
