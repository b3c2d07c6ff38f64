"""The one-pass backward of 64 -> 64 layers (feature gradient and parameter gradients from one walk over the in-edge
lists, Sec. 3.1's gradients regrouped by the listed point): cases aimed at what is particular to it.

Its contraction over points carries the points' own feature rows as f16 halves scaled per channel from a SAMPLE of the
rows; a row far above the sampled magnitudes overflows f16, the kernel raises a flag and the stand-alone
parameter-gradient kernel takes over.  The outlier tests plant such rows: without the fall-back the result would be
Inf / NaN, so passing them shows the fall-back ran and is correct."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, ExactWorkspace, dev, to_layout, from_layout, say
from helpers import rel_err
from test_gpu_parity import random_problem
from test_gpu_dynamic_range import rel_err_per_channel

pytestmark = pytest.mark.gpu

# the kernel's control words close the planned workspace: a 64-word flag block (word 0: 0 = the one-pass result stands,
# 1 = a feature row overflowed f16, 2 = the check after the reduction found the result unresolved), then 1024 records
CONTROL_BYTES = 4 * (64 + 128 * 1024)


def run_bwd(pos, nbr, feat, theta, bias, g, layout, B, N, K):
    """-> grad_feat, grad_theta, grad_bias, and the flag: non-zero if the parameter gradients were handed to the
    stand-alone kernel.  With caller-supplied lists the control words are the last region of the planned workspace."""
    dnbr = dev(nbr)
    edges = fx.flex_inedges_build(dnbr)
    w = ExactWorkspace(fx.OP_CONV_BWD, B, N, K, 64, 64, layout)
    gf, gt, gb = fx.flexconv_bwd(to_layout(feat, layout), dev(pos), dnbr, dev(theta), dev(bias), to_layout(g, layout),
                                 layout=layout, workspace=w.ws, in_edges=edges)
    torch.cuda.synchronize()
    w.check()
    handed_over = int(w.ws[w.need - CONTROL_BYTES:w.need - CONTROL_BYTES + 4].view(torch.int32).item())
    return from_layout(gf, layout), gt.cpu().numpy(), gb.cpu().numpy(), handed_over


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K", [(1, 1, 1), (1, 31, 4), (1, 33, 8), (2, 1000, 8), (3, 4097, 16), (1, 60000, 9)])
def test_sizes_around_the_tile(B, N, K, layout):
    say(f"one-pass backward: B={B} N={N} K={K} layout={layout}")
    assert fx.kernel_route(fx.OP_CONV_BWD, B, N, K, 64, 64, layout) == 7
    pos, nbr, feat, theta, bias, g = random_problem(900 + N + K, B, N, K, 64, 64, local=(N > 2000))
    gf, gt, gb, handed_over = run_bwd(pos, nbr, feat, theta, bias, g, layout, B, N, K)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    errs = dict(gf=rel_err(gf, rgf), gt=rel_err(gt, rgt), gb=rel_err(gb, rgb))
    say("  " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()) + f" handed over: {handed_over}")
    assert max(errs.values()) <= TOL, errs
    assert not handed_over or N * K < 64, "ordinary data must stay on the one-pass kernel"


@pytest.mark.parametrize("kind", ["few_huge_rows", "one_huge_channel_value", "growing_along_the_cloud",
                                  "large_features_where_the_gradient_is_tiny", "inf_free_tiny"])
def test_rows_far_from_the_sampled_magnitudes(kind):
    B, N, K = 1, 200_000, 8
    say(f"one-pass backward, outliers: {kind}")
    pos, nbr, feat, theta, bias, g = random_problem(77, B, N, K, 64, 64, local=True)
    rng = np.random.default_rng(5)
    if kind == "few_huge_rows":                     # 40 rows 2^40 above the rest: most workgroups never sample theirs
        feat[0, :, rng.choice(N, 40, replace=False)] *= np.float32(2.0 ** 40)
    elif kind == "one_huge_channel_value":          # a single element
        feat[0, 17, N // 2 + 11] = np.float32(3.0e30)
    elif kind == "growing_along_the_cloud":         # magnitudes rising by 2^60 from the first point to the last
        feat *= np.exp2(np.linspace(-30, 30, N, dtype=np.float64)).astype(np.float32)[None, None, :]
        g *= np.exp2(np.linspace(20, -20, N, dtype=np.float64)).astype(np.float32)[None, None, :]
    elif kind == "large_features_where_the_gradient_is_tiny":
        # two clouds (no edges between them; every workgroup walks tiles of both): one with features 2^40 larger and
        # an upstream gradient 2^60 smaller than the other's.  It sets the channel exponents, contributes nothing, and
        # pushes the other cloud's features below the f16 range: the one-pass result is small and wrong
        B, N = 2, 100_000
        pos, nbr, feat, theta, bias, g = random_problem(77, B, N, K, 64, 64, local=True)
        feat[0] *= np.float32(2.0 ** 40)
        g[0] *= np.float32(2.0 ** -60)
    else:                                           # everything tiny: the channel exponents reach their clamp
        feat *= np.float32(2.0 ** -100)
    gf, gt, gb, handed_over = run_bwd(pos, nbr, feat, theta, bias, g, fx.BNC, B, N, K)
    assert np.isfinite(gt).all() and np.isfinite(gb).all() and np.isfinite(gf).all()
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    errs = dict(gf=rel_err(gf, rgf), gt=rel_err(gt, rgt), gb=rel_err(gb, rgb))
    say("  " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()) + f" handed over: {handed_over}")
    assert max(errs.values()) <= TOL, errs
    # a trend along the cloud is mild inside one workgroup's stretch of it: the one-pass result stands (and is right)
    expect = {"few_huge_rows": 1, "one_huge_channel_value": 1, "growing_along_the_cloud": 0,
              "large_features_where_the_gradient_is_tiny": 2, "inf_free_tiny": 0}[kind]
    assert handed_over == expect, "overflowing rows hand over at once, an unresolved result after the check"


def test_channel_scales_2p24_apart_on_a_cloud_of_many_tiles():
    # the per-channel metric of the dynamic-range tests at a size where every workgroup walks dozens of tiles
    B, N, K = 1, 300_000, 8
    pos, nbr, feat, theta, bias, g = random_problem(78, B, N, K, 64, 64, local=True)
    rng = np.random.default_rng(6)
    s = np.exp2(rng.integers(-12, 13, size=64)).astype(np.float32)
    s[0], s[-1] = 2.0 ** 12, 2.0 ** -12
    feat = feat * s[None, :, None]
    theta = theta / s[None, :, None]
    bias = bias / s[:, None]
    gf, gt, gb, handed_over = run_bwd(pos, nbr, feat, theta, bias, g, fx.BNC, B, N, K)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    errs = dict(gf=rel_err_per_channel(gf, rgf, 1), gt=rel_err_per_channel(gt, rgt, 1), gb=rel_err_per_channel(gb, rgb, 0))
    say("  per-channel: " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()) + f" handed over: {handed_over}")
    assert max(errs.values()) <= TOL, errs
    assert not handed_over, "channel scales are what the per-channel exponents are for"


def test_zero_upstream_gradient_and_zero_features():
    B, N, K = 1, 5000, 8
    pos, nbr, feat, theta, bias, g = random_problem(79, B, N, K, 64, 64)
    for zf, zg in ((True, False), (False, True)):
        f2 = np.zeros_like(feat) if zf else feat
        g2 = np.zeros_like(g) if zg else g
        gf, gt, gb, _ = run_bwd(pos, nbr, f2, theta, bias, g2, fx.BNC, B, N, K)
        rgf, rgt, rgb = oracle.flexconv_bwd(f2, pos, nbr, theta, bias, g2)
        assert np.all(gt == 0) and np.all(gb == 0)
        assert (np.all(gf == 0) if zg else rel_err(gf, rgf) <= TOL)


@pytest.mark.parametrize("kind", ["relu_sparse_features_dead_channels", "gradient_on_a_tenth_of_the_points",
                                  "heavy_tailed_features"])
def test_ordinary_training_tensors_stay_on_the_one_pass_kernel(kind):
    """What real layers see: activations after a ReLU (mostly zeros, some channels dead), an upstream gradient that
    is zero on unlabelled points, magnitudes with heavy tails.  None of it may trip the hand-over."""
    B, N, K = 1, 250_000, 8
    pos, nbr, feat, theta, bias, g = random_problem(81, B, N, K, 64, 64, local=True)
    rng = np.random.default_rng(8)
    if kind == "relu_sparse_features_dead_channels":
        feat = np.maximum(feat - 1.0, 0.0).astype(np.float32)          # 84 % zeros
        feat[:, [3, 17, 40], :] = 0.0                                   # dead channels
        g[:, [5, 60], :] = 0.0                                          # output channels without gradient
    elif kind == "gradient_on_a_tenth_of_the_points":
        g[:, :, rng.random(N) > 0.1] = 0.0
    else:
        feat = (feat * np.exp(1.5 * rng.standard_normal((B, 1, N)))).astype(np.float32)     # log-normal row scales
        g = (g * np.exp(1.5 * rng.standard_normal((B, 1, N)))).astype(np.float32)
    gf, gt, gb, handed_over = run_bwd(pos, nbr, feat, theta, bias, g, fx.BNC, B, N, K)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    errs = dict(gf=rel_err(gf, rgf), gt=rel_err(gt, rgt), gb=rel_err(gb, rgb))
    say(f"one-pass backward, {kind}: " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()) + f" handed over: {handed_over}")
    assert max(errs.values()) <= TOL, errs
    assert not handed_over
