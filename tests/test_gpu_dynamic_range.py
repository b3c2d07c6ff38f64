"""GPU parity where the operands of the contraction span a wide dynamic range.

The kernels contract on the f16 matrix cores with every fp32 value carried as two scaled halves, so what has to be
shown is that magnitudes far apart inside one point's aggregate or inside the parameter matrix do not cost bits:
input channels whose scales differ by 2^24 with the parameters scaled the other way (every channel then contributes
alike to every output, Eq. 4's sum over c), output channels 2^24 apart, and a first-layer input of mixed units
(metres, 0..255 colours, [0,1] normalised coordinates).  Errors are judged channel by channel: the floor of the
relative error is the RMS of the reference over that channel alone, so a small-scale channel is not hidden behind a
large one."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, dev, to_layout, from_layout, say
from helpers import rel_err
from test_gpu_parity import random_problem

pytestmark = pytest.mark.gpu


def rel_err_per_channel(got, ref, axis):
    """max over the channels along `axis` of max |got-ref| / max(|ref|, RMS of that channel's reference)."""
    got = np.moveaxis(np.asarray(got, np.float64), axis, 0).reshape(ref.shape[axis], -1)
    ref = np.moveaxis(np.asarray(ref, np.float64), axis, 0).reshape(ref.shape[axis], -1)
    rms = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    ok = rms[:, 0] > 0
    return float(np.max(np.abs(got[ok] - ref[ok]) / np.maximum(np.abs(ref[ok]), rms[ok])))


def run_all(pos, nbr, feat, theta, bias, g, layout):
    a = (to_layout(feat, layout), dev(pos), dev(nbr), dev(theta), dev(bias))
    out = fx.flexconv_fwd(*a, layout=layout)
    gf, gt, gb = fx.flexconv_bwd(*a, to_layout(g, layout), layout=layout)
    torch.cuda.synchronize()
    return from_layout(out, layout), from_layout(gf, layout), gt.cpu().numpy(), gb.cpu().numpy()


SHAPES = [(1, 1000, 8, 64, 64), (2, 300, 8, 32, 64), (1, 400, 16, 128, 128), (1, 300, 9, 64, 32),
          (1, 300, 8, 256, 128), (1, 500, 8, 9, 64), (1, 300, 8, 20, 13)]


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K,Din,Dout", SHAPES)
def test_input_channels_2p24_apart(B, N, K, Din, Dout, layout):
    say(f"dynamic range, input channels: B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    pos, nbr, feat, theta, bias, g = random_problem(300 + N + Din, B, N, K, Din, Dout)
    rng = np.random.default_rng(Din * 1000 + Dout)
    s = np.exp2(rng.integers(-12, 13, size=Din)).astype(np.float32)
    s[0], s[-1] = 2.0 ** 12, 2.0 ** -12
    feat = feat * s[None, :, None]                    # powers of two: exact
    theta = theta / s[None, :, None]
    bias = bias / s[:, None]
    out, gf, gt, gb = run_all(pos, nbr, feat, theta, bias, g, layout)
    ref = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    errs = dict(fwd=rel_err_per_channel(out, ref, 1), grad_feat=rel_err_per_channel(gf, rgf, 1),
                grad_theta=rel_err_per_channel(gt, rgt, 1), grad_bias=rel_err_per_channel(gb, rgb, 0))
    say("  per-channel rel err: " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()))
    assert max(errs.values()) <= TOL, errs


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K,Din,Dout", SHAPES)
def test_output_channels_2p24_apart(B, N, K, Din, Dout, layout):
    say(f"dynamic range, output channels: B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    pos, nbr, feat, theta, bias, g = random_problem(400 + N + Dout, B, N, K, Din, Dout)
    rng = np.random.default_rng(Din * 1000 + Dout + 1)
    s = np.exp2(rng.integers(-12, 13, size=Dout)).astype(np.float32)
    s[0], s[-1] = 2.0 ** -12, 2.0 ** 12
    theta = theta * s[None, None, :]
    bias = bias * s[None, :]
    g = g / s[None, :, None]                          # every output channel weighs alike in the feature gradient
    out, gf, gt, gb = run_all(pos, nbr, feat, theta, bias, g, layout)
    ref = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    errs = dict(fwd=rel_err_per_channel(out, ref, 1), grad_feat=rel_err_per_channel(gf, rgf, 1),
                grad_theta=rel_err_per_channel(gt, rgt, 2), grad_bias=rel_err_per_channel(gb, rgb, 1))
    say("  per-channel rel err: " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()))
    assert max(errs.values()) <= TOL, errs


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
def test_first_layer_input_of_mixed_units(layout):
    # xyz in metres in a 10 x 10 x 3 room, 0..255 colours, [0,1] normalised coordinates; neighbours a few cm away
    B, N, K, Din, Dout = 1, 4000, 8, 9, 64
    say(f"dynamic range, mixed units: layout={layout}")
    rng = np.random.default_rng(99)
    xyz = (rng.random((B, 3, N)) * np.array([10.0, 10.0, 3.0])[None, :, None]).astype(np.float32)
    order = np.argsort(xyz[0, 0])
    xyz = np.ascontiguousarray(xyz[:, :, order])
    nbr = ((np.arange(N)[None, None, :] + rng.integers(-10, 11, size=(B, K, N))) % N).astype(np.int32)
    nbr[:, 0, :] = np.arange(N)
    rgb = rng.integers(0, 256, size=(B, 3, N)).astype(np.float32)
    feat = np.concatenate([xyz, rgb, xyz / np.array([10.0, 10.0, 3.0], np.float32)[None, :, None]], axis=1)
    std = (4.0 * Din * K) ** -0.5
    theta = (rng.standard_normal((3, Din, Dout)) * std).astype(np.float32)
    bias = (rng.standard_normal((Din, Dout)) * std).astype(np.float32)
    g = rng.standard_normal((B, Dout, N)).astype(np.float32)
    out, gf, gt, gb = run_all(xyz, nbr, feat, theta, bias, g, layout)
    ref = oracle.flexconv_fwd(feat, xyz, nbr, theta, bias)
    rgf, rgt, rgb_ = oracle.flexconv_bwd(feat, xyz, nbr, theta, bias, g)
    errs = dict(fwd=rel_err_per_channel(out, ref, 1), grad_feat=rel_err_per_channel(gf, rgf, 1),
                grad_theta=rel_err_per_channel(gt, rgt, 1), grad_bias=rel_err_per_channel(gb, rgb_, 0),
                fwd_whole=rel_err(out, ref))
    say("  per-channel rel err: " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()))
    assert max(errs.values()) <= TOL, errs
