"""GPU parity for the 1x1-convolution + flex-convolution block evaluated as ONE flex-convolution with composed
parameters (flexconv_compose_1x1 + flexconv_fwd / flexconv_bwd + flexconv_compose_1x1_bwd), against the CPU
oracle's two-step block."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import dev, to_layout, from_layout, say
from helpers import rel_err
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu
TOL = 1e-4      # the flex-conv tolerance: the composition itself is summed in double


def _block(x, W, layout):
    dW, dth, dbi = dev(W), dev(x.theta), dev(x.bias)
    tc, bc = fx.flexconv_compose_1x1(dW, dth, dbi)
    feat, pos, nbr, g = to_layout(x.feat, layout), dev(x.pos), dev(x.nbr), to_layout(x.grad_out, layout)
    out = fx.flexconv_fwd(feat, pos, nbr, tc, bc, layout=layout)
    gf, gtc, gbc = fx.flexconv_bwd(feat, pos, nbr, tc, bc, g, layout=layout)
    gW, gt, gb = fx.flexconv_compose_1x1_bwd(dW, dth, dbi, gtc, gbc)
    torch.cuda.synchronize()
    return tc, bc, out, gf, gW, gt, gb


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("cfg_i,n,Din0", [(0, 1500, 32), (1, 700, 64), (0, 333, 9), (1, 257, 48)])
def test_block_matches_oracle(cfg_i, n, Din0, layout):
    say(f"block cfg{cfg_i} n={n} Din0={Din0} layout={layout}")
    cfg = CONFIGS[cfg_i]
    x = make_inputs(cfg, n_override=n)
    Dmid = x.cfg.Din
    rng = np.random.default_rng(100 + Din0)
    W = (rng.standard_normal((Dmid, Din0)) / np.sqrt(Din0)).astype(np.float32)
    feat0 = rng.standard_normal((x.cfg.B, Din0, x.cfg.N)).astype(np.float32)
    x.feat = feat0
    tc, bc, out, gf, gW, gt, gb = _block(x, W, layout)
    # the composed parameters against the plain sums in double
    rtc = np.einsum("ce,dco->deo", W.astype(np.float64), x.theta.astype(np.float64))
    rbc = np.einsum("ce,co->eo", W.astype(np.float64), x.bias.astype(np.float64))
    assert rel_err(tc.cpu().numpy(), rtc) <= 1e-6 and rel_err(bc.cpu().numpy(), rbc) <= 1e-6
    ro = oracle.block_fwd(feat0, x.pos, x.nbr, W, x.theta, x.bias)
    rf, rW, rt, rb = oracle.block_bwd(feat0, x.pos, x.nbr, W, x.theta, x.bias, x.grad_out)
    assert rel_err(from_layout(out, layout), ro) <= TOL
    assert rel_err(from_layout(gf, layout), rf) <= TOL
    assert rel_err(gW.cpu().numpy(), rW) <= TOL
    assert rel_err(gt.cpu().numpy(), rt) <= TOL
    assert rel_err(gb.cpu().numpy(), rb) <= TOL


@pytest.mark.parametrize("Din0,Dmid,Dout", [(100, 130, 70), (200, 64, 257), (1, 5, 3), (64, 256, 128)])
def test_compose_kernels_on_ragged_and_multi_tile_widths(Din0, Dmid, Dout):
    """The composition and its transposes are plain matrix products over the channel indices: compared with their
    definition (float64 einsum) at widths that span several 64 x 64 tiles and leave ragged edges."""
    say(f"compose Din0={Din0} Dmid={Dmid} Dout={Dout}")
    rng = np.random.default_rng(Din0 + Dout)
    W = rng.standard_normal((Dmid, Din0)).astype(np.float32)
    theta = rng.standard_normal((3, Dmid, Dout)).astype(np.float32)
    bias = rng.standard_normal((Dmid, Dout)).astype(np.float32)
    gtc = rng.standard_normal((3, Din0, Dout)).astype(np.float32)
    gbc = rng.standard_normal((Din0, Dout)).astype(np.float32)
    tc, bc = fx.flexconv_compose_1x1(dev(W), dev(theta), dev(bias))
    gW, gt, gb = fx.flexconv_compose_1x1_bwd(dev(W), dev(theta), dev(bias), dev(gtc), dev(gbc))
    torch.cuda.synchronize()
    W64, t64, b64, gtc64, gbc64 = (a.astype(np.float64) for a in (W, theta, bias, gtc, gbc))
    assert rel_err(tc.cpu().numpy(), np.einsum("ce,dco->deo", W64, t64)) <= 1e-6
    assert rel_err(bc.cpu().numpy(), np.einsum("ce,co->eo", W64, b64)) <= 1e-6
    assert rel_err(gt.cpu().numpy(), np.einsum("ce,deo->dco", W64, gtc64)) <= 1e-6
    assert rel_err(gb.cpu().numpy(), np.einsum("ce,eo->co", W64, gbc64)) <= 1e-6
    assert rel_err(gW.cpu().numpy(), np.einsum("dco,deo->ce", t64, gtc64) + np.einsum("co,eo->ce", b64, gbc64)) <= 1e-6
