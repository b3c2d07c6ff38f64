"""GPU parity for the flex-conv gradient with respect to the point locations."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, ExactWorkspace, dev, to_layout, say
from helpers import rel_err
from test_gpu_parity import random_problem
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu

SHAPES = [
    # B, N, K, Din, Dout
    (1, 1000, 8, 64, 64),      # matrix-core kernels, several tiles + ragged tail
    (2, 77, 8, 32, 32),
    (1, 300, 16, 64, 32),
    (2, 100, 8, 32, 64),
    (1, 257, 8, 9, 64),        # widths without a location-gradient kernel of their own: 64-channel column blocks
    (1, 300, 8, 256, 128),     # 4 x 2 blocks
    (2, 200, 8, 100, 200),     # ragged last blocks
    (1, 150, 9, 128, 128),
    (1, 130, 5, 64, 64),       # K not a multiple of 8: last batch of a tile has empty slots
    (2, 333, 9, 64, 64),
    (1, 500, 13, 32, 64),
    (1, 211, 20, 64, 32),
    (2, 150, 6, 5, 7),
    (1, 64, 1, 32, 32),
]


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K,Din,Dout", SHAPES)
def test_bwd_pos_matches_oracle(B, N, K, Din, Dout, layout):
    say(f"bwd_pos B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    pos, nbr, feat, theta, bias, g = random_problem(40 + N, B, N, K, Din, Dout)
    ref = oracle.flexconv_bwd_pos(feat, nbr, theta, g)
    dnbr = dev(nbr)
    a = (to_layout(feat, layout), dnbr, dev(theta), to_layout(g, layout))
    # workspaces of exactly the size the library asks for, guarded behind their end
    w = ExactWorkspace(fx.OP_CONV_BWD_POS_BUILD, B, N, K, Din, Dout, layout)
    gp = fx.flexconv_bwd_pos(*a, layout=layout, workspace=w.ws)
    w.check()
    w2 = ExactWorkspace(fx.OP_CONV_BWD_POS, B, N, K, Din, Dout, layout)
    gp2 = fx.flexconv_bwd_pos(*a, layout=layout, in_edges=fx.flex_inedges_build(dnbr), workspace=w2.ws)
    w2.check()
    if K == 1 and not ref.any():
        # every point is its own only neighbour: the two ends of each edge coincide and the exact result is 0.
        # The matrix-core path forms the two ends' sums separately, so what is left is rounding, measured
        # against the size of one edge's term s_d = sum_{c,o} theta[d,c,o] feat[c,n] grad_out[o,l].
        s_edge = np.einsum("dco,bcl,bol->bdl", theta.astype(np.float64), feat.astype(np.float64), g.astype(np.float64))
        scale = np.abs(s_edge).max()
        assert np.abs(gp.cpu().numpy()).max() <= TOL * scale
        assert np.abs(gp2.cpu().numpy()).max() <= TOL * scale
        return
    assert rel_err(gp.cpu().numpy(), ref) <= TOL
    assert rel_err(gp2.cpu().numpy(), ref) <= TOL
    # translation invariance of the layer: a cloud's location gradients sum to zero
    assert float(gp.double().sum(dim=2).abs().max()) <= 1e-3 * float(gp.double().abs().sum(dim=2).max() + 1e-30)


def test_bwd_pos_single_random_neighbour():
    # K = 1 with a neighbour other than the point itself: seven of a batch's eight slots are empty
    say("bwd_pos K=1 random neighbour")
    pos, nbr, feat, theta, bias, g = random_problem(7, 2, 301, 1, 64, 64, local=False)
    ref = oracle.flexconv_bwd_pos(feat, nbr, theta, g)
    gp = fx.flexconv_bwd_pos(to_layout(feat, fx.BNC), dev(nbr), dev(theta), to_layout(g, fx.BNC), layout=fx.BNC)
    torch.cuda.synchronize()
    assert rel_err(gp.cpu().numpy(), ref) <= TOL


def test_bwd_pos_config1_and_directional_derivative():
    cfg = CONFIGS[1]
    x = make_inputs(cfg)
    ref = oracle.flexconv_bwd_pos(x.feat, x.nbr, x.theta, x.grad_out)
    feat, nbr, theta, g = to_layout(x.feat, fx.BNC), dev(x.nbr), dev(x.theta), to_layout(x.grad_out, fx.BNC)
    gp = fx.flexconv_bwd_pos(feat, nbr, theta, g, layout=fx.BNC)
    torch.cuda.synchronize()
    assert rel_err(gp.cpu().numpy(), ref) <= TOL
    # <grad_pos, dpos> equals the change of <g, fwd> along dpos (the layer is affine in pos): tie to the forward kernel
    pos, bias = dev(x.pos), dev(x.bias)
    dpos = torch.randn(pos.shape, device="cuda", generator=torch.Generator("cuda").manual_seed(3)) * 0.01
    f1 = fx.flexconv_fwd(feat, pos + dpos, nbr, theta, bias, layout=fx.BNC).double()
    f0 = fx.flexconv_fwd(feat, pos - dpos, nbr, theta, bias, layout=fx.BNC).double()
    lhs = float(((f1 - f0) * g.double()).sum()) / 2.0
    rhs = float((gp.double() * dpos.double()).sum())
    assert abs(lhs - rhs) <= 2e-3 * max(abs(lhs), abs(rhs), 1e-12)
