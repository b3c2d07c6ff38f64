"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element
at sizes that span several tiles and a ragged tail, in both layouts."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, ExactWorkspace, dev, to_layout, from_layout, say
from helpers import rel_err
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def random_problem(seed, B, N, K, Din, Dout, local=True):
    rng = np.random.default_rng(seed)
    pos = rng.standard_normal((B, 3, N)).astype(np.float32)
    if local:   # neighbours near the centre index, with self first
        nbr = (np.arange(N)[None, None, :] + rng.integers(-20, 21, size=(B, K, N))) % N
        nbr[:, 0, :] = np.arange(N)
    else:
        nbr = rng.integers(0, N, size=(B, K, N))
    nbr = nbr.astype(np.int32)
    feat = rng.standard_normal((B, Din, N)).astype(np.float32)
    theta = (rng.standard_normal((3, Din, Dout)) / np.sqrt(4 * Din * K)).astype(np.float32)
    bias = (rng.standard_normal((Din, Dout)) / np.sqrt(4 * Din * K)).astype(np.float32)
    g = rng.standard_normal((B, Dout, N)).astype(np.float32)
    return pos, nbr, feat, theta, bias, g


SHAPES = [
    # B, N, K, Din, Dout
    (1, 1000, 8, 64, 64),      # several tiles + ragged tail
    (2, 77, 3, 32, 32),        # two clouds, tail only tiles
    (1, 300, 16, 128, 128),
    (1, 257, 8, 9, 64),        # first-layer shape, padded depth
    (1, 130, 5, 64, 9),
    (2, 100, 8, 32, 64),
    (1, 100, 8, 64, 32),
    (1, 100, 4, 64, 128),
    (1, 100, 4, 128, 64),
    (1, 200, 40, 64, 64),      # K larger than one staging chunk
    (1, 64, 1, 32, 32),        # K = 1
    (1, 8, 8, 64, 64),         # one partial tile, every point a neighbour of every point
    (3, 17, 8, 64, 64),        # three clouds, each a single ragged tile
    (1, 48, 16, 64, 64),       # exactly one tile of the widest kernel, two batches
    (2, 49, 8, 32, 32),        # one point past a tile
    (1, 700, 9, 64, 64),       # the paper's profiling K: second batch of every tile masked past K, upper half skipped
    (2, 333, 12, 64, 64),      # masked tail batch whose lower half is full
    (1, 250, 20, 32, 64),      # three batches, the last one half empty
    (1, 500, 13, 9, 64),       # masked tail, single-float lanes
    (1, 333, 8, 256, 256),     # wide layers: passes over 64- / 128-channel column blocks
    (2, 150, 8, 128, 256),
    (1, 200, 16, 256, 128),
    (1, 130, 9, 384, 128),     # masked tail in the block passes
    (1, 500, 8, 512, 512),     # many parameter blocks, few tiles: one workgroup per block of the parameter gradient
    (1, 4000, 8, 256, 256),    # several workgroups share a block
    (2, 150, 6, 5, 7),         # widths without a kernel of their own: zero-padded to the nearest that has one
    (1, 90, 4, 20, 16),
    (1, 300, 8, 3, 64),        # colour-only input features
    (1, 300, 8, 64, 13),       # class scores
    (1, 200, 8, 100, 100),
    (1, 150, 8, 200, 300),     # padded to a wide layer
    (2, 150, 8, 64, 256),
]


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K,Din,Dout", SHAPES)
def test_flexconv_fwd_matches_oracle(B, N, K, Din, Dout, layout):
    say(f"fwd B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    pos, nbr, feat, theta, bias, _ = random_problem(10 + N, B, N, K, Din, Dout)
    ref = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    # a workspace of exactly the size the library asks for, guarded behind its end
    w = ExactWorkspace(fx.OP_CONV_FWD, B, N, K, Din, Dout, layout)
    out = fx.flexconv_fwd(to_layout(feat, layout), dev(pos), dev(nbr), dev(theta), dev(bias), layout=layout,
                          workspace=w.ws)
    w.check()
    assert rel_err(from_layout(out, layout), ref) <= TOL


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K,Din,Dout", SHAPES)
def test_flexconv_bwd_matches_oracle(B, N, K, Din, Dout, layout):
    say(f"bwd B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    pos, nbr, feat, theta, bias, g = random_problem(20 + N, B, N, K, Din, Dout)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    # in-edge lists built inside the call, in a workspace of exactly the size the library asks for
    w = ExactWorkspace(fx.OP_CONV_BWD_BUILD, B, N, K, Din, Dout, layout)
    gf, gt, gb = fx.flexconv_bwd(to_layout(feat, layout), dev(pos), dev(nbr), dev(theta), dev(bias),
                                 to_layout(g, layout), layout=layout, workspace=w.ws)
    w.check()
    assert rel_err(from_layout(gf, layout), rgf) <= TOL
    assert rel_err(gt.cpu().numpy(), rgt) <= TOL
    assert rel_err(gb.cpu().numpy(), rgb) <= TOL
    # and with caller-supplied lists (a smaller plan)
    dnbr = dev(nbr)
    w2 = ExactWorkspace(fx.OP_CONV_BWD, B, N, K, Din, Dout, layout)
    gf2, gt2, gb2 = fx.flexconv_bwd(to_layout(feat, layout), dev(pos), dnbr, dev(theta), dev(bias),
                                    to_layout(g, layout), layout=layout, in_edges=fx.flex_inedges_build(dnbr),
                                    workspace=w2.ws)
    w2.check()
    assert rel_err(from_layout(gf2, layout), rgf) <= TOL
    assert rel_err(gt2.cpu().numpy(), rgt) <= TOL and rel_err(gb2.cpu().numpy(), rgb) <= TOL


def test_flexconv_bwd_partial_outputs_and_prebuilt_inedges():
    B, N, K, Din, Dout = 2, 333, 8, 64, 64
    pos, nbr, feat, theta, bias, g = random_problem(5, B, N, K, Din, Dout, local=False)
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    d = dict(layout=fx.BNC)
    args = (to_layout(feat, fx.BNC), dev(pos), dev(nbr), dev(theta), dev(bias), to_layout(g, fx.BNC))
    edges = fx.flex_inedges_build(args[2])
    gf, gt, gb = fx.flexconv_bwd(*args, in_edges=edges, **d)
    gf2, none_t, none_b = fx.flexconv_bwd(*args, need_params=False, **d)
    none_f, gt2, gb2 = fx.flexconv_bwd(*args, need_feat=False, **d)
    torch.cuda.synchronize()
    assert none_t is None and none_b is None and none_f is None
    assert rel_err(from_layout(gf, fx.BNC), rgf) <= TOL and rel_err(gt.cpu().numpy(), rgt) <= TOL
    assert torch.equal(gf, gf2)                      # gather form: bit-reproducible
    # the parameter gradients alone come from their own kernel, together with the feature gradient from the
    # one-pass kernel: two routes, each held to the oracle, and each bit-reproducible from call to call
    assert rel_err(gt2.cpu().numpy(), rgt) <= TOL and rel_err(gb2.cpu().numpy(), rgb) <= TOL
    assert rel_err(gb.cpu().numpy(), rgb) <= TOL
    gf3, gt3, gb3 = fx.flexconv_bwd(*args, in_edges=edges, **d)
    _, gt4, gb4 = fx.flexconv_bwd(*args, need_feat=False, **d)
    assert torch.equal(gf, gf3) and torch.equal(gt, gt3) and torch.equal(gb, gb3)
    assert torch.equal(gt2, gt4) and torch.equal(gb2, gb4)


def test_inedges_are_the_transposed_graph():
    rng = np.random.default_rng(3)
    B, N, K = 3, 500, 7
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    nbr[0, :, :] = 5                                   # one point with in-degree K*N
    off, src = fx.flex_inedges_build(dev(nbr))
    off, src = off.cpu().numpy(), src.cpu().numpy()
    assert off[0] == 0 and off[-1] == B * K * N and (np.diff(off) >= 0).all()
    for b in range(B):
        for m in rng.integers(0, N, size=40).tolist() + [5]:
            g = b * N + m
            got = src[off[g]:off[g + 1]]
            want = np.sort(np.nonzero(nbr[b] == m)[1])
            assert np.array_equal(np.sort(got), want)
            assert np.array_equal(got, want)            # ascending, whatever the length


def test_degenerate_neighbourhoods():
    # every point lists point 0 only; and every point lists itself K times
    B, N, K, Din, Dout = 1, 200, 4, 32, 32
    pos, nbr, feat, theta, bias, g = random_problem(8, B, N, K, Din, Dout)
    for case in (np.zeros_like(nbr), np.broadcast_to(np.arange(N, dtype=np.int32), nbr.shape).copy()):
        ref = oracle.flexconv_fwd(feat, pos, case, theta, bias)
        rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, case, theta, bias, g)
        a = (to_layout(feat, fx.BNC), dev(pos), dev(case), dev(theta), dev(bias))
        out = fx.flexconv_fwd(*a, layout=fx.BNC)
        gf, gt, gb = fx.flexconv_bwd(*a, to_layout(g, fx.BNC), layout=fx.BNC)
        torch.cuda.synchronize()
        assert rel_err(from_layout(out, fx.BNC), ref) <= TOL
        assert rel_err(from_layout(gf, fx.BNC), rgf) <= TOL
        assert rel_err(gt.cpu().numpy(), rgt) <= TOL or np.abs(rgt).max() < 1e-12   # self only: every difference is 0
        assert rel_err(gb.cpu().numpy(), rgb) <= TOL


POOL_SHAPES = [(1, 1000, 8, 64), (2, 77, 3, 32), (1, 130, 16, 128), (2, 150, 6, 5), (1, 64, 1, 9), (2, 200, 20, 12),
               (1, 40, 9, 18), (1, 300, 8, 1280), (2, 100, 5, 2052)]   # the last two: rows wider than a block


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,N,K,C", POOL_SHAPES)
def test_flexpool_matches_oracle_bit_exactly(B, N, K, C, layout):
    say(f"pool B={B} N={N} K={K} C={C} layout={layout}")
    rng = np.random.default_rng(N + C)
    feat = rng.integers(-3, 4, size=(B, C, N)).astype(np.float32)       # many ties
    feat[:, :, ::7] = -0.0
    feat[:, :, 1::9] = rng.standard_normal(feat[:, :, 1::9].shape).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    g = rng.standard_normal((B, C, N)).astype(np.float32)
    ro, ra = oracle.flexpool_fwd(feat, nbr)
    dnbr = dev(nbr)
    out, arg = fx.flexpool_fwd(to_layout(feat, layout), dnbr, layout=layout)
    gf = fx.flexpool_bwd(to_layout(g, layout), arg, layout=layout)                       # atomic scatter
    edges = fx.flex_inedges_build(dnbr)
    gf2 = fx.flexpool_bwd(to_layout(g, layout), arg, layout=layout, in_edges=edges, K=K)  # in-edge gather
    gf3 = fx.flexpool_bwd(to_layout(g, layout), arg, layout=layout, in_edges=edges)
    torch.cuda.synchronize()
    assert np.array_equal(from_layout(arg, layout), ra)
    assert np.array_equal(from_layout(out, layout).view(np.uint32), ro.view(np.uint32))
    rgf = oracle.flexpool_bwd(g, ra)
    assert rel_err(from_layout(gf, layout), rgf) <= 1e-5
    assert rel_err(from_layout(gf2, layout), rgf) <= 1e-5
    assert torch.equal(gf2, gf3)                                                          # fixed order


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
def test_flexpool_hub_point_and_unlisted_points(layout):
    # one point that every centre lists (an in-edge list of N entries), many points that nobody lists
    say(f"pool hub layout={layout}")
    B, N, K, C = 2, 3000, 5, 20
    rng = np.random.default_rng(77)
    feat = rng.standard_normal((B, C, N)).astype(np.float32)
    feat[:, ::2, 0] = 10.0                                   # the hub wins every other channel everywhere
    nbr = rng.integers(0, N // 3, size=(B, K, N)).astype(np.int32)   # the upper two thirds are never listed
    nbr[:, 0, :] = 0
    nbr[:, 1, :] = 0                                         # listed twice by every centre
    g = rng.standard_normal((B, C, N)).astype(np.float32)
    ro, ra = oracle.flexpool_fwd(feat, nbr)
    dnbr = dev(nbr)
    out, arg = fx.flexpool_fwd(to_layout(feat, layout), dnbr, layout=layout)
    gf = fx.flexpool_bwd(to_layout(g, layout), arg, layout=layout, in_edges=fx.flex_inedges_build(dnbr))
    torch.cuda.synchronize()
    assert np.array_equal(from_layout(arg, layout), ra)
    assert np.array_equal(from_layout(out, layout).view(np.uint32), ro.view(np.uint32))
    rgf = oracle.flexpool_bwd(g, ra)
    got = from_layout(gf, layout)
    assert rel_err(got, rgf) <= 1e-5
    assert not got[:, :, N // 3:].any()


def test_validate_neighbors_counts_out_of_range():
    nbr = np.zeros((2, 3, 50), np.int32)
    nbr[0, 1, 4] = 50
    nbr[1, 2, 7] = -1
    assert fx.flex_validate_neighbors(dev(nbr)) == 2
    assert fx.flex_validate_neighbors(dev(np.zeros((1, 2, 9), np.int32))) == 0


@pytest.mark.parametrize("ci", [0, 1])
def test_config_full_parity(ci):
    cfg = CONFIGS[ci]
    say(f"config {ci}: {cfg.name}")
    x = make_inputs(cfg)
    ref = oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias)
    rgf, rgt, rgb = oracle.flexconv_bwd(x.feat, x.pos, x.nbr, x.theta, x.bias, x.grad_out)
    for layout in (fx.BNC, fx.BCN):
        a = (to_layout(x.feat, layout), dev(x.pos), dev(x.nbr), dev(x.theta), dev(x.bias))
        out = fx.flexconv_fwd(*a, layout=layout)
        gf, gt, gb = fx.flexconv_bwd(*a, to_layout(x.grad_out, layout), layout=layout)
        torch.cuda.synchronize()
        errs = (rel_err(from_layout(out, layout), ref), rel_err(from_layout(gf, layout), rgf),
                rel_err(gt.cpu().numpy(), rgt), rel_err(gb.cpu().numpy(), rgb))
        say(f"  layout {layout}: rel err fwd/gfeat/gtheta/gbias = " + " ".join(f"{e:.2e}" for e in errs))
        assert max(errs) <= TOL
        if "pool_fwd" in cfg.runs:
            ro, ra = oracle.flexpool_fwd(x.feat, x.nbr)
            po, pa = fx.flexpool_fwd(a[0], a[2], layout=layout)
            pg = fx.flexpool_bwd(to_layout(x.grad_out, layout), pa, layout=layout)
            pg2 = fx.flexpool_bwd(to_layout(x.grad_out, layout), pa, layout=layout,
                                  in_edges=fx.flex_inedges_build(a[2]))
            torch.cuda.synchronize()
            assert np.array_equal(from_layout(pa, layout), ra)
            assert np.array_equal(from_layout(po, layout).view(np.uint32), ro.view(np.uint32))
            rpg = oracle.flexpool_bwd(x.grad_out, ra)
            assert rel_err(from_layout(pg, layout), rpg) <= 1e-5
            assert rel_err(from_layout(pg2, layout), rpg) <= 1e-5
