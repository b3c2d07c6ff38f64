"""Seeded random valid shapes (cloud count, size, K, widths, layout, with and without prebuilt lists) through the
entry points against the oracle: the widths draw from values that have kernels of their own, that run as block
passes, and that run zero-padded, so every dispatch path is crossed with ragged sizes and odd K."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, ExactWorkspace, dev, to_layout, from_layout, say
from helpers import rel_err

pytestmark = pytest.mark.gpu
WIDTHS = [1, 3, 5, 9, 13, 20, 32, 33, 64, 65, 100, 128, 129, 192, 256, 300, 384]
CHANNELS = [1, 3, 4, 5, 12, 16, 32, 33, 64, 68, 128, 192, 256, 260]


@pytest.mark.parametrize("case", range(24))
def test_convolution_entry_points_on_random_shapes(case):
    rng = np.random.default_rng(7000 + case)
    B, N = int(rng.integers(1, 4)), int(rng.integers(1, 400))
    K = int(rng.integers(1, min(N, 20) + 1))
    Din, Dout, layout = int(rng.choice(WIDTHS)), int(rng.choice(WIDTHS)), int(rng.integers(0, 2))
    if Din * Dout > 256 * 256:
        Dout = 64
    say(f"random conv case {case}: B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    pos = rng.standard_normal((B, 3, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    if rng.random() < 0.5:
        nbr[:, 0, :] = np.arange(N)
    feat = rng.standard_normal((B, Din, N)).astype(np.float32)
    theta = (rng.standard_normal((3, Din, Dout)) / np.sqrt(4 * Din * K)).astype(np.float32)
    bias = (rng.standard_normal((Din, Dout)) / np.sqrt(4 * Din * K)).astype(np.float32)
    g = rng.standard_normal((B, Dout, N)).astype(np.float32)
    dn = dev(nbr)
    a = (to_layout(feat, layout), dev(pos), dn, dev(theta), dev(bias))
    # every call gets a workspace of exactly the size the library asks for, guarded behind its end
    w = ExactWorkspace(fx.OP_CONV_FWD, B, N, K, Din, Dout, layout)
    out = fx.flexconv_fwd(*a, layout=layout, workspace=w.ws)
    w.check()
    edges = fx.flex_inedges_build(dn) if rng.random() < 0.5 else None
    w = ExactWorkspace(fx.OP_CONV_BWD if edges is not None else fx.OP_CONV_BWD_BUILD, B, N, K, Din, Dout, layout)
    gf, gt, gb = fx.flexconv_bwd(*a, to_layout(g, layout), layout=layout, in_edges=edges, workspace=w.ws)
    w.check()
    w = ExactWorkspace(fx.OP_CONV_BWD_POS if edges is not None else fx.OP_CONV_BWD_POS_BUILD, B, N, K, Din, Dout, layout)
    gp = fx.flexconv_bwd_pos(a[0], dn, a[3], to_layout(g, layout), layout=layout, in_edges=edges, workspace=w.ws)
    w.check()
    assert rel_err(from_layout(out, layout), oracle.flexconv_fwd(feat, pos, nbr, theta, bias)) <= TOL
    rgf, rgt, rgb = oracle.flexconv_bwd(feat, pos, nbr, theta, bias, g)
    assert rel_err(from_layout(gf, layout), rgf) <= TOL
    assert rel_err(gt.cpu().numpy(), rgt) <= TOL and rel_err(gb.cpu().numpy(), rgb) <= TOL
    rgp = oracle.flexconv_bwd_pos(feat, nbr, theta, g)
    if np.abs(rgp).max() > 0:       # all-self neighbourhoods cancel exactly in the oracle (covered elsewhere)
        assert rel_err(gp.cpu().numpy(), rgp) <= TOL


@pytest.mark.parametrize("case", range(16))
def test_pooling_and_upsampling_entry_points_on_random_shapes(case):
    rng = np.random.default_rng(9000 + case)
    B, N = int(rng.integers(1, 4)), int(rng.integers(2, 500))
    K, C = int(rng.integers(1, min(N, 20) + 1)), int(rng.choice(CHANNELS))
    layout, Ns = int(rng.integers(0, 2)), int(rng.integers(1, N + 1))
    say(f"random pool case {case}: B={B} N={N} K={K} C={C} Ns={Ns} layout={layout}")
    feat = rng.integers(-3, 4, size=(B, C, N)).astype(np.float32)                  # many ties
    feat[:, :, ::5] = rng.standard_normal(feat[:, :, ::5].shape).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    sel = np.stack([np.sort(rng.permutation(N)[:Ns]) for _ in range(B)]).astype(np.int32)
    dn, ds = dev(nbr), dev(sel)
    bits = lambda t: from_layout(t, layout).view(np.uint32)
    po, pa = fx.flexpool_fwd(to_layout(feat, layout), dn, layout=layout)
    ro, ra = oracle.flexpool_fwd(feat, nbr)
    assert np.array_equal(from_layout(pa, layout), ra) and np.array_equal(bits(po), ro.view(np.uint32))
    gfull = rng.standard_normal((B, C, N)).astype(np.float32)
    e_full = fx.flex_inedges_build(dn)
    pg = fx.flexpool_bwd(to_layout(gfull, layout), pa, layout=layout, in_edges=e_full)
    assert rel_err(from_layout(pg, layout), oracle.flexpool_bwd(gfull, ra)) <= 1e-5
    so, sa = fx.flexpool_sub_fwd(to_layout(feat, layout), dn, ds, layout=layout)
    rso, rsa = oracle.flexpool_sub_fwd(feat, nbr, sel)
    assert np.array_equal(from_layout(sa, layout), rsa) and np.array_equal(bits(so), rso.view(np.uint32))
    g = rng.standard_normal((B, C, Ns)).astype(np.float32)
    sg = fx.flexpool_sub_bwd(to_layout(g, layout), sa, N, layout=layout, in_edges=fx.flex_inedges_build_sub(dn, ds))
    assert rel_err(from_layout(sg, layout), oracle.flexpool_sub_bwd(g, rsa, sel, N)) <= 1e-5
    small = rng.standard_normal((B, C, Ns)).astype(np.float32)
    small[:, :, ::3] = 0.0
    uo, ua = fx.flexupsample_fwd(to_layout(small, layout), ds, dn, layout=layout)
    ruo, rua = oracle.flexupsample_fwd(small, sel, nbr)
    assert np.array_equal(from_layout(ua, layout), rua) and np.array_equal(bits(uo), ruo.view(np.uint32))
    ug = fx.flexupsample_bwd(to_layout(gfull, layout), ua, ds, e_full, layout=layout)
    assert rel_err(from_layout(ug, layout), oracle.flexupsample_bwd(gfull, rua, sel)) <= 1e-5
