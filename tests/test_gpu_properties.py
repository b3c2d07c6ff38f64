"""Properties of the GPU path that need no oracle: translation of the cloud, permutation of the
neighbour slots, point relabelling, and agreement of the two tensor layouts."""
import numpy as np
import pytest
import torch

import paper_1803_07289_amd as fx
from gpu_util import dev, to_layout, from_layout, say
from helpers import rel_err
from test_gpu_parity import random_problem

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,N,K,Din,Dout", [(2, 500, 8, 64, 64), (1, 300, 5, 32, 32), (1, 200, 16, 64, 32)])
def test_translation_leaves_every_result_bit_identical(B, N, K, Din, Dout):
    # positions on a dyadic grid and a dyadic shift: pos + t is exact in float32, so every position
    # difference, hence every output bit, must be unchanged (the layer sees only differences, Sec. 3.1)
    pos, nbr, feat, theta, bias, g = random_problem(7 + N, B, N, K, Din, Dout)
    pos = (np.round(pos * 256) / 256).astype(np.float32)
    shift = np.array([4.0, -2.5, 16.0], np.float32)[None, :, None]
    a = (to_layout(feat, fx.BNC), dev(nbr), dev(theta), dev(bias))
    out0 = fx.flexconv_fwd(a[0], dev(pos), *a[1:], layout=fx.BNC)
    out1 = fx.flexconv_fwd(a[0], dev(pos + shift), *a[1:], layout=fx.BNC)
    gf0, gt0, gb0 = fx.flexconv_bwd(a[0], dev(pos), *a[1:], to_layout(g, fx.BNC), layout=fx.BNC)
    gf1, gt1, gb1 = fx.flexconv_bwd(a[0], dev(pos + shift), *a[1:], to_layout(g, fx.BNC), layout=fx.BNC)
    torch.cuda.synchronize()
    assert torch.equal(out0, out1) and torch.equal(gf0, gf1) and torch.equal(gt0, gt1) and torch.equal(gb0, gb1)


def test_slot_permutation_and_relabelling():
    B, N, K, Din, Dout = 2, 400, 8, 64, 64
    pos, nbr, feat, theta, bias, g = random_problem(3, B, N, K, Din, Dout, local=False)
    rng = np.random.default_rng(5)
    a = lambda p, n, f: (to_layout(f, fx.BNC), dev(p), dev(n), dev(theta), dev(bias))
    out = fx.flexconv_fwd(*a(pos, nbr, feat), layout=fx.BNC)
    po, pa = fx.flexpool_fwd(to_layout(feat, fx.BNC), dev(nbr), layout=fx.BNC)
    # a different slot order per point: same sums (other rounding order), same pooling result bit for bit
    perm = np.argsort(rng.random((B, K, N)), axis=1)
    nbr2 = np.take_along_axis(nbr, perm, axis=1)
    out2 = fx.flexconv_fwd(*a(pos, nbr2, feat), layout=fx.BNC)
    po2, pa2 = fx.flexpool_fwd(to_layout(feat, fx.BNC), dev(nbr2), layout=fx.BNC)
    torch.cuda.synchronize()
    assert rel_err(from_layout(out2, fx.BNC), from_layout(out, fx.BNC)) <= 1e-5
    assert torch.equal(po, po2) and torch.equal(pa, pa2)
    # relabelling the points of each cloud permutes the outputs the same way
    sigma = np.stack([rng.permutation(N) for _ in range(B)])            # new index -> old index
    inv = np.argsort(sigma, axis=1)                                     # old index -> new index
    pos3 = np.take_along_axis(pos, sigma[:, None, :], axis=2)
    feat3 = np.take_along_axis(feat, sigma[:, None, :], axis=2)
    nbr3 = np.stack([inv[b][nbr[b][:, sigma[b]]] for b in range(B)]).astype(np.int32)
    out3 = fx.flexconv_fwd(*a(pos3, nbr3, feat3), layout=fx.BNC)
    torch.cuda.synchronize()
    want = np.take_along_axis(from_layout(out, fx.BNC), sigma[:, None, :], axis=2)
    assert rel_err(from_layout(out3, fx.BNC), want) <= 1e-5


def test_layouts_agree():
    B, N, K, Din, Dout = 2, 333, 8, 64, 64
    pos, nbr, feat, theta, bias, g = random_problem(9, B, N, K, Din, Dout)
    res = {}
    for layout in (fx.BNC, fx.BCN):
        a = (to_layout(feat, layout), dev(pos), dev(nbr), dev(theta), dev(bias))
        out = fx.flexconv_fwd(*a, layout=layout)
        gf, gt, gb = fx.flexconv_bwd(*a, to_layout(g, layout), layout=layout)
        gp = fx.flexconv_bwd_pos(a[0], a[2], a[3], to_layout(g, layout), layout=layout)
        torch.cuda.synchronize()
        res[layout] = (from_layout(out, layout), from_layout(gf, layout), gt.cpu().numpy(), gb.cpu().numpy(), gp.cpu().numpy())
    for x, y in zip(res[fx.BNC], res[fx.BCN]):
        assert rel_err(x, y) <= 1e-5
