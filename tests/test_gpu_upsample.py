"""GPU parity for flex-upsampling: forward bit-exact against the CPU oracle (values and winners),
backward within the pooling-backward tolerance, both layouts, ragged sizes, and the selection check."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import dev, to_layout, from_layout, say
from helpers import rel_err
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1000, 250, 8, 64), (2, 77, 20, 3, 32), (1, 130, 130, 16, 128), (2, 150, 37, 6, 5), (1, 64, 1, 1, 9)]


@pytest.mark.parametrize("layout", [fx.BNC, fx.BCN], ids=["bnc", "bcn"])
@pytest.mark.parametrize("B,Nf,Ns,K,C", SHAPES)
def test_flexupsample_matches_oracle(B, Nf, Ns, K, C, layout):
    say(f"upsample B={B} Nf={Nf} Ns={Ns} K={K} C={C} layout={layout}")
    rng = np.random.default_rng(Nf + C)
    feat = rng.integers(-2, 3, size=(B, C, Ns)).astype(np.float32)          # ties with the zero fill
    feat[:, :, ::5] = rng.standard_normal(feat[:, :, ::5].shape).astype(np.float32)
    feat[:, :, 1::7] = -0.0
    sel = np.stack([rng.permutation(Nf)[:Ns] for _ in range(B)]).astype(np.int32)
    nbr = rng.integers(0, Nf, size=(B, K, Nf)).astype(np.int32)
    g = rng.standard_normal((B, C, Nf)).astype(np.float32)
    ro, ra = oracle.flexupsample_fwd(feat, sel, nbr)
    dsel, dnbr = dev(sel), dev(nbr)
    assert fx.flex_validate_selection(dsel, Nf) == 0
    out, arg = fx.flexupsample_fwd(to_layout(feat, layout), dsel, dnbr, layout=layout)
    edges = fx.flex_inedges_build(dnbr)
    gs = fx.flexupsample_bwd(to_layout(g, layout), arg, dsel, edges, layout=layout)
    gs2 = fx.flexupsample_bwd(to_layout(g, layout), arg, dsel, edges, layout=layout)
    torch.cuda.synchronize()
    assert np.array_equal(from_layout(arg, layout), ra)
    assert np.array_equal(from_layout(out, layout).view(np.uint32), ro.view(np.uint32))
    assert rel_err(from_layout(gs, layout), oracle.flexupsample_bwd(g, ra, sel)) <= 1e-5
    assert torch.equal(gs, gs2)                                               # fixed summation order


def test_selection_check_counts_bad_entries():
    sel = np.stack([np.arange(10), np.arange(10) + 3]).astype(np.int32)
    assert fx.flex_validate_selection(dev(sel), 40) == 0
    sel[0, 4] = sel[0, 2]          # repeated
    sel[1, 0] = 40                 # out of range
    sel[1, 1] = -1
    assert fx.flex_validate_selection(dev(sel), 40) == 3


def test_flexupsample_room_scale():
    """A room cloud of 200k points, every 4th point (random choice) kept in the smaller layer, 128 channels:
    the shape of a decoder stage (the resolution drops by a factor 4 per stage)."""
    cfg = CONFIGS[3]
    x = make_inputs(cfg, with_grad=False, n_override=200_000)
    Nf, K, C = 200_000, cfg.K, 128
    rng = np.random.default_rng(11)
    Ns = Nf // 4
    sel = np.sort(rng.permutation(Nf)[:Ns]).astype(np.int32)[None]
    feat = rng.standard_normal((1, C, Ns)).astype(np.float32)
    g = rng.standard_normal((1, C, Nf)).astype(np.float32)
    ro, ra = oracle.flexupsample_fwd(feat, sel, x.nbr)
    dnbr, dsel = dev(x.nbr), dev(sel)
    out, arg = fx.flexupsample_fwd(to_layout(feat, fx.BNC), dsel, dnbr, layout=fx.BNC)
    gs = fx.flexupsample_bwd(to_layout(g, fx.BNC), arg, dsel, fx.flex_inedges_build(dnbr), layout=fx.BNC)
    torch.cuda.synchronize()
    assert np.array_equal(from_layout(arg, fx.BNC), ra)
    assert np.array_equal(from_layout(out, fx.BNC).view(np.uint32), ro.view(np.uint32))
    assert rel_err(from_layout(gs, fx.BNC), oracle.flexupsample_bwd(g, ra, sel)) <= 1e-5
