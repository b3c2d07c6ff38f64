"""GPU parity for flex-max-pooling with subsampling: forward bit-exact against the CPU oracle (values
and winners), backward within the pooling-backward tolerance in both forms (atomics, in-edge gather),
both layouts, ragged sizes, and agreement with the full pooling layer on the kept rows."""
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
@pytest.mark.parametrize("B,N,Ns,K,C", SHAPES)
def test_flexpool_sub_matches_oracle(B, N, Ns, K, C, layout):
    say(f"pool_sub B={B} N={N} Ns={Ns} K={K} C={C} layout={layout}")
    rng = np.random.default_rng(N + C)
    feat = rng.integers(-2, 3, size=(B, C, N)).astype(np.float32)            # many ties
    feat[:, :, ::5] = rng.standard_normal(feat[:, :, ::5].shape).astype(np.float32)
    feat[:, :, 1::7] = -0.0
    sel = np.stack([rng.permutation(N)[:Ns] for _ in range(B)]).astype(np.int32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    g = rng.standard_normal((B, C, Ns)).astype(np.float32)
    ro, ra = oracle.flexpool_sub_fwd(feat, nbr, sel)
    dsel, dnbr = dev(sel), dev(nbr)
    out, arg = fx.flexpool_sub_fwd(to_layout(feat, layout), dnbr, dsel, layout=layout)
    edges = fx.flex_inedges_build_sub(dnbr, dsel)
    dg = to_layout(g, layout)
    gf_gather = fx.flexpool_sub_bwd(dg, arg, N, layout=layout, in_edges=edges)
    gf_gather2 = fx.flexpool_sub_bwd(dg, arg, N, layout=layout, in_edges=edges)
    gf_atomic = fx.flexpool_sub_bwd(dg, arg, N, layout=layout)
    torch.cuda.synchronize()
    # the lists: for every point, the ascending rows j of the kept centres that name it, once per slot
    off, src = edges[0].cpu().numpy(), edges[1].cpu().numpy()
    for b in range(B):
        want = [[] for _ in range(N)]
        for j in range(Ns):
            for k in range(K):
                want[nbr[b, k, sel[b, j]]].append(j)
        for m in range(0, N, max(1, N // 50)):
            assert list(src[off[b * N + m]:off[b * N + m + 1]]) == sorted(want[m])
    assert np.array_equal(from_layout(arg, layout), ra)
    assert np.array_equal(from_layout(out, layout).view(np.uint32), ro.view(np.uint32))
    ref = oracle.flexpool_sub_bwd(g, ra, sel, N)
    assert rel_err(from_layout(gf_gather, layout), ref) <= 1e-5
    assert rel_err(from_layout(gf_atomic, layout), ref) <= 1e-5
    assert torch.equal(gf_gather, gf_gather2)                                  # fixed summation order


def test_flexpool_sub_equals_full_pooling_on_kept_rows():
    rng = np.random.default_rng(5)
    B, N, K, C, Ns = 2, 3000, 8, 64, 750
    feat = torch.from_numpy(rng.standard_normal((B, N, C)).astype(np.float32)).cuda()
    nbr = dev(rng.integers(0, N, size=(B, K, N)).astype(np.int32))
    sel = np.stack([np.sort(rng.permutation(N)[:Ns]) for _ in range(B)]).astype(np.int32)
    fo, fa = fx.flexpool_fwd(feat, nbr, layout=fx.BNC)
    so, sa = fx.flexpool_sub_fwd(feat, nbr, dev(sel), layout=fx.BNC)
    idx = torch.from_numpy(sel.astype(np.int64)).cuda()[:, :, None].expand(B, Ns, C)
    assert torch.equal(so, torch.gather(fo, 1, idx)) and torch.equal(sa, torch.gather(fa, 1, idx))


def test_flexpool_sub_room_scale():
    """A room cloud of 200k points, a quarter of them kept (the encoder's reduction per stage), 128 channels."""
    cfg = CONFIGS[3]
    x = make_inputs(cfg, with_grad=False, n_override=200_000)
    N, C = 200_000, 128
    rng = np.random.default_rng(12)
    Ns = N // 4
    sel = np.sort(rng.permutation(N)[:Ns]).astype(np.int32)[None]
    feat = rng.standard_normal((1, C, N)).astype(np.float32)
    g = rng.standard_normal((1, C, Ns)).astype(np.float32)
    ro, ra = oracle.flexpool_sub_fwd(feat, x.nbr, sel)
    dnbr, dsel = dev(x.nbr), dev(sel)
    out, arg = fx.flexpool_sub_fwd(to_layout(feat, fx.BNC), dnbr, dsel, layout=fx.BNC)
    gf = fx.flexpool_sub_bwd(to_layout(g, fx.BNC), arg, N, layout=fx.BNC,
                             in_edges=fx.flex_inedges_build_sub(dnbr, dsel))
    torch.cuda.synchronize()
    assert np.array_equal(from_layout(arg, fx.BNC), ra)
    assert np.array_equal(from_layout(out, fx.BNC).view(np.uint32), ro.view(np.uint32))
    assert rel_err(from_layout(gf, fx.BNC), oracle.flexpool_sub_bwd(g, ra, sel, N)) <= 1e-5
