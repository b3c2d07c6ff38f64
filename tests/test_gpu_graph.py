"""The entry points enqueue kernels only (no allocation, no synchronisation, no memset nodes), so a whole
layer step can be captured into a HIP graph and replayed.  Every replay is checked against the eager result,
with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import paper_1803_07289_amd as fx
from gpu_util import dev, to_layout, say
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg_i,n,widths", [(1, None, None), (0, 3000, None), (0, 2000, (256, 128)), (0, 1500, (20, 13))],
                         ids=["config1", "config0", "wide_256x128", "padded_20x13"])
def test_layer_step_replays_from_a_graph(cfg_i, n, widths):
    cfg = CONFIGS[cfg_i]
    if widths is not None:      # block passes / zero-padded copies: more kernels per entry point, still kernels only
        cfg = type(cfg)(**{**cfg.__dict__, "Din": widths[0], "Dout": widths[1]})
    x = make_inputs(cfg, n_override=n)
    say(f"graph capture {x.cfg.name} N={x.cfg.N}")
    L = fx.BNC
    feat, g = to_layout(x.feat, L), to_layout(x.grad_out, L)
    pos, nbr, theta, bias = dev(x.pos), dev(x.nbr), dev(x.theta), dev(x.bias)
    edges = fx.flex_inedges_build(nbr)
    gpool = torch.randn_like(feat)

    def step():
        out = fx.flexconv_fwd(feat, pos, nbr, theta, bias, layout=L)
        gf, gt, gb = fx.flexconv_bwd(feat, pos, nbr, theta, bias, g, layout=L, in_edges=edges)
        po, pa = fx.flexpool_fwd(feat, nbr, layout=L)
        pg = fx.flexpool_bwd(gpool, pa, layout=L, in_edges=edges)
        return out, gf, gt, gb, po, pa, pg

    eager = [t.clone() for t in step()]            # also sizes the cached workspaces before capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = step()
    for r in range(3):
        for t in captured:
            t.fill_(7) if t.dtype == torch.int32 else t.fill_(float("nan"))     # stale results must be overwritten
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(captured, eager):
            assert torch.equal(a, b), f"replay {r}"
        _ = fx.flexconv_fwd(feat, pos, nbr, theta, bias, layout=L)            # eager work between the replays
        torch.cuda.synchronize()


def test_planned_pooling_replays_from_a_graph():
    """flexpool_fwd_planned and flexpool_bwd_planned = a fill kernel (the tile counters) and two kernels each:
    capturable like the rest; a cloud large enough for the planned kernels to be the ones that run."""
    B, N, K, C = 1, 600_000, 8, 64
    say(f"graph capture of the planned pooling passes, N={N}")
    rng = np.random.default_rng(1)
    nbr = dev(((np.arange(N)[None, None, :] + rng.integers(-20, 21, size=(B, K, N))) % N).astype(np.int32))
    feat = torch.randn(B, N, C, device="cuda")
    gpool = torch.randn_like(feat)
    edges = fx.flex_inedges_build(nbr)
    plan = fx.flexpool_plan_build(edges, B, N)
    fplan = fx.flexpool_fwd_plan_build(nbr)

    def step():
        po, pa = fx.flexpool_fwd_planned(feat, nbr, fplan, layout=fx.BNC)
        return po, pa, fx.flexpool_bwd_planned(gpool, pa, edges, plan, layout=fx.BNC)

    eager = [t.clone() for t in step()]
    plain = fx.flexpool_fwd(feat, nbr, layout=fx.BNC)
    listed = fx.flexpool_bwd(gpool, eager[1], layout=fx.BNC, in_edges=edges)
    torch.cuda.synchronize()
    assert torch.equal(plain[0].view(torch.int32), eager[0].view(torch.int32)) and torch.equal(plain[1], eager[1])
    assert torch.equal(listed.view(torch.int32), eager[2].view(torch.int32))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = step()
    for r in range(3):
        for t in captured:
            t.fill_(7) if t.dtype == torch.int32 else t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(captured, eager):
            assert torch.equal(a, b), f"replay {r}"
        _ = fx.flexpool_bwd_planned(gpool, eager[1], edges, plan, layout=fx.BNC)    # eager work between the replays
        torch.cuda.synchronize()
