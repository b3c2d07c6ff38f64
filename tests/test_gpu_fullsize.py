"""GPU parity at the full sizes of configs 2-4, in the launch configuration bench.py times
(point-major layout, Z-order points, prebuilt in-edge lists): sampled outputs the oracle can
compute one by one, full parameter gradients, and properties that hold at any size."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, dev, say
from helpers import rel_err
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def bnc(a):
    return torch.from_numpy(a).cuda().transpose(1, 2).contiguous()


def sample_ranges(N, rng, width=272):
    starts = [0, N // 2 - 7, N - width] + [int(v) for v in rng.integers(0, N - width, size=2)]
    return [(s, s + width) for s in starts]


@pytest.mark.parametrize("ci", [2, 3, 4])
def test_full_size_config(ci):
    cfg = CONFIGS[ci]
    say(f"config {ci}: {cfg.name} generating inputs")
    x = make_inputs(cfg, with_grad=("conv_bwd" in cfg.runs))
    B, N, K, Din, Dout = cfg.B, cfg.N, cfg.K, cfg.Din, cfg.Dout
    rng = np.random.default_rng(100 + ci)
    feat, pos, nbr, theta, bias = bnc(x.feat), dev(x.pos), dev(x.nbr), dev(x.theta), dev(x.bias)
    assert fx.flex_validate_neighbors(nbr) == 0

    say("  k-nearest neighbours on the GPU")
    # the workload's neighbour tensor comes from an independent exact search on the CPU (float64 distances): the
    # neighbourhoods must agree as sets (a float32 / float64 rounding difference could swap a K-th neighbour)
    knn = fx.flex_knn(pos, K)
    agree = (torch.sort(knn, 1).values == torch.sort(nbr, 1).values).all(1).float().mean().item()
    say(f"  neighbourhoods equal to the harness's: {agree:.6f}")
    assert agree >= 0.99999
    del knn

    say("  forward")
    out = fx.flexconv_fwd(feat, pos, nbr, theta, bias, layout=fx.BNC)
    torch.cuda.synchronize()
    worst = 0.0
    for (s0, s1) in sample_ranges(N, rng):
        ref = oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias, l_range=(s0, s1))
        got = out[:, s0:s1, :].transpose(1, 2).cpu().numpy()
        worst = max(worst, rel_err(got, ref))
    say(f"  fwd sampled rel err {worst:.2e}")
    assert worst <= TOL
    assert bool(torch.isfinite(out).all())

    if "conv_bwd" in cfg.runs:
        say("  backward")
        g = bnc(x.grad_out)
        edges = fx.flex_inedges_build(nbr)
        gf, gt, gb = fx.flexconv_bwd(feat, pos, nbr, theta, bias, g, layout=fx.BNC, in_edges=edges)
        torch.cuda.synchronize()
        off = edges[0].cpu().numpy()
        assert off[0] == 0 and off[-1] == B * K * N and (np.diff(off) >= 0).all()
        targets = np.unique(np.concatenate([rng.integers(0, B * N, size=500), [0, B * N - 1],
                                            [int(np.argmax(np.diff(off)))]])).astype(np.int64)
        ref_rows = oracle.flexconv_grad_feat_at(x.pos, x.nbr, x.theta, x.bias, x.grad_out, targets)
        got_rows = gf.reshape(B * N, Din)[torch.from_numpy(targets).cuda()].cpu().numpy()
        e_gf = rel_err(got_rows, ref_rows)
        _, rgt, rgb = oracle.flexconv_bwd(x.feat, x.pos, x.nbr, x.theta, x.bias, x.grad_out, want_feat=False)
        e_gt, e_gb = rel_err(gt.cpu().numpy(), rgt), rel_err(gb.cpu().numpy(), rgb)
        say(f"  grad_feat (sampled) {e_gf:.2e}  grad_theta {e_gt:.2e}  grad_bias {e_gb:.2e}")
        assert max(e_gf, e_gt, e_gb) <= TOL
        # adjoint identity at full size: <g, fwd(v)> == <grad_feat, v>
        v = torch.randn(feat.shape, device="cuda", generator=torch.Generator("cuda").manual_seed(ci))
        lhs = float((fx.flexconv_fwd(v, pos, nbr, theta, bias, layout=fx.BNC).double() * g.double()).sum())
        rhs = float((gf.double() * v.double()).sum())
        assert abs(lhs - rhs) <= 1e-4 * max(abs(lhs), float(g.double().norm() * v.double().norm()) * 1e-3)
        del v

    if "pool_fwd" in cfg.runs:
        say("  pooling")
        po, pa = fx.flexpool_fwd(feat, nbr, layout=fx.BNC)
        torch.cuda.synchronize()
        for (s0, s1) in sample_ranges(N, rng):
            ro, ra = oracle.flexpool_fwd(x.feat, x.nbr, l_range=(s0, s1))
            assert np.array_equal(pa[:, s0:s1, :].transpose(1, 2).cpu().numpy(), ra)
            assert np.array_equal(po[:, s0:s1, :].transpose(1, 2).cpu().numpy().view(np.uint32), ro.view(np.uint32))
        # everywhere: the value is the winner's, bit for bit, and self (slot 0 here) never beats it
        gathered = torch.gather(feat, 1, pa.long())
        assert torch.equal(gathered.view(torch.int32), po.view(torch.int32))
        assert bool((po >= feat).all())
        del gathered
        gp = bnc(x.grad_out) if x.grad_out is not None and Din == Dout else torch.randn_like(feat)
        pool_edges = edges if "conv_bwd" in cfg.runs else fx.flex_inedges_build(nbr)
        pg = fx.flexpool_bwd(gp, pa, layout=fx.BNC, in_edges=pool_edges)     # the form bench.py times
        pg_scatter = fx.flexpool_bwd(gp, pa, layout=fx.BNC)
        torch.cuda.synchronize()
        assert float((pg - pg_scatter).abs().max()) <= 1e-4 * float(gp.abs().max()) * K
        # mass conservation per (cloud, channel) and exact rows on a sample
        m_got, m_ref = pg.double().sum(1).cpu().numpy(), gp.double().sum(1).cpu().numpy()
        assert np.abs(m_got - m_ref).max() <= 1e-6 * gp.double().abs().sum(1).max().item()
        ref = oracle.flexpool_bwd(gp.transpose(1, 2).contiguous().cpu().numpy(), pa.transpose(1, 2).contiguous().cpu().numpy())
        cols = rng.integers(0, N, size=4000)
        assert rel_err(pg[:, torch.from_numpy(cols).cuda(), :].transpose(1, 2).cpu().numpy(), ref[:, :, cols]) <= 1e-5
        # the channel-major kernels at this size: same winners, same bits; the gather sums in the same (list) order
        say("  pooling, channel-major")
        po_c, pa_c = fx.flexpool_fwd(feat.transpose(1, 2).contiguous(), nbr, layout=fx.BCN)
        assert torch.equal(pa_c.transpose(1, 2), pa)
        assert torch.equal(po_c.transpose(1, 2).view(torch.int32), po.view(torch.int32))
        del po_c
        pg_c = fx.flexpool_bwd(gp.transpose(1, 2).contiguous(), pa_c, layout=fx.BCN, in_edges=pool_edges)
        torch.cuda.synchronize()
        assert torch.equal(pg_c.transpose(1, 2), pg)
        del pg_c, pa_c


def test_wide_layer_at_a_deeper_stage_size():
    """256 -> 256 on 200 000 room points (the shape of a deeper stage of the paper's network): the block-pass kernels
    at a size where every workgroup walks many tiles in every pass."""
    from workloads.configs import Config
    base = CONFIGS[3]
    cfg = Config(**{**base.__dict__, "N": 200_000, "Din": 256, "Dout": 256, "name": "room200k_256x256"})
    say("wide layer: generating inputs")
    x = make_inputs(cfg)
    B, N, K, Din, Dout = cfg.B, cfg.N, cfg.K, cfg.Din, cfg.Dout
    rng = np.random.default_rng(321)
    feat, pos, nbr, theta, bias, g = bnc(x.feat), dev(x.pos), dev(x.nbr), dev(x.theta), dev(x.bias), bnc(x.grad_out)
    edges = fx.flex_inedges_build(nbr)
    out = fx.flexconv_fwd(feat, pos, nbr, theta, bias, layout=fx.BNC)
    gf, gt, gb = fx.flexconv_bwd(feat, pos, nbr, theta, bias, g, layout=fx.BNC, in_edges=edges)
    torch.cuda.synchronize()
    say("  forward, sampled")
    for (s0, s1) in sample_ranges(N, rng):
        ref = oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias, l_range=(s0, s1))
        assert rel_err(out[:, s0:s1, :].transpose(1, 2).cpu().numpy(), ref) <= TOL
    say("  feature gradient, sampled")
    targets = np.unique(np.concatenate([rng.integers(0, B * N, size=300), [0, B * N - 1]])).astype(np.int64)
    ref_rows = oracle.flexconv_grad_feat_at(x.pos, x.nbr, x.theta, x.bias, x.grad_out, targets)
    assert rel_err(gf.reshape(B * N, Din)[torch.from_numpy(targets).cuda()].cpu().numpy(), ref_rows) <= TOL
    say("  parameter gradients, block by block against the 64 -> 64 kernels on contiguous slices")
    for (hi, ho) in [(0, 0), (3, 1), (2, 3)]:
        f_blk = feat[:, :, 64 * hi:64 * hi + 64].contiguous()
        g_blk = g[:, :, 64 * ho:64 * ho + 64].contiguous()
        t_blk = theta[:, 64 * hi:64 * hi + 64, 64 * ho:64 * ho + 64].contiguous()
        b_blk = bias[64 * hi:64 * hi + 64, 64 * ho:64 * ho + 64].contiguous()
        _, rt, rb = fx.flexconv_bwd(f_blk, pos, nbr, t_blk, b_blk, g_blk, layout=fx.BNC, need_feat=False)
        assert rel_err(gt[:, 64 * hi:64 * hi + 64, 64 * ho:64 * ho + 64].cpu().numpy(), rt.cpu().numpy()) <= TOL
        assert rel_err(gb[64 * hi:64 * hi + 64, 64 * ho:64 * ho + 64].cpu().numpy(), rb.cpu().numpy()) <= TOL
    # and one block against the oracle itself
    say("  one parameter block against the oracle")
    _, ot, ob = oracle.flexconv_bwd(np.ascontiguousarray(x.feat[:, 64:128]), x.pos, x.nbr,
                                    np.ascontiguousarray(x.theta[:, 64:128, 128:192]),
                                    np.ascontiguousarray(x.bias[64:128, 128:192]),
                                    np.ascontiguousarray(x.grad_out[:, 128:192]), want_feat=False)
    assert rel_err(gt[:, 64:128, 128:192].cpu().numpy(), ot) <= TOL
    assert rel_err(gb[64:128, 128:192].cpu().numpy(), ob) <= TOL
