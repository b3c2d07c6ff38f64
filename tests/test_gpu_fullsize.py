"""GPU parity at the full sizes of configs 2-4, in the launch configuration bench.py times
(point-major layout, Z-order points, prebuilt in-edge lists): the forward pass and pooling on every
point of the cloud against the oracle (a slice plus at least 10^5 random points should the oracle
outrun its time budget), the feature gradient on more than 10^5 random rows, the parameter
gradients in full, the channel-major entry against the point-major result on whole tensors, and
properties that hold at any size."""
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


ORACLE_BUDGET_S = 100.0      # per oracle-checked tensor; beyond it the check falls back to a slice plus random ranges


class _Work:
    pass


@pytest.fixture(scope="module", params=[2, 3, 4], ids=["cfg2", "cfg3", "cfg4"])
def work(request):
    """One configuration's inputs on the host (as the oracle takes them) and on the device (point-major, Z-order
    points, prebuilt in-edge lists: the launch configuration bench.py times).  Built once per configuration."""
    ci = request.param
    cfg = CONFIGS[ci]
    say(f"config {ci}: {cfg.name} generating inputs")
    w = _Work()
    w.ci, w.cfg = ci, cfg
    w.x = make_inputs(cfg, with_grad=("conv_bwd" in cfg.runs))
    w.feat, w.pos, w.nbr = bnc(w.x.feat), dev(w.x.pos), dev(w.x.nbr)
    w.theta, w.bias = dev(w.x.theta), dev(w.x.bias)
    w.g = bnc(w.x.grad_out) if w.x.grad_out is not None else None
    w.edges = fx.flex_inedges_build(w.nbr)
    w.rng = np.random.default_rng(100 + ci)
    assert fx.flex_validate_neighbors(w.nbr) == 0
    yield w
    del w.feat, w.pos, w.nbr, w.g, w.edges, w.x
    torch.cuda.empty_cache()


def check_all_points(N, rng, what, got_cols, ref_cols, chunk=1 << 19):
    """Element-by-element check of a per-centre output over ALL points of the cloud, chunk by chunk, while the
    oracle keeps within its time budget; if it does not, what is left is checked on the points of the first
    sixteenth of the cloud plus at least 10^5 points in random ranges.  got_cols(l0, l1) / ref_cols(l0, l1) return
    the [B,C,l1-l0] columns of the device result / of the oracle.  Returns (checked points, max relative error
    with the RMS of the checked reference as the floor)."""
    import time
    t0 = time.time()
    refs, gots, spans = [], [], []
    l0, full = 0, True
    while l0 < N:
        l1 = min(N, l0 + chunk)
        refs.append(ref_cols(l0, l1))
        gots.append(got_cols(l0, l1))
        spans.append((l0, l1))
        l0 = l1
        elapsed = time.time() - t0
        if l0 < N and elapsed * (N / l0) > ORACLE_BUDGET_S and l0 >= N // 16:
            full = False
            break
    if not full:
        width = 256
        for s0 in rng.integers(l0, N - width, size=(100_000 + width - 1) // width):
            refs.append(ref_cols(int(s0), int(s0) + width))
            gots.append(got_cols(int(s0), int(s0) + width))
            spans.append((int(s0), int(s0) + width))
    points = sum(b - a for a, b in spans)
    say(f"  {what}: {'all' if full else 'first slice + random ranges:'} {points} points checked against the oracle "
        f"in {time.time() - t0:.1f}s")
    return points, refs, gots


def max_rel_err(refs, gots):
    sq = sum(float(np.sum(np.square(r, dtype=np.float64))) for r in refs)
    n = sum(r.size for r in refs)
    rms = np.sqrt(sq / max(n, 1))
    worst = 0.0
    for r, g in zip(refs, gots):
        r = np.asarray(r, np.float64)
        worst = max(worst, float(np.max(np.abs(np.asarray(g, np.float64) - r) / np.maximum(np.abs(r), rms))))
    return worst


def test_neighbour_search_agrees_with_the_harness(work):
    # the workload's neighbour tensor comes from an independent exact search on the CPU (float64 distances): the
    # neighbourhoods must agree as sets (a float32 / float64 rounding difference could swap a K-th neighbour)
    knn = fx.flex_knn(work.pos, work.cfg.K)
    agree = (torch.sort(knn, 1).values == torch.sort(work.nbr, 1).values).all(1).float().mean().item()
    say(f"  neighbourhoods equal to the harness's: {agree:.6f}")
    assert agree >= 0.99999


def test_forward_every_point(work):
    x, N = work.x, work.cfg.N
    out = fx.flexconv_fwd(work.feat, work.pos, work.nbr, work.theta, work.bias, layout=fx.BNC)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    points, refs, gots = check_all_points(
        N, work.rng, "forward",
        lambda a, b: out[:, a:b, :].transpose(1, 2).cpu().numpy(),
        lambda a, b: oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias, l_range=(a, b)))
    err = max_rel_err(refs, gots)
    say(f"  forward rel err {err:.2e}")
    assert points >= min(N, N // 16 + 100_000) and err <= TOL
    del refs, gots
    # the channel-major entry (transposed copies, other kernels for 128 -> 128) against the point-major result
    out_c = fx.flexconv_fwd(work.feat.transpose(1, 2).contiguous(), work.pos, work.nbr, work.theta, work.bias,
                            layout=fx.BCN)
    torch.cuda.synchronize()
    scale = float(out.double().pow(2).mean().sqrt())
    diff = float((out_c.transpose(1, 2) - out).abs().max())
    say(f"  channel-major vs point-major: max |diff| / RMS = {diff / scale:.2e}")
    assert diff <= 2e-6 * scale


def test_backward_rows_and_parameter_gradients(work):
    if "conv_bwd" not in work.cfg.runs:
        pytest.skip("forward-only configuration")
    x, cfg, rng = work.x, work.cfg, work.rng
    B, N, K, Din = cfg.B, cfg.N, cfg.K, cfg.Din
    gf, gt, gb = fx.flexconv_bwd(work.feat, work.pos, work.nbr, work.theta, work.bias, work.g, layout=fx.BNC,
                                 in_edges=work.edges)
    torch.cuda.synchronize()
    off = work.edges[0].cpu().numpy()
    assert off[0] == 0 and off[-1] == B * K * N and (np.diff(off) >= 0).all()
    # feature gradient: at least 10^5 random rows, the two ends and the point with the longest in-edge list
    targets = np.unique(np.concatenate([rng.integers(0, B * N, size=120_000), [0, B * N - 1],
                                        [int(np.argmax(np.diff(off)))]])).astype(np.int64)
    assert targets.size >= 100_000
    ref_rows = oracle.flexconv_grad_feat_at(x.pos, x.nbr, x.theta, x.bias, x.grad_out, targets)
    got_rows = gf.reshape(B * N, Din)[torch.from_numpy(targets).cuda()].cpu().numpy()
    e_gf = rel_err(got_rows, ref_rows)
    # parameter gradients: every element, the oracle summing over every point
    _, rgt, rgb = oracle.flexconv_bwd(x.feat, x.pos, x.nbr, x.theta, x.bias, x.grad_out, want_feat=False)
    e_gt, e_gb = rel_err(gt.cpu().numpy(), rgt), rel_err(gb.cpu().numpy(), rgb)
    say(f"  grad_feat ({targets.size} rows) {e_gf:.2e}  grad_theta {e_gt:.2e}  grad_bias {e_gb:.2e}")
    assert max(e_gf, e_gt, e_gb) <= TOL
    # adjoint identity over the whole cloud: <g, fwd(v)> == <grad_feat, v>
    v = torch.randn(work.feat.shape, device="cuda", generator=torch.Generator("cuda").manual_seed(work.ci))
    lhs = float((fx.flexconv_fwd(v, work.pos, work.nbr, work.theta, work.bias, layout=fx.BNC).double()
                 * work.g.double()).sum())
    rhs = float((gf.double() * v.double()).sum())
    assert abs(lhs - rhs) <= 1e-4 * max(abs(lhs), float(work.g.double().norm() * v.double().norm()) * 1e-3)
    del v
    # channel-major entry (in-edge lists built inside the call) against the point-major result, whole tensors
    gf_c, gt_c, gb_c = fx.flexconv_bwd(work.feat.transpose(1, 2).contiguous(), work.pos, work.nbr, work.theta,
                                       work.bias, work.g.transpose(1, 2).contiguous(), layout=fx.BCN)
    torch.cuda.synchronize()
    s_gf = float(gf.double().pow(2).mean().sqrt())
    assert float((gf_c.transpose(1, 2) - gf).abs().max()) <= 2e-6 * s_gf
    assert rel_err(gt_c.cpu().numpy(), rgt) <= TOL and rel_err(gb_c.cpu().numpy(), rgb) <= TOL


def test_pooling_every_point(work):
    if "pool_fwd" not in work.cfg.runs:
        pytest.skip("configuration without pooling")
    x, cfg, rng = work.x, work.cfg, work.rng
    N, K = cfg.N, cfg.K
    feat = work.feat
    po, pa = fx.flexpool_fwd(feat, work.nbr, layout=fx.BNC)
    torch.cuda.synchronize()
    # every point against the oracle, bit for bit
    ro, ra = oracle.flexpool_fwd(x.feat, x.nbr)
    assert torch.equal(pa.transpose(1, 2).cpu(), torch.from_numpy(ra))
    assert torch.equal(po.transpose(1, 2).cpu().view(torch.int32), torch.from_numpy(ro).view(torch.int32))
    del ro
    # the form bench.py times: through the static gather plan; the same comparisons in the same order
    fplan = fx.flexpool_fwd_plan_build(work.nbr)
    ppo, ppa = fx.flexpool_fwd_planned(feat, work.nbr, fplan, layout=fx.BNC)
    torch.cuda.synchronize()
    assert torch.equal(ppa, pa) and torch.equal(ppo.view(torch.int32), po.view(torch.int32))
    del ppo, ppa, fplan
    gp = work.g if work.g is not None and cfg.Din == cfg.Dout else torch.randn_like(feat)
    pg = fx.flexpool_bwd(gp, pa, layout=fx.BNC, in_edges=work.edges)
    pg_scatter = fx.flexpool_bwd(gp, pa, layout=fx.BNC)
    # the form bench.py times: through the static gather plan; the same sums in the same order as the list form
    plan = fx.flexpool_plan_build(work.edges, cfg.B, N)
    pg_planned = fx.flexpool_bwd_planned(gp, pa, work.edges, plan, layout=fx.BNC)
    torch.cuda.synchronize()
    assert torch.equal(pg_planned.view(torch.int32), pg.view(torch.int32))
    del pg_planned, plan
    assert float((pg - pg_scatter).abs().max()) <= 1e-4 * float(gp.abs().max()) * K
    del pg_scatter
    # every element of the backward pass against the oracle's routing by its own table
    ref = oracle.flexpool_bwd(gp.transpose(1, 2).contiguous().cpu().numpy(), ra)
    assert rel_err(pg.transpose(1, 2).cpu().numpy(), ref) <= 1e-5
    del ref, ra
    # the channel-major kernels at this size: same winners, same bits; the gather sums in the same (list) order
    say("  pooling, channel-major")
    po_c, pa_c = fx.flexpool_fwd(feat.transpose(1, 2).contiguous(), work.nbr, layout=fx.BCN)
    assert torch.equal(pa_c.transpose(1, 2), pa)
    assert torch.equal(po_c.transpose(1, 2).view(torch.int32), po.view(torch.int32))
    del po_c
    pg_c = fx.flexpool_bwd(gp.transpose(1, 2).contiguous(), pa_c, layout=fx.BCN, in_edges=work.edges)
    torch.cuda.synchronize()
    assert torch.equal(pg_c.transpose(1, 2), pg)


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
