"""GPU parity for flex-max-pooling through the static gather plans.  Backward (flexpool_plan_build,
flexpool_bwd_planned): the result must equal the list form of flexpool_bwd bit for bit (same sums, same order) and
the CPU oracle within the pooling-backward tolerance.  Forward (flexpool_fwd_plan_build, flexpool_fwd_planned): values
and winners must equal flexpool_fwd's bit for bit, and the oracle's.  The cases reach every branch of the planned kernels: tiles
whose rows are all staged, tiles with more distinct rows than the plan lists (entries fetched directly), tiles with
more entries than the plan covers (served entry by entry), lists longer than a row group's sixteen slot words,
repeated entries, ragged tails, several clouds, fewer tiles than workgroups; clouds without locality, where the
plans do not pay and the plain steps run in the planned ones' place (backward: a second kernel; forward: a branch of
the planned kernel); and the widths and layouts the plans have no kernel for, which run the plain kernels.  The planned kernels are chosen from 2^18 points on (the last three sizes);
test_gpu_fallbacks.py runs this file once more with FLEX_POOL_PLAN=1, which selects it at every size.  (The 7M-point configuration: test_gpu_fullsize.py.)"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import dev, to_layout, from_layout, say
from helpers import rel_err

pytestmark = pytest.mark.gpu


def lists(kind, rng, B, N, K):
    if kind == "random":                 # no locality: a tile of 32 points is listed by up to 32 K distinct centres
        return rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    near = ((np.arange(N)[None, None, :] + rng.integers(-20, 21, size=(B, K, N))) % N).astype(np.int32)
    if kind == "local":
        return near
    if kind == "hub":                    # one point listed by half the cloud (at most 5000 centres): its tile has far more than 512 entries
        near[:, 0, : min(N // 2, 5000)] = min(7, N - 1)
        return near
    if kind == "long_list":              # one point listed by 40 centres: more than sixteen entries, tile still covered
        near[:, 0, 100:140] = 105
        return near
    if kind == "scattered":              # 150 centres from all over the cloud list points of one tile: more distinct
        for b in range(B):               # rows than the plan lists, fewer entries than it covers
            who = rng.choice(N, 150, replace=False)
            near[b, 1, who] = rng.integers(320, 352, size=150)
        return near
    if kind == "repeats":                # every centre lists its first neighbour twice
        near[:, K - 1, :] = near[:, 0, :]
        return near
    if kind == "far":                    # the centres of one tile list points from all over the cloud: more distinct
        if K >= 6:                       # rows than the forward plan lists, fewer entries than it covers
            near[:, 1:6, 320:352] = rng.integers(0, N, size=(B, 5, 32))
        return near
    raise ValueError(kind)


def run_case(seed, B, N, K, C, layout, kind):
    rng = np.random.default_rng(seed)
    feat = rng.integers(-2, 3, size=(B, C, N)).astype(np.float32)            # many ties
    feat[:, :, ::3] = rng.standard_normal(feat[:, :, ::3].shape).astype(np.float32)
    g = rng.standard_normal((B, C, N)).astype(np.float32)
    nbr = lists(kind, rng, B, N, K)
    dn = dev(nbr)
    df = to_layout(feat, layout)
    out, arg = fx.flexpool_fwd(df, dn, layout=layout)
    fplan = fx.flexpool_fwd_plan_build(dn)
    for _ in range(2):
        pout, parg = fx.flexpool_fwd_planned(df, dn, fplan, layout=layout)
        torch.cuda.synchronize()
        assert torch.equal(arg, parg) and torch.equal(out.view(torch.int32), pout.view(torch.int32))
    ro, ra = oracle.flexpool_fwd(feat, nbr)
    assert np.array_equal(from_layout(pout, layout), ro.astype(np.float32))
    edges = fx.flex_inedges_build(dn)
    plan = fx.flexpool_plan_build(edges, B, N)
    dg = to_layout(g, layout)
    ref = fx.flexpool_bwd(dg, arg, layout=layout, in_edges=edges)
    got = fx.flexpool_bwd_planned(dg, arg, edges, plan, layout=layout)
    again = fx.flexpool_bwd_planned(dg, arg, edges, plan, layout=layout)
    torch.cuda.synchronize()
    assert torch.equal(ref.view(torch.int32), got.view(torch.int32)), float((ref - got).abs().max())
    assert torch.equal(got.view(torch.int32), again.view(torch.int32))
    assert np.array_equal(from_layout(arg, layout), ra)
    # fp32 sums in list order against the oracle's fp64: 1e-5 for neighbourhood-sized lists; the hub point adds up
    # N / 2 terms one after the other (about n 2^-24 of the sum of magnitudes: the list form's own accuracy)
    assert rel_err(from_layout(got, layout), oracle.flexpool_bwd(g, ra)) <= (1e-4 if kind == "hub" else 1e-5)
    return plan, fplan


@pytest.mark.parametrize("kind", ["local", "random", "hub", "long_list", "scattered", "repeats", "far"])
@pytest.mark.parametrize("B,N,K", [(1, 1, 1), (1, 31, 4), (2, 33, 8), (3, 1000, 8), (1, 5000, 16), (2, 4097, 9),
                                   (1, 70000, 8), (2, 300_001, 8), (1, 600_000, 9), (64, 9001, 8)])
def test_planned_backward_equals_the_list_form(B, N, K, kind):
    if kind in ("hub", "long_list", "scattered", "far") and N < 1000:
        pytest.skip("needs a cloud with room for the construction")
    say(f"pool plan: B={B} N={N} K={K} lists={kind}")
    plan, fplan = run_case(100 * N + K, B, N, K, 64, fx.BNC, kind)
    # what the plan says about its tiles: every branch of the kernel is reached by some case
    tiles = B * ((N + 31) // 32)
    cnt = plan[256:256 + 4 * tiles].view(torch.int32).cpu().numpy()
    uncovered = int(plan[:4].view(torch.int32).item())
    say(f"  tiles {tiles}: not covered {int((cnt < 0).sum())}, with direct entries {int(((cnt >= 0) & (cnt >= 2 ** 30)).sum())}"
        f" -> {'list form' if uncovered * 8 > tiles else 'planned kernel'}")
    assert uncovered == int(((cnt < 0) | (cnt >= 2 ** 30)).sum())
    if kind == "hub":                    # a few tiles served entry by entry inside the planned kernel
        assert (cnt < 0).any() and (K > 9 or uncovered * 8 <= tiles)
    if kind == "scattered" and K <= 9:   # a few tiles with entries fetched directly inside the planned kernel
        assert ((cnt >= 0) & (cnt >= 2 ** 30)).any() and uncovered * 8 <= tiles
    if kind == "random" and N >= 1000:   # no locality at all: the plan does not pay, the list form runs
        assert uncovered * 8 > tiles
    if kind == "local" and K <= 9:       # the paper's neighbourhood sizes: every row of every tile is staged
        assert (cnt >= 0).all() and (cnt < 2 ** 30).all()
    # the forward plan: the same header over the neighbour lists themselves
    fcnt = fplan[256:256 + 4 * tiles].view(torch.int32).cpu().numpy()
    funcovered = int(fplan[:4].view(torch.int32).item())
    say(f"  forward: not covered {int((fcnt < 0).sum())}, with direct entries {int(((fcnt >= 0) & (fcnt >= 2 ** 30)).sum())}"
        f" -> {'plain kernel' if funcovered * 8 > tiles else 'planned kernel'}")
    assert funcovered == int(((fcnt < 0) | (fcnt >= 2 ** 30)).sum())
    if kind == "far" and 6 <= K <= 9:    # one tile per cloud fetches rows directly inside the planned kernel
        assert ((fcnt >= 0) & (fcnt >= 2 ** 30)).sum() >= B and funcovered * 8 <= tiles
    if kind == "random" and N >= 1000:
        assert funcovered * 8 > tiles
    if kind in ("local", "hub", "long_list", "scattered", "repeats") and K <= 9:
        assert (fcnt >= 0).all() and (fcnt < 2 ** 30).all()


@pytest.mark.parametrize("C,layout,K", [(64, fx.BCN, 8), (32, fx.BNC, 8), (192, fx.BNC, 8), (5, fx.BCN, 8),
                                        (64, fx.BNC, 13), (64, fx.BNC, 20)])
def test_widths_layouts_and_list_lengths_without_a_planned_kernel_run_the_list_form(C, layout, K):
    say(f"pool plan, list form behind it: C={C} layout={layout} K={K}")
    run_case(7 + C + K, 2, 700, K, C, layout, "local")


@pytest.mark.parametrize("kind", ["local", "hub", "scattered", "random"])
@pytest.mark.parametrize("B,N,C", [(1, 3000, 128), (2, 1001, 256), (1, 530_000, 128)])
def test_wider_rows_run_the_planned_kernel_once_per_64_channels(B, N, C, kind):
    say(f"pool plan: B={B} N={N} C={C} lists={kind}")
    run_case(N + C, B, N, 8, C, fx.BNC, kind)


def test_plan_arguments_are_checked():
    L = fx.lib()
    B, N, K = 1, 500, 8
    rng = np.random.default_rng(0)
    dn = dev(lists("local", rng, B, N, K))
    off, src = fx.flex_inedges_build(dn)
    need = int(L.flexpool_plan_bytes(B, N, K))
    assert need > 0 and need % 256 == 0
    assert int(L.flexpool_plan_bytes(B, N, N + 1)) == 0 and int(L.flexpool_plan_bytes(0, N, K)) == 0
    plan = torch.empty(need, dtype=torch.uint8, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.flexpool_plan_build(p(off), p(src), B, N, K, p(plan), need - 1, None) == 4        # FLEX_ERR_WORKSPACE
    assert L.flexpool_plan_build(None, p(src), B, N, K, p(plan), need, None) == 1               # FLEX_ERR_NULL
    assert L.flexpool_plan_build(p(off), p(src), B, N, K, p(plan), need, None) == 0
    g = torch.zeros(B, N, 64, device="cuda")
    arg = torch.zeros(B, N, 64, dtype=torch.int32, device="cuda")
    out = torch.empty_like(g)
    assert L.flexpool_bwd_planned(p(g), p(arg), p(out), p(off), p(src), p(plan), need - 1, B, N, K, 64, fx.BNC, None) == 4
    assert L.flexpool_bwd_planned(p(g), p(arg), p(out), p(off), p(src), None, need, B, N, K, 64, fx.BNC, None) == 1
    assert L.flexpool_bwd_planned(p(g), p(arg), p(out), p(off), p(src), p(plan), need, B, N, K, 64, 7, None) == 2
    assert L.flexpool_fwd_plan_build(p(dn), B, N, K, p(plan), need - 1, None) == 4
    assert L.flexpool_fwd_plan_build(None, B, N, K, p(plan), need, None) == 1
    assert L.flexpool_fwd_plan_build(p(dn), B, N, K, p(plan), need, None) == 0
    assert L.flexpool_fwd_planned(p(g), p(dn), p(out), p(arg), p(plan), need - 1, B, N, K, 64, fx.BNC, None) == 4
    assert L.flexpool_fwd_planned(p(g), p(dn), p(out), p(arg), None, need, B, N, K, 64, fx.BNC, None) == 1
    assert L.flexpool_fwd_planned(p(g), p(dn), p(out), p(arg), p(plan), need, B, N, K, 64, 7, None) == 2
    assert L.flexpool_fwd_planned(p(g), p(dn), p(out), p(arg), p(plan), need, B, N, K, 64, fx.BNC, None) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("case", range(12))
def test_planned_passes_on_random_shapes(case):
    """Seeded random cloud counts, sizes, K and widths with a planned kernel, lists with and without locality
    (under FLEX_POOL_PLAN=1 every case runs the planned kernels; without it the sizes here run the plain ones)."""
    rng = np.random.default_rng(7100 + case)
    B, N = int(rng.integers(1, 4)), int(rng.integers(2, 3000))
    K, C = int(rng.integers(1, min(N, 20) + 1)), int(rng.choice([64, 128, 256]))
    kind = str(rng.choice(["local", "random", "repeats"]))
    say(f"random planned case {case}: B={B} N={N} K={K} C={C} lists={kind}")
    run_case(7100 + case, B, N, K, C, fx.BNC, kind)
