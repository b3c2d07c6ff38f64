"""The primitives chained the way the paper's encoder / decoder uses them (Sec. 4.3): neighbour search, flex-convolution,
inverse-density sub-sampling, flex-max-pooling with subsampling, a flex-convolution on the coarser cloud with its own
neighbourhoods, flex-upsampling back.  Index results (neighbours, selection, winners) must equal the oracle's exactly,
so the two chains stay comparable; the final features agree to the flex-conv tolerance."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import dev, to_layout, from_layout, say
from helpers import rel_err
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def test_encoder_decoder_stage_matches_oracle_chain():
    x = make_inputs(CONFIGS[2], with_grad=False, n_override=6000)       # room surfaces
    N, K, C = 6000, 8, 64
    rng = np.random.default_rng(21)
    pos = x.pos
    feat = rng.standard_normal((1, C, N)).astype(np.float32)
    th1 = (rng.standard_normal((3, C, C)) / np.sqrt(4 * C * K)).astype(np.float32)
    b1 = (rng.standard_normal((C, C)) / np.sqrt(4 * C * K)).astype(np.float32)
    th2 = (rng.standard_normal((3, C, C)) / np.sqrt(4 * C * K)).astype(np.float32)
    b2 = (rng.standard_normal((C, C)) / np.sqrt(4 * C * K)).astype(np.float32)
    Ns = N // 4
    u = rng.integers(0, 2 ** 32, size=(1, Ns), dtype=np.uint64).astype(np.uint32)

    # ---- oracle chain (its own intermediates all the way) ----
    o_nbr = oracle.knn(pos, K)
    o_f1 = oracle.flexconv_fwd(feat, pos, o_nbr, th1, b1).astype(np.float32)
    o_phi = oracle.idiss_phi(pos, o_nbr).astype(np.float32)
    o_sel = oracle.selection_make_distinct(oracle.idiss_sample(o_phi, u), N)     # repeats move to the next free index
    o_pool, o_arg = oracle.flexpool_sub_fwd(o_f1, o_nbr, o_sel)
    o_pos_s = np.ascontiguousarray(pos[:, :, o_sel[0]])
    o_nbr_s = oracle.knn(o_pos_s, K)
    o_f2 = oracle.flexconv_fwd(o_pool, o_pos_s, o_nbr_s, th2, b2).astype(np.float32)
    o_up, o_uparg = oracle.flexupsample_fwd(o_f2, o_sel, o_nbr)

    # ---- library chain ----
    L = fx.BNC
    dpos = dev(pos)
    nbr = fx.flex_knn(dpos, K)
    assert np.array_equal(nbr.cpu().numpy(), o_nbr)
    f1 = fx.flexconv_fwd(to_layout(feat, L), dpos, nbr, dev(th1), dev(b1), layout=L)
    phi = fx.flex_idiss_phi(dpos, nbr)
    assert rel_err(phi.cpu().numpy(), o_phi) <= 2e-6
    # the draw is an integer procedure on phi's bits: both sides get the oracle's phi so that one rounding of phi
    # cannot send the two chains to different points
    sel_raw = fx.flex_idiss_sample(dev(o_phi), torch.from_numpy(u.view(np.int32)).cuda())
    sel = fx.flex_selection_make_distinct(sel_raw, N)
    assert np.array_equal(sel.cpu().numpy(), o_sel)
    assert fx.flex_validate_selection(sel, N) == 0
    pool, arg = fx.flexpool_sub_fwd(f1, nbr, sel, layout=L)
    pos_s = torch.index_select(dpos, 2, sel[0].long()).contiguous()
    nbr_s = fx.flex_knn(pos_s, K)
    assert np.array_equal(nbr_s.cpu().numpy(), o_nbr_s)
    f2 = fx.flexconv_fwd(pool, pos_s, nbr_s, dev(th2), dev(b2), layout=L)
    up, uparg = fx.flexupsample_fwd(f2, sel, nbr, layout=L)
    torch.cuda.synchronize()

    say("stage errors", rel_err(from_layout(f1, L), o_f1), rel_err(from_layout(f2, L), o_f2), rel_err(from_layout(up, L), o_up))
    assert rel_err(from_layout(f1, L), o_f1) <= 1e-4
    # pooling picks winners from features that differ in the last bits between the chains: near-ties may resolve
    # differently, so winners are compared where the oracle's margin is clear, values everywhere
    assert rel_err(from_layout(pool, L), o_pool) <= 1e-4
    assert (from_layout(arg, L) == o_arg).mean() >= 0.999
    assert rel_err(from_layout(f2, L), o_f2) <= 2e-4
    assert rel_err(from_layout(up, L), o_up) <= 2e-4
    assert (from_layout(uparg, L) == o_uparg).mean() >= 0.999
