"""GPU parity for inverse density importance sub-sampling: phi within fp32 rounding of the fp64 oracle, the draw
bit-exact against the oracle's sequential integer procedure on the same phi and random words."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import dev, say
from helpers import rel_err
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def _words(rng, B, Ns):
    return rng.integers(0, 2 ** 32, size=(B, Ns), dtype=np.uint64).astype(np.uint32)


def _draw(phi, u):
    du = torch.from_numpy(u.view(np.int32)).cuda()
    sel = fx.flex_idiss_sample(dev(phi), du)
    torch.cuda.synchronize()
    return sel.cpu().numpy()


@pytest.mark.parametrize("B,N,K", [(2, 1000, 8), (1, 4099, 16), (3, 77, 3)])
def test_phi_matches_oracle(B, N, K):
    say(f"idiss phi B={B} N={N} K={K}")
    rng = np.random.default_rng(N)
    pos = rng.random((B, 3, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    phi = fx.flex_idiss_phi(dev(pos), dev(nbr))
    torch.cuda.synchronize()
    assert rel_err(phi.cpu().numpy(), oracle.idiss_phi(pos, nbr)) <= 2e-6


@pytest.mark.parametrize("B,N,Ns", [(2, 1000, 250), (1, 2048, 2048), (3, 77, 1), (1, 5000, 1250), (2, 2049, 700)])
def test_draw_is_bit_exact(B, N, Ns):
    say(f"idiss draw B={B} N={N} Ns={Ns}")
    rng = np.random.default_rng(N + Ns)
    phi = rng.random((B, N)).astype(np.float32)
    phi[0, ::9] = 0.0
    phi[-1, N // 2] = 300.0                                    # spans many strata
    u = _words(rng, B, Ns)
    assert np.array_equal(_draw(phi, u), oracle.idiss_sample(phi, u))


def test_draw_degenerate_clouds():
    rng = np.random.default_rng(7)
    u = _words(rng, 2, 64)
    phi = np.zeros((2, 256), np.float32)                       # coincident points: uniform
    phi[1] = 0.25
    sel = _draw(phi, u)
    assert np.array_equal(sel, oracle.idiss_sample(phi, u))
    assert np.array_equal(sel // 4, np.tile(np.arange(64), (2, 1)))


def test_idiss_room_scale_end_to_end():
    """A room cloud of 400k points: phi from the library, a quarter of the points drawn; the draw must equal the
    oracle's on the library's own phi is not allowed as a check (no oracle input may come from the GPU), so the
    oracle's phi (rounded to fp32) feeds both draws and the library's phi is compared separately."""
    cfg = CONFIGS[2]
    x = make_inputs(cfg, with_grad=False, n_override=400_000)
    N = 400_000
    ophi = oracle.idiss_phi(x.pos, x.nbr)
    gphi = fx.flex_idiss_phi(dev(x.pos), dev(x.nbr))
    torch.cuda.synchronize()
    assert rel_err(gphi.cpu().numpy(), ophi) <= 2e-6
    phi32 = ophi.astype(np.float32)
    u = _words(np.random.default_rng(8), 1, N // 4)
    sel = _draw(phi32, u)
    assert np.array_equal(sel, oracle.idiss_sample(phi32, u))
    # sparse regions are favoured: the drawn points' mean phi exceeds the cloud's
    assert phi32[0][sel[0]].mean() > phi32.mean()


@pytest.mark.parametrize("B,N,Ns", [(2, 1000, 400), (1, 10, 10), (3, 5000, 1), (1, 300_000, 75_000), (2, 4097, 4000)])
def test_make_distinct_is_bit_exact(B, N, Ns):
    say(f"make distinct B={B} N={N} Ns={Ns}")
    rng = np.random.default_rng(N + Ns)
    sel = np.sort(rng.integers(0, N, size=(B, Ns)), axis=1).astype(np.int32)
    sel[0, Ns // 2:] = np.maximum(sel[0, Ns // 2:], N - 3)          # repeats piled up against the end
    got = fx.flex_selection_make_distinct(dev(sel), N)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.selection_make_distinct(sel, N))


def test_idiss_draw_made_distinct_feeds_upsampling():
    rng = np.random.default_rng(5)
    N, Ns = 20_000, 5_000
    phi = rng.random((1, N)).astype(np.float32) ** 4                 # strongly uneven: many repeats
    u = _words(rng, 1, Ns)
    sel = fx.flex_idiss_sample(dev(phi), torch.from_numpy(u.view(np.int32)).cuda())
    assert fx.flex_validate_selection(sel, N) > 0                    # the raw draw repeats points
    fx.flex_selection_make_distinct(sel, N)
    assert fx.flex_validate_selection(sel, N) == 0
    assert np.array_equal(sel.cpu().numpy(), oracle.selection_make_distinct(oracle.idiss_sample(phi, u), N))
