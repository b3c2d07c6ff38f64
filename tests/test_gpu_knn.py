"""GPU parity for the grid k-nearest-neighbour search: the index tensor must equal the exhaustive CPU search bit for
bit (same float32 squared distance, ties to the lower index) on generic, degenerate and tie-heavy clouds."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import dev, say
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def _check(pos, K):
    nbr = fx.flex_knn(dev(pos), K)
    torch.cuda.synchronize()
    ref = oracle.knn(pos, K)
    got = nbr.cpu().numpy()
    bad = np.argwhere(got != ref)
    assert bad.size == 0, (bad[:5], got[tuple(bad[0])], ref[tuple(bad[0])])


@pytest.mark.parametrize("B,N,K", [(2, 3000, 8), (1, 5000, 16), (3, 700, 9), (1, 10, 10), (1, 1, 1), (2, 257, 1),
                                   (1, 2000, 32), (1, 1500, 5)])
def test_knn_uniform_cube(B, N, K):
    say(f"knn cube B={B} N={N} K={K}")
    pos = np.random.default_rng(N + K).random((B, 3, N)).astype(np.float32)
    _check(pos, K)


def test_knn_lattice_with_many_ties():
    rng = np.random.default_rng(1)
    pos = rng.integers(0, 12, size=(2, 3, 4000)).astype(np.float32)     # equal distances and coincident points
    _check(pos, 8)
    _check(pos * np.float32(0.37), 16)


def test_knn_degenerate_shapes():
    rng = np.random.default_rng(2)
    N = 3000
    flat = rng.random((1, 3, N)).astype(np.float32); flat[0, 2] = 0.25           # a plane
    line = np.zeros((1, 3, N), np.float32); line[0, 0] = rng.random(N)            # a line
    same = np.full((1, 3, 500), 1.5, np.float32)                                 # one location
    far = rng.random((1, 3, N)).astype(np.float32) * 0.5 + np.float32(1000.0)    # far from the origin: coarse float grid
    clumps = (rng.integers(0, 3, size=(1, 3, N)) * 100.0 + rng.normal(0, 0.01, (1, 3, N))).astype(np.float32)
    for name, pos, K in (("plane", flat, 8), ("line", line, 8), ("one location", same, 8), ("offset", far, 8),
                         ("clumps", clumps, 16)):
        say("knn", name)
        _check(pos, K)


def test_knn_room_cloud_matches_and_feeds_the_layers():
    """Room surfaces (the workload's geometry), 30k points: equal to the exhaustive search, and the tensor is a valid
    input of the other entry points."""
    x = make_inputs(CONFIGS[2], with_grad=False, n_override=30_000)
    _check(x.pos, 8)
    nbr = fx.flex_knn(dev(x.pos), 8)
    assert fx.flex_validate_neighbors(nbr) == 0
    assert torch.equal(nbr[0, 0].cpu(), torch.arange(30_000, dtype=torch.int32))   # jittered points: no coincidences
