"""Pins for the CPU oracle's exhaustive k-nearest-neighbour search (CPU only)."""
import numpy as np

import oracle
from helpers import grid2d
from workloads.knn import knn_kdtree


def test_knn_matches_float32_numpy_ranking_with_ties():
    rng = np.random.default_rng(0)
    B, N, K = 2, 60, 7
    pos = rng.integers(0, 4, size=(B, 3, N)).astype(np.float32)       # a coarse lattice: many equal distances
    nbr = oracle.knn(pos, K)
    for b in range(B):
        p = pos[b]
        for l in range(N):
            d = p - p[:, l:l + 1]
            d2 = (d[0] * d[0] + d[1] * d[1]) + d[2] * d[2]            # float32, the same operation order
            order = np.lexsort((np.arange(N), d2))                     # by d2, then by index
            assert list(nbr[b, :, l]) == list(order[:K])


def test_knn_agrees_with_a_kd_tree_on_generic_points():
    # generic positions have no ties and gaps far above float32 rounding: any exact method must agree
    rng = np.random.default_rng(1)
    N, K = 500, 8
    pos = rng.random((1, 3, N)).astype(np.float32)
    nbr = oracle.knn(pos, K)
    ref = knn_kdtree(pos[0].T.astype(np.float64), K)
    assert np.array_equal(nbr[0], ref)
    assert np.array_equal(nbr[0, 0], np.arange(N))                     # every point is its own nearest


def test_knn_on_a_grid_is_the_3x3_stencil():
    H, W = 6, 7
    pos, stencil, _ = grid2d(H, W, 1.0)
    nbr = oracle.knn(pos, 9)
    for y in range(1, H - 1):
        for x in range(1, W - 1):
            l = y * W + x
            assert sorted(nbr[0, :, l]) == sorted(stencil[0, :, l])
            assert nbr[0, 0, l] == l
            assert sorted(nbr[0, 1:5, l]) == sorted([l - 1, l + 1, l - W, l + W])   # the four at distance 1 first


def test_knn_k_equals_n_and_duplicates():
    pos = np.zeros((1, 3, 5), np.float32)
    pos[0, 0] = [0, 1, 1, 3, 0]                                          # points 0,4 and 1,2 coincide
    nbr = oracle.knn(pos, 5)
    assert list(nbr[0, :, 0]) == [0, 4, 1, 2, 3]
    assert list(nbr[0, :, 2]) == [1, 2, 0, 4, 3]
