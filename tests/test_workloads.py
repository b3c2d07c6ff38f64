"""The seeded input recipes: shapes, determinism, neighbour validity (CPU only)."""
import numpy as np
from workloads import CONFIGS, make_inputs
from workloads.knn import knn_bruteforce, knn_kdtree
from workloads.clouds import morton_order


def test_config_shapes_match_the_five_workloads():
    shapes = [(c.B, c.N, c.K, c.Din, c.Dout) for c in CONFIGS]
    assert shapes == [(1, 4096, 8, 32, 32), (8, 4096, 16, 64, 64), (1, 1_000_000, 8, 9, 64),
                      (1, 1_000_000, 8, 128, 128), (1, 7_000_000, 8, 64, 64)]


def test_inputs_are_seeded_and_typed():
    a = make_inputs(CONFIGS[0])
    b = make_inputs(CONFIGS[0])
    for f in ("pos", "nbr", "feat", "theta", "bias", "grad_out"):
        x, y = getattr(a, f), getattr(b, f)
        assert np.array_equal(x, y)
    assert a.pos.dtype == np.float32 and a.nbr.dtype == np.int32
    assert a.nbr.shape == (1, 8, 4096) and a.theta.shape == (3, 32, 32)
    assert (a.nbr[0, 0] == np.arange(4096)).all()            # self is the nearest neighbour
    assert abs(a.theta.std() - (4 * 32 * 8) ** -0.5) < 0.1 * (4 * 32 * 8) ** -0.5


def test_knn_kdtree_equals_bruteforce():
    rng = np.random.default_rng(3)
    p = rng.random((1500, 3)).astype(np.float32)
    assert np.array_equal(knn_bruteforce(p, 8), knn_kdtree(p, 8))


def test_room_inputs_small_and_morton_locality():
    x = make_inputs(CONFIGS[2], n_override=20000)
    assert x.pos.shape == (1, 3, 20000) and x.feat.shape == (1, 9, 20000)
    assert x.feat.min() >= 0 and x.feat.max() < 1
    assert x.pos[0, 0].min() > -0.1 and x.pos[0, 0].max() < 10.1 and x.pos[0, 2].max() < 3.1
    d = np.abs(x.nbr[0] - np.arange(20000)[None])
    y = make_inputs(CONFIGS[2], n_override=20000, order="shuffled")
    d2 = np.abs(y.nbr[0] - np.arange(20000)[None])
    assert np.median(d) * 20 < np.median(d2)                 # Z-order keeps neighbours close in memory
    p = np.random.default_rng(0).random((1000, 3))
    o = morton_order(p)
    assert sorted(o.tolist()) == list(range(1000))
