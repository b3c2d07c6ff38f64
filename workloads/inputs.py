"""Draw every input array of one configuration from seeded streams."""
from dataclasses import dataclass
import numpy as np

from .configs import Config
from .clouds import uniform_cube, box_surface_cloud, room_cloud, morton_order
from .knn import knn_bruteforce, knn_kdtree


@dataclass
class Inputs:
    cfg: Config
    order: str
    pos: np.ndarray       # float32 [B,3,N]
    nbr: np.ndarray       # int32   [B,K,N]
    feat: np.ndarray      # float32 [B,Din,N]
    theta: np.ndarray     # float32 [3,Din,Dout]
    bias: np.ndarray      # float32 [Din,Dout]
    grad_out: np.ndarray  # float32 [B,Dout,N]


def _rng(seed, stream):
    return np.random.default_rng([seed, stream])


def _cloud(cfg, rng):
    if cfg.cloud == "cube":
        return uniform_cube(rng, cfg.N)
    if cfg.cloud == "box":
        return box_surface_cloud(rng, cfg.N, sigma=0.005, clutter=0.2)
    if cfg.cloud == "room":
        return room_cloud(rng, cfg.N, size=(10.0, 10.0, 3.0), n_boxes=30, sigma=0.005)
    if cfg.cloud == "hall":
        return room_cloud(rng, cfg.N, size=(25.0, 25.0, 4.0), n_boxes=200, sigma=0.003)
    raise ValueError(cfg.cloud)


def make_inputs(cfg: Config, order: str = "morton", with_grad: bool = True,
                n_override: int = None) -> Inputs:
    """order: 'morton' (Z-order sorted), 'generator' (as drawn) or 'shuffled'.
    The small brute-force configs (0, 1) keep generator order unless asked.
    n_override shrinks N (same recipe) for quick tests."""
    if n_override is not None:
        cfg = Config(**{**cfg.__dict__, "N": int(n_override)})
    B, N, K, Din, Dout = cfg.B, cfg.N, cfg.K, cfg.Din, cfg.Dout
    if cfg.knn == "brute" and order == "morton":
        order = "generator"
    pos = np.empty((B, 3, N), np.float32)
    nbr = np.empty((B, K, N), np.int32)
    for b in range(B):
        rng = _rng(cfg.seed, 100 + b)
        pts = _cloud(cfg, rng)
        if order == "morton":
            pts = pts[morton_order(pts)]
        elif order == "shuffled":
            pts = pts[_rng(cfg.seed, 200 + b).permutation(N)]
        elif order != "generator":
            raise ValueError(order)
        pos[b] = pts.T
        nbr[b] = knn_bruteforce(pts, K) if cfg.knn == "brute" else knn_kdtree(pts, K)
    rf = _rng(cfg.seed, 1)
    if cfg.feat == "normal":
        feat = rf.standard_normal((B, Din, N), dtype=np.float32)
    else:
        feat = rf.random((B, Din, N), dtype=np.float32)
    std = (4.0 * Din * K) ** -0.5
    theta = (_rng(cfg.seed, 2).standard_normal((3, Din, Dout), dtype=np.float32) * np.float32(std))
    bias = (_rng(cfg.seed, 3).standard_normal((Din, Dout), dtype=np.float32) * np.float32(std))
    grad_out = (_rng(cfg.seed, 4).standard_normal((B, Dout, N), dtype=np.float32)
                if with_grad else None)
    return Inputs(cfg, order, pos, nbr, feat, theta, bias, grad_out)
