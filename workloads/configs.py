"""The five workload configurations (shapes and recipes), indexed 0..4."""
from dataclasses import dataclass


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    B: int
    N: int
    K: int
    Din: int
    Dout: int
    cloud: str          # "cube" | "box" | "room" | "hall"
    knn: str            # "brute" | "kdtree"
    feat: str           # "normal" | "uniform"
    runs: tuple         # which ops the config exercises
    seed: int


CONFIGS = (
    Config(0, "cube4k_k8_32x32", 1, 4096, 8, 32, 32, "cube", "brute", "normal",
           ("conv_fwd", "conv_bwd"), 0),
    Config(1, "box8x4k_k16_64x64", 8, 4096, 16, 64, 64, "box", "brute", "normal",
           ("conv_fwd", "conv_bwd", "pool_fwd", "pool_bwd"), 1),
    Config(2, "room1m_k8_9x64", 1, 1_000_000, 8, 9, 64, "room", "kdtree", "uniform",
           ("conv_fwd",), 2),
    Config(3, "room1m_k8_128x128", 1, 1_000_000, 8, 128, 128, "room", "kdtree", "normal",
           ("conv_fwd", "conv_bwd", "pool_fwd", "pool_bwd"), 3),
    Config(4, "hall7m_k8_64x64", 1, 7_000_000, 8, 64, 64, "hall", "kdtree", "normal",
           ("conv_fwd", "conv_bwd", "pool_fwd", "pool_bwd"), 4),
)


def get_config(i: int) -> Config:
    return CONFIGS[i]
