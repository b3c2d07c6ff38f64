"""Seeded synthetic inputs for the flex-convolution hot path.

This package only *draws inputs*: point clouds, neighbour indices, features,
parameters and upstream gradients.  It contains none of the method's
arithmetic (no flex-conv weights, sums, maxima or gradients), so both the
CPU oracle's tests and the GPU path's tests may feed from it.
"""
from .configs import CONFIGS, Config, get_config          # noqa: F401
from .clouds import (uniform_cube, box_surface_cloud, room_cloud,  # noqa: F401
                     morton_order)
from .knn import knn_bruteforce, knn_kdtree                 # noqa: F401
from .inputs import make_inputs, Inputs                     # noqa: F401
