"""Helpers for the GPU parity tests: move numpy inputs to the device in either layout."""
import numpy as np
import torch

import paper_1803_07289_amd as fx

TOL = 1e-4   # max |gpu-ref| / max(|ref|, RMS(ref)), fp32 GPU vs fp64 oracle


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_layout(a_bcn, layout):
    """numpy [B,C,N] -> device tensor in the asked layout."""
    if layout == fx.BNC:
        return dev(np.ascontiguousarray(a_bcn.transpose(0, 2, 1)))
    return dev(a_bcn)


def from_layout(t, layout):
    """device tensor -> numpy [B,C,N]."""
    a = t.detach().cpu().numpy()
    return a.transpose(0, 2, 1) if layout == fx.BNC else a


def say(*a):
    print(*a, flush=True)
