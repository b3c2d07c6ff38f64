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


CANARY_BYTES = 4096


class ExactWorkspace:
    """A caller workspace of exactly the size the library asks for, with a guard pattern right behind it.

    `ws` (what the entry point is given) is a view of the first `need` bytes of a larger allocation, so the library
    is told `need` and not a byte more; check() fails if anything was written past the end."""

    def __init__(self, op, B, N, K, Din, Dout, layout):
        self.need = max(fx.workspace_bytes(op, B, N, K, Din, Dout, layout), 256)
        self.buf = torch.empty(self.need + CANARY_BYTES, dtype=torch.uint8, device="cuda")
        self.buf[self.need:] = 0xA5
        self.ws = self.buf[:self.need]

    def check(self):
        torch.cuda.synchronize()
        assert bool((self.buf[self.need:] == 0xA5).all()), "the library wrote past the workspace it asked for"
