"""Shared test utilities (tiny clouds, grids, error metric).  No method arithmetic
for the GPU path lives here; the numpy formulas below are the independent
re-derivations used to pin the oracle."""
import os
import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def tiny_problem(seed, B=2, N=11, K=3, Din=3, Dout=2, self_first=False):
    rng = np.random.default_rng(seed)
    pos = rng.standard_normal((B, 3, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    if self_first:
        nbr[:, 0, :] = np.arange(N)
    feat = rng.standard_normal((B, Din, N)).astype(np.float32)
    theta = rng.standard_normal((3, Din, Dout)).astype(np.float32)
    bias = rng.standard_normal((Din, Dout)).astype(np.float32)
    g = rng.standard_normal((B, Dout, N)).astype(np.float32)
    return pos, nbr, feat, theta, bias, g


def dense_weights(pos, nbr, theta, bias, centre_minus_neighbour=False):
    """W[b,l,k,c,o]: the flex-conv weight of every (centre, slot, c, o), float64."""
    pos = pos.astype(np.float64)
    B, K, N = nbr.shape
    bi = np.arange(B)[:, None, None]
    pn = pos[bi, :, nbr.transpose(0, 2, 1)]            # [B,N,K,3]
    pl = pos.transpose(0, 2, 1)[:, :, None, :]         # [B,N,1,3]
    dp = (pl - pn) if centre_minus_neighbour else (pn - pl)
    return np.einsum("dco,blkd->blkco", theta.astype(np.float64), dp) + bias.astype(np.float64)


def gathered(feat, nbr):
    """F[b,l,k,c] = feat[b,c,nbr[b,k,l]] in float64."""
    B, K, N = nbr.shape
    bi = np.arange(B)[:, None, None]
    return feat.astype(np.float64).transpose(0, 2, 1)[bi, nbr.transpose(0, 2, 1), :]


def grid2d(H, W, h):
    """Points on an HxW grid in the z=0 plane (index = y*W+x) and the 9-offset
    neighbour table (clamped at the border; only the interior is compared)."""
    ys, xs = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    pos = np.stack([xs.ravel() * h, ys.ravel() * h, np.zeros(H * W)], 0).astype(np.float32)[None]
    offs = [(dy, dx) for dy in (-1, 0, 1) for dx in (-1, 0, 1)]
    nbr = np.empty((1, 9, H * W), np.int32)
    for k, (dy, dx) in enumerate(offs):
        yy = np.clip(ys + dy, 0, H - 1)
        xx = np.clip(xs + dx, 0, W - 1)
        nbr[0, k] = (yy * W + xx).ravel()
    return pos, nbr, offs


def read_golden_kernels():
    out, name, rows = {}, None, []
    for line in open(os.path.join(GOLDEN, "prewitt_blur_3x3.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line[0].isalpha():
            if name:
                out[name] = np.array(rows, np.float64)
            name, rows = line, []
        else:
            rows.append([float(t) for t in line.split()])
    out[name] = np.array(rows, np.float64)
    return out


def rel_err(got, ref):
    """max |got-ref| / max(|ref|, RMS(ref)) per tensor (the parity metric)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0
