"""ctypes wrapper around the plain-C CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  It does not import, and is not imported by,
the GPU package.  All arrays are host numpy arrays in the paper's
channel-major layouts; results are float64 unless stated.
"""
import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (OpenMP) into oracle/liboracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_count_bad_neighbors.restype = ctypes.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(rc, name):
    if rc != 0:
        raise RuntimeError(f"{name} failed with status {rc}")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def count_bad_neighbors(nbr, N) -> int:
    nbr = _i32(nbr)
    B, K, N_ = nbr.shape
    assert N_ == N
    return int(_load().oracle_count_bad_neighbors(_p(nbr), B, N, K))


def flexconv_fwd(feat, pos, nbr, theta, bias, l_range=None):
    """Returns float64 out [B,Dout,L]: all N columns, or columns l_range=(l0,l1) only."""
    feat, pos, theta, bias, nbr = _f32(feat), _f32(pos), _f32(theta), _f32(bias), _i32(nbr)
    B, Din, N = feat.shape
    K = nbr.shape[1]
    Dout = theta.shape[2]
    assert pos.shape == (B, 3, N) and nbr.shape == (B, K, N)
    assert theta.shape == (3, Din, Dout) and bias.shape == (Din, Dout)
    assert count_bad_neighbors(nbr, N) == 0
    l0, l1 = (0, N) if l_range is None else l_range
    out = np.zeros((B, Dout, l1 - l0), np.float64)
    _check(_load().oracle_flexconv_fwd(_p(feat), _p(pos), _p(nbr), _p(theta), _p(bias), _p(out),
                                       B, N, K, Din, Dout, int(l0), int(l1)), "oracle_flexconv_fwd")
    return out


def flexconv_bwd(feat, pos, nbr, theta, bias, grad_out, l_range=None,
                 want_feat=True, want_params=True):
    """Returns (grad_feat [B,Din,N], grad_theta [3,Din,Dout], grad_bias [Din,Dout]) in float64."""
    feat, pos, theta, bias, nbr = _f32(feat), _f32(pos), _f32(theta), _f32(bias), _i32(nbr)
    grad_out = _f32(grad_out)
    B, Din, N = feat.shape
    K = nbr.shape[1]
    Dout = theta.shape[2]
    assert grad_out.shape == (B, Dout, N)
    assert count_bad_neighbors(nbr, N) == 0
    l0, l1 = (0, N) if l_range is None else l_range
    gf = np.zeros((B, Din, N), np.float64) if want_feat else None
    gt = np.zeros((3, Din, Dout), np.float64) if want_params else None
    gb = np.zeros((Din, Dout), np.float64) if want_params else None
    _check(_load().oracle_flexconv_bwd(_p(feat), _p(pos), _p(nbr), _p(theta), _p(bias), _p(grad_out),
                                       _p(gf), _p(gt), _p(gb), B, N, K, Din, Dout, int(l0), int(l1)),
           "oracle_flexconv_bwd")
    return gf, gt, gb


def flexconv_grad_feat_at(pos, nbr, theta, bias, grad_out, targets):
    """grad_feat rows at flat targets (b*N+m): float64 [len(targets), Din]."""
    pos, theta, bias, nbr, grad_out = _f32(pos), _f32(theta), _f32(bias), _i32(nbr), _f32(grad_out)
    B, K, N = nbr.shape
    _, Din, Dout = theta.shape
    assert count_bad_neighbors(nbr, N) == 0
    targets = np.ascontiguousarray(targets, dtype=np.int64)
    out = np.zeros((targets.size, Din), np.float64)
    _check(_load().oracle_flexconv_grad_feat_at(_p(pos), _p(nbr), _p(theta), _p(bias), _p(grad_out),
                                                _p(targets), ctypes.c_int64(targets.size), _p(out),
                                                B, N, K, Din, Dout), "oracle_flexconv_grad_feat_at")
    return out


def flexpool_fwd(feat, nbr, l_range=None):
    """Returns (out float32, argmax int32), both [B,C,L]: all N columns or l_range only."""
    feat, nbr = _f32(feat), _i32(nbr)
    B, C, N = feat.shape
    K = nbr.shape[1]
    assert count_bad_neighbors(nbr, N) == 0
    l0, l1 = (0, N) if l_range is None else l_range
    out = np.zeros((B, C, l1 - l0), np.float32)
    arg = np.zeros((B, C, l1 - l0), np.int32)
    _check(_load().oracle_flexpool_fwd(_p(feat), _p(nbr), _p(out), _p(arg), B, N, K, C, int(l0), int(l1)),
           "oracle_flexpool_fwd")
    return out, arg


def flexpool_bwd(grad_out, argmax, l_range=None):
    """Returns grad_feat float64 [B,C,N]."""
    grad_out, argmax = _f32(grad_out), _i32(argmax)
    B, C, N = grad_out.shape
    assert argmax.shape == (B, C, N)
    l0, l1 = (0, N) if l_range is None else l_range
    if l1 > l0:
        assert argmax[:, :, l0:l1].min() >= 0 and argmax[:, :, l0:l1].max() < N
    gf = np.zeros((B, C, N), np.float64)
    _check(_load().oracle_flexpool_bwd(_p(grad_out), _p(argmax), _p(gf), B, N, C, int(l0), int(l1)),
           "oracle_flexpool_bwd")
    return gf


def flexpool_sub_fwd(feat, nbr, sel):
    """Flex-max-pooling then subsampling: feat [B,C,N], nbr [B,K,N], sel int32 [B,Ns].
    Returns (out float32, argmax int32), both [B,C,Ns]."""
    feat, nbr, sel = _f32(feat), _i32(nbr), _i32(sel)
    B, C, N = feat.shape
    K = nbr.shape[1]
    Ns = sel.shape[1]
    assert sel.shape == (B, Ns) and nbr.shape == (B, K, N)
    assert count_bad_neighbors(nbr, N) == 0
    out = np.zeros((B, C, Ns), np.float32)
    arg = np.zeros((B, C, Ns), np.int32)
    _check(_load().oracle_flexpool_sub_fwd(_p(feat), _p(nbr), _p(sel), _p(out), _p(arg), B, N, Ns, K, C),
           "oracle_flexpool_sub_fwd")
    return out, arg


def flexpool_sub_bwd(grad_out, argmax, sel, N):
    """Backward of flexpool_sub_fwd: grad_out / argmax [B,C,Ns], sel [B,Ns].  Returns grad_feat float64 [B,C,N]."""
    grad_out, argmax, sel = _f32(grad_out), _i32(argmax), _i32(sel)
    B, C, Ns = grad_out.shape
    assert argmax.shape == (B, C, Ns) and sel.shape == (B, Ns)
    gf = np.zeros((B, C, N), np.float64)
    _check(_load().oracle_flexpool_sub_bwd(_p(grad_out), _p(argmax), _p(sel), _p(gf), B, int(N), Ns, C),
           "oracle_flexpool_sub_bwd")
    return gf


def flexupsample_fwd(feat_small, sel, nbr, l_range=None):
    """Flex-upsampling: feat_small [B,C,Ns], sel int32 [B,Ns] (indices in the larger layer),
    nbr int32 [B,K,Nf].  Returns (out float32, argmax int32), both [B,C,L]."""
    feat_small, sel, nbr = _f32(feat_small), _i32(sel), _i32(nbr)
    B, C, Ns = feat_small.shape
    _, K, Nf = nbr.shape
    assert sel.shape == (B, Ns)
    assert count_bad_neighbors(nbr, Nf) == 0
    l0, l1 = (0, Nf) if l_range is None else l_range
    out = np.zeros((B, C, l1 - l0), np.float32)
    arg = np.zeros((B, C, l1 - l0), np.int32)
    _check(_load().oracle_flexupsample_fwd(_p(feat_small), _p(sel), _p(nbr), _p(out), _p(arg),
                                           B, Ns, Nf, K, C, int(l0), int(l1)), "oracle_flexupsample_fwd")
    return out, arg


def flexupsample_bwd(grad_out, argmax, sel):
    """Returns grad_small float64 [B,C,Ns]."""
    grad_out, argmax, sel = _f32(grad_out), _i32(argmax), _i32(sel)
    B, C, Nf = grad_out.shape
    Ns = sel.shape[1]
    assert argmax.shape == (B, C, Nf) and sel.shape == (B, Ns)
    gs = np.zeros((B, C, Ns), np.float64)
    _check(_load().oracle_flexupsample_bwd(_p(grad_out), _p(argmax), _p(sel), _p(gs), B, Ns, Nf, C),
           "oracle_flexupsample_bwd")
    return gs


def flexconv_bwd_pos(feat, nbr, theta, grad_out):
    """Gradient of the flex-conv layer with respect to the point locations: float64 [B,3,N]."""
    feat, nbr, theta, grad_out = _f32(feat), _i32(nbr), _f32(theta), _f32(grad_out)
    B, Din, N = feat.shape
    K = nbr.shape[1]
    Dout = theta.shape[2]
    assert theta.shape == (3, Din, Dout) and grad_out.shape == (B, Dout, N) and nbr.shape == (B, K, N)
    assert count_bad_neighbors(nbr, N) == 0
    gp = np.zeros((B, 3, N), np.float64)
    _check(_load().oracle_flexconv_bwd_pos(_p(feat), _p(nbr), _p(theta), _p(grad_out), _p(gp), B, N, K, Din, Dout),
           "oracle_flexconv_bwd_pos")
    return gp


def block_fwd(feat, pos, nbr, W, theta, bias):
    """1x1 convolution (W [Dmid,Din0], no bias) then flex-convolution (theta [3,Dmid,Dout], bias [Dmid,Dout]).
    Returns float64 out [B,Dout,N]."""
    feat, pos, W, theta, bias, nbr = _f32(feat), _f32(pos), _f32(W), _f32(theta), _f32(bias), _i32(nbr)
    B, Din0, N = feat.shape
    K = nbr.shape[1]
    Dmid, Dout = theta.shape[1], theta.shape[2]
    assert W.shape == (Dmid, Din0) and bias.shape == (Dmid, Dout) and pos.shape == (B, 3, N)
    assert count_bad_neighbors(nbr, N) == 0
    out = np.zeros((B, Dout, N), np.float64)
    _check(_load().oracle_block_fwd(_p(feat), _p(pos), _p(nbr), _p(W), _p(theta), _p(bias), _p(out),
                                    B, N, K, Din0, Dmid, Dout), "oracle_block_fwd")
    return out


def block_bwd(feat, pos, nbr, W, theta, bias, grad_out):
    """Backward of block_fwd.  Returns (grad_feat [B,Din0,N], grad_W [Dmid,Din0], grad_theta [3,Dmid,Dout],
    grad_bias [Dmid,Dout]) in float64."""
    feat, pos, W, theta, bias, nbr = _f32(feat), _f32(pos), _f32(W), _f32(theta), _f32(bias), _i32(nbr)
    grad_out = _f32(grad_out)
    B, Din0, N = feat.shape
    K = nbr.shape[1]
    Dmid, Dout = theta.shape[1], theta.shape[2]
    assert W.shape == (Dmid, Din0) and bias.shape == (Dmid, Dout) and grad_out.shape == (B, Dout, N)
    assert count_bad_neighbors(nbr, N) == 0
    gf = np.zeros((B, Din0, N), np.float64)
    gW = np.zeros((Dmid, Din0), np.float64)
    gt = np.zeros((3, Dmid, Dout), np.float64)
    gb = np.zeros((Dmid, Dout), np.float64)
    _check(_load().oracle_block_bwd(_p(feat), _p(pos), _p(nbr), _p(W), _p(theta), _p(bias), _p(grad_out),
                                    _p(gf), _p(gW), _p(gt), _p(gb), B, N, K, Din0, Dmid, Dout), "oracle_block_bwd")
    return gf, gW, gt, gb


def idiss_phi(pos, nbr):
    """Sum of the distances to the K neighbours (Sec. 3.2).  Returns float64 [B,N]."""
    pos, nbr = _f32(pos), _i32(nbr)
    B, _, N = pos.shape
    K = nbr.shape[1]
    assert count_bad_neighbors(nbr, N) == 0
    phi = np.zeros((B, N), np.float64)
    _check(_load().oracle_idiss_phi(_p(pos), _p(nbr), _p(phi), B, N, K), "oracle_idiss_phi")
    return phi


def idiss_sample(phi, u):
    """Stratified draw of Ns = u.shape[1] points per cloud proportional to phi float32 [B,N], with the
    caller's random words u uint32 [B,Ns].  Returns sel int32 [B,Ns], ascending."""
    phi = _f32(phi)
    u = np.ascontiguousarray(u, dtype=np.uint32)
    B, N = phi.shape
    Ns = u.shape[1]
    assert u.shape == (B, Ns)
    sel = np.zeros((B, Ns), np.int32)
    _check(_load().oracle_idiss_sample(_p(phi), _p(u), _p(sel), B, N, Ns), "oracle_idiss_sample")
    return sel


def knn(pos, K):
    """Exhaustive K nearest neighbours (self included), float32 distances, ties by lower index.
    pos [B,3,N] -> nbr int32 [B,K,N]."""
    pos = _f32(pos)
    B, _, N = pos.shape
    nbr = np.zeros((B, int(K), N), np.int32)
    _check(_load().oracle_knn(_p(pos), _p(nbr), B, N, int(K)), "oracle_knn")
    return nbr


def selection_make_distinct(sel, N):
    """Ascending selection int32 [B,Ns] with repeats -> distinct ascending (repeats moved to the next free index)."""
    out = np.array(sel, dtype=np.int32, order="C", copy=True)
    B, Ns = out.shape
    _check(_load().oracle_selection_make_distinct(_p(out), B, int(N), Ns), "oracle_selection_make_distinct")
    return out
