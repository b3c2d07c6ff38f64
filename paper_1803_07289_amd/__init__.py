"""Python binding of libflexconv (flex-convolution / flex-max-pooling on gfx950).

Argument marshalling only: every step of the path runs in the HIP library.
Tensors are torch CUDA tensors (device memory and streams come from PyTorch);
work is enqueued on torch's current stream.  The functions carry the names of
the C entry points declared in include/flexconv.h.

There is no CPU fallback: if the shared library has not been built the first
call raises.
"""
import ctypes
import os

import torch

BCN = 0   # [B,C,N]  channel-major, the paper's form
BNC = 1   # [B,N,C]  point-major, the library's native form
OP_CONV_FWD, OP_CONV_BWD, OP_CONV_BWD_BUILD, OP_INEDGES, OP_UPSAMPLE = 0, 1, 2, 3, 4
OP_CONV_BWD_POS, OP_CONV_BWD_POS_BUILD = 5, 6
OP_IDISS = 7
OP_KNN = 8

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflexconv.so")
_lib = None
_workspaces = {}

_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
_SIGS = {
    "flexconv_fwd": (_i, [_vp] * 6 + [_i] * 6 + [_vp, _sz, _vp]),
    "flexconv_fwd_noalloc": (_i, [_vp] * 6 + [_i] * 6 + [_vp]),
    "flexconv_bwd": (_i, [_vp] * 11 + [_i] * 6 + [_vp, _sz, _vp]),
    "flex_inedges_build": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "flexpool_fwd": (_i, [_vp] * 4 + [_i] * 5 + [_vp]),
    "flexpool_bwd": (_i, [_vp] * 5 + [_i] * 5 + [_vp]),
    "flexpool_plan_bytes": (_sz, [_i] * 3),
    "flexpool_plan_build": (_i, [_vp, _vp, _i, _i, _i, _vp, _sz, _vp]),
    "flexpool_bwd_planned": (_i, [_vp] * 6 + [_sz] + [_i] * 5 + [_vp]),
    "flexpool_fwd_plan_build": (_i, [_vp, _i, _i, _i, _vp, _sz, _vp]),
    "flexpool_fwd_planned": (_i, [_vp] * 5 + [_sz] + [_i] * 5 + [_vp]),
    "flexconv_bwd_pos": (_i, [_vp] * 7 + [_i] * 6 + [_vp, _sz, _vp]),
    "flexconv_compose_1x1": (_i, [_vp] * 5 + [_i] * 3 + [_vp]),
    "flexconv_compose_1x1_bwd": (_i, [_vp] * 8 + [_i] * 3 + [_vp]),
    "flex_selection_make_distinct": (_i, [_vp, _i, _i, _i, _vp, _sz, _vp]),
    "flex_knn": (_i, [_vp, _vp, _i, _i, _i, _vp, _sz, _vp]),
    "flex_idiss_phi": (_i, [_vp] * 3 + [_i] * 3 + [_vp]),
    "flex_idiss_sample": (_i, [_vp] * 3 + [_i] * 3 + [_vp, _sz, _vp]),
    "flexpool_sub_fwd": (_i, [_vp] * 5 + [_i] * 6 + [_vp]),
    "flexpool_sub_bwd": (_i, [_vp] * 5 + [_i] * 6 + [_vp]),
    "flex_inedges_build_sub": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "flexupsample_fwd": (_i, [_vp] * 5 + [_i] * 6 + [_vp, _sz, _vp]),
    "flexupsample_bwd": (_i, [_vp] * 6 + [_i] * 6 + [_vp]),
    "flex_validate_selection": (_i, [_vp, _i, _i, _i, _vp, _vp, _sz, _vp]),
    "flexconv_workspace_bytes": (_sz, [_i] * 7),
    "flex_validate_neighbors": (_i, [_vp, _i, _i, _i, _vp, _vp]),
    "flexconv_has_fast_path": (_i, [_i, _i]),
    "flexconv_kernel_route": (_i, [_i] * 7),
    "flex_status_string": (ctypes.c_char_p, [_i]),
    "flex_calibrate_copy": (_i, [_vp, _vp, _sz, _vp]),
    "flex_calibrate_mfma_f16": (_i, [_i, _vp, ctypes.POINTER(ctypes.c_double), _vp]),
}


def lib():
    """The loaded shared library (raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_1803_07289_amd.build` (no CPU fallback exists)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


class FlexError(RuntimeError):
    pass


def _check(status, what):
    if status != 0:
        raise FlexError(f"{what}: {lib().flex_status_string(status).decode()} (status {status})")


def _layout(layout):
    if layout in (BCN, "bcn", "BCN"):
        return BCN
    if layout in (BNC, "bnc", "BNC"):
        return BNC
    raise ValueError(f"unknown layout {layout!r}")


def _dev(t, dtype, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dims(feat, nbr, layout):
    """(B, N, K, C) from a feature tensor and the index tensor."""
    if feat.dim() != 3 or nbr.dim() != 3:
        raise ValueError("feat and nbr must be 3-D")
    B, K, N = nbr.shape
    C = feat.shape[1] if layout == BCN else feat.shape[2]
    want = (B, C, N) if layout == BCN else (B, N, C)
    if tuple(feat.shape) != want:
        raise ValueError(f"feat shape {tuple(feat.shape)} does not match nbr {tuple(nbr.shape)} in this layout")
    return B, N, K, C


def workspace_bytes(op, B, N, K, Din, Dout, layout=BCN):
    return int(lib().flexconv_workspace_bytes(op, B, N, K, Din, Dout, _layout(layout)))


def _workspace(device, nbytes):
    """A cached, grow-only scratch tensor per device (256-byte aligned by the allocator)."""
    key = (device.type, device.index)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        _workspaces[key] = None
        ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _ws_arg(workspace, device, need):
    """(tensor, byte count handed to the library): a caller's workspace with its own size, else the cached one
    with exactly the size the library asked for, so that the library's own size check sees `need`."""
    if workspace is not None:
        if not workspace.is_cuda or workspace.dtype != torch.uint8 or not workspace.is_contiguous():
            raise TypeError("workspace must be a contiguous CUDA uint8 tensor")
        return workspace, workspace.numel()
    return _workspace(device, need), max(int(need), 256)


def kernel_route(op, B, N, K, Din, Dout, layout=BCN):
    """Which kernel family a call of these sizes runs on (a flex_route value of include/flexconv.h; host query)."""
    return int(lib().flexconv_kernel_route(op, B, N, K, Din, Dout, _layout(layout)))


def flexconv_fwd(feat, pos, nbr, theta, bias, layout=BCN, out=None, workspace=None):
    """Flex-convolution forward (Eq. 4 with the weight of Eq. 6).  Returns out."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(pos, torch.float32, "pos"); _dev(nbr, torch.int32, "nbr")
    _dev(theta, torch.float32, "theta"); _dev(bias, torch.float32, "bias")
    B, N, K, Din = _dims(feat, nbr, layout)
    if theta.dim() != 3 or theta.shape[0] != 3 or theta.shape[1] != Din:
        raise ValueError("theta must be [3,Din,Dout]")
    Dout = theta.shape[2]
    if tuple(bias.shape) != (Din, Dout) or tuple(pos.shape) != (B, 3, N):
        raise ValueError("bias must be [Din,Dout] and pos [B,3,N]")
    shape = (B, Dout, N) if layout == BCN else (B, N, Dout)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=feat.device)
    elif tuple(_dev(out, torch.float32, "out").shape) != shape:
        raise ValueError("out has the wrong shape")
    need = workspace_bytes(OP_CONV_FWD, B, N, K, Din, Dout, layout)
    ws, ws_bytes = _ws_arg(workspace, feat.device, need)
    _check(lib().flexconv_fwd(_ptr(feat), _ptr(pos), _ptr(nbr), _ptr(theta), _ptr(bias), _ptr(out),
                              B, N, K, Din, Dout, layout, _ptr(ws), ws_bytes, _stream()), "flexconv_fwd")
    return out


def flexconv_fwd_noalloc(feat, pos, nbr, theta, bias, out, layout=BCN):
    """flexconv_fwd into the caller's `out`, with the library's static scratch memory instead of a workspace:
    neither this wrapper nor the library allocates.  Raises FlexError (status 6) when the call needs more
    scratch than the static buffer holds."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(pos, torch.float32, "pos"); _dev(nbr, torch.int32, "nbr")
    _dev(theta, torch.float32, "theta"); _dev(bias, torch.float32, "bias"); _dev(out, torch.float32, "out")
    B, N, K, Din = _dims(feat, nbr, layout)
    if theta.dim() != 3 or theta.shape[0] != 3 or theta.shape[1] != Din:
        raise ValueError("theta must be [3,Din,Dout]")
    Dout = theta.shape[2]
    if tuple(bias.shape) != (Din, Dout) or tuple(pos.shape) != (B, 3, N):
        raise ValueError("bias must be [Din,Dout] and pos [B,3,N]")
    if tuple(out.shape) != ((B, Dout, N) if layout == BCN else (B, N, Dout)):
        raise ValueError("out has the wrong shape")
    _check(lib().flexconv_fwd_noalloc(_ptr(feat), _ptr(pos), _ptr(nbr), _ptr(theta), _ptr(bias), _ptr(out),
                                      B, N, K, Din, Dout, layout, _stream()), "flexconv_fwd_noalloc")
    return out


def flex_inedges_build(nbr, workspace=None):
    """Transposed neighbour graph of nbr [B,K,N]: (in_off int32 [B*N+1], in_src int32 [B*K*N])."""
    _dev(nbr, torch.int32, "nbr")
    B, K, N = nbr.shape
    in_off = torch.empty(B * N + 1, dtype=torch.int32, device=nbr.device)
    in_src = torch.empty(B * K * N, dtype=torch.int32, device=nbr.device)
    need = workspace_bytes(OP_INEDGES, B, N, K, 1, 1, BCN)
    ws, ws_bytes = _ws_arg(workspace, nbr.device, need)
    _check(lib().flex_inedges_build(_ptr(nbr), B, N, K, _ptr(in_off), _ptr(in_src), _ptr(ws), ws_bytes,
                                    _stream()), "flex_inedges_build")
    return in_off, in_src


def flexconv_bwd(feat, pos, nbr, theta, bias, grad_out, layout=BCN, in_edges=None,
                 need_feat=True, need_params=True, workspace=None):
    """Flex-convolution backward.  Returns (grad_feat, grad_theta, grad_bias); entries not asked
    for are None.  in_edges = (in_off, in_src) from flex_inedges_build, or None to build per call."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(pos, torch.float32, "pos"); _dev(nbr, torch.int32, "nbr")
    _dev(theta, torch.float32, "theta"); _dev(bias, torch.float32, "bias")
    _dev(grad_out, torch.float32, "grad_out")
    B, N, K, Din = _dims(feat, nbr, layout)
    if theta.dim() != 3 or theta.shape[0] != 3 or theta.shape[1] != Din:
        raise ValueError("theta must be [3,Din,Dout]")
    Dout = theta.shape[2]
    if tuple(bias.shape) != (Din, Dout) or tuple(pos.shape) != (B, 3, N):
        raise ValueError("bias must be [Din,Dout] and pos [B,3,N]")
    gshape = (B, Dout, N) if layout == BCN else (B, N, Dout)
    if tuple(grad_out.shape) != gshape:
        raise ValueError("grad_out has the wrong shape")
    gf = torch.empty_like(feat) if need_feat else None
    gt = torch.empty_like(theta) if need_params else None
    gb = torch.empty_like(bias) if need_params else None
    off = src = None
    if in_edges is not None:
        off, src = in_edges
        _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src")
        if off.numel() != B * N + 1 or src.numel() != B * K * N:
            raise ValueError("in_edges do not match nbr")
    op = OP_CONV_BWD if in_edges is not None else OP_CONV_BWD_BUILD
    need = workspace_bytes(op, B, N, K, Din, Dout, layout)
    ws, ws_bytes = _ws_arg(workspace, feat.device, need)
    _check(lib().flexconv_bwd(_ptr(feat), _ptr(pos), _ptr(nbr), _ptr(theta), _ptr(bias), _ptr(grad_out),
                              _ptr(gf), _ptr(gt), _ptr(gb), _ptr(off), _ptr(src),
                              B, N, K, Din, Dout, layout, _ptr(ws), ws_bytes, _stream()), "flexconv_bwd")
    return gf, gt, gb


def flexconv_bwd_pos(feat, nbr, theta, grad_out, layout=BCN, in_edges=None, workspace=None):
    """Gradient of the flex-convolution with respect to the point locations: [B,3,N] like pos."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(nbr, torch.int32, "nbr"); _dev(theta, torch.float32, "theta")
    _dev(grad_out, torch.float32, "grad_out")
    B, N, K, Din = _dims(feat, nbr, layout)
    if theta.dim() != 3 or theta.shape[0] != 3 or theta.shape[1] != Din:
        raise ValueError("theta must be [3,Din,Dout]")
    Dout = theta.shape[2]
    if tuple(grad_out.shape) != ((B, Dout, N) if layout == BCN else (B, N, Dout)):
        raise ValueError("grad_out has the wrong shape")
    off = src = None
    if in_edges is not None:
        off, src = in_edges
        _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src")
        if off.numel() != B * N + 1 or src.numel() != B * K * N:
            raise ValueError("in_edges do not match nbr")
    gp = torch.empty((B, 3, N), dtype=torch.float32, device=feat.device)
    op = OP_CONV_BWD_POS if in_edges is not None else OP_CONV_BWD_POS_BUILD
    need = workspace_bytes(op, B, N, K, Din, Dout, layout)
    ws, ws_bytes = _ws_arg(workspace, feat.device, need)
    _check(lib().flexconv_bwd_pos(_ptr(feat), _ptr(nbr), _ptr(theta), _ptr(grad_out), _ptr(off), _ptr(src), _ptr(gp),
                                  B, N, K, Din, Dout, layout, _ptr(ws), ws_bytes, _stream()), "flexconv_bwd_pos")
    return gp


def flexpool_fwd(feat, nbr, layout=BCN):
    """Flex-max-pooling forward.  Returns (out, argmax int32), both shaped like feat."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(nbr, torch.int32, "nbr")
    B, N, K, C = _dims(feat, nbr, layout)
    out = torch.empty_like(feat)
    arg = torch.empty(feat.shape, dtype=torch.int32, device=feat.device)
    _check(lib().flexpool_fwd(_ptr(feat), _ptr(nbr), _ptr(out), _ptr(arg), B, N, K, C, layout, _stream()),
           "flexpool_fwd")
    return out, arg


def flexpool_bwd(grad_out, argmax, layout=BCN, in_edges=None, K=None):
    """Flex-max-pooling backward (routing by the recorded winners).  Returns grad_feat.
    in_edges = (in_off, in_src) of the forward pass's nbr selects the atomic-free gather form."""
    layout = _layout(layout)
    _dev(grad_out, torch.float32, "grad_out"); _dev(argmax, torch.int32, "argmax")
    if grad_out.dim() != 3 or grad_out.shape != argmax.shape:
        raise ValueError("grad_out and argmax must be 3-D and equal in shape")
    B = grad_out.shape[0]
    C, N = (grad_out.shape[1], grad_out.shape[2]) if layout == BCN else (grad_out.shape[2], grad_out.shape[1])
    off = src = None
    k = 1
    if in_edges is not None:
        off, src = in_edges
        _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src")
        if off.numel() != B * N + 1 or src.numel() % (B * N) != 0:
            raise ValueError("in_edges do not match the tensors")
        k = src.numel() // (B * N)
        if K is not None and K != k:
            raise ValueError("in_edges were built for a different K")
    gf = torch.empty_like(grad_out)
    _check(lib().flexpool_bwd(_ptr(grad_out), _ptr(argmax), _ptr(gf), _ptr(off), _ptr(src), B, N, k, C, layout,
                              _stream()), "flexpool_bwd")
    return gf


def flexpool_plan_build(in_edges, B, N):
    """Static gather plan of the pooling backward pass for the lists in_edges = (in_off, in_src) of B clouds of N
    points: a uint8 device tensor to pass to flexpool_bwd_planned.  Depends on the lists only: build once per cloud."""
    off, src = in_edges
    _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src")
    if off.numel() != B * N + 1 or src.numel() % (B * N) != 0:
        raise ValueError("in_edges do not match (B, N)")
    K = src.numel() // (B * N)
    need = int(lib().flexpool_plan_bytes(B, N, K))
    if need == 0:
        raise ValueError("sizes out of range")
    plan = torch.empty(need, dtype=torch.uint8, device=off.device)
    _check(lib().flexpool_plan_build(_ptr(off), _ptr(src), B, N, K, _ptr(plan), need, _stream()), "flexpool_plan_build")
    return plan


def flexpool_fwd_plan_build(nbr):
    """Static gather plan of the pooling forward pass for nbr [B,K,N]: a uint8 device tensor to pass to
    flexpool_fwd_planned.  Depends on nbr only: build once per cloud."""
    _dev(nbr, torch.int32, "nbr")
    B, K, N = nbr.shape
    need = int(lib().flexpool_plan_bytes(B, N, K))
    if need == 0:
        raise ValueError("sizes out of range")
    plan = torch.empty(need, dtype=torch.uint8, device=nbr.device)
    _check(lib().flexpool_fwd_plan_build(_ptr(nbr), B, N, K, _ptr(plan), need, _stream()), "flexpool_fwd_plan_build")
    return plan


def flexpool_fwd_planned(feat, nbr, plan, layout=BCN):
    """Flex-max-pooling forward through the static gather plan: (out, argmax) of flexpool_fwd, bit for bit."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(nbr, torch.int32, "nbr"); _dev(plan, torch.uint8, "plan")
    if feat.dim() != 3 or nbr.dim() != 3 or nbr.shape[0] != feat.shape[0]:
        raise ValueError("feat must be 3-D and nbr [B,K,N]")
    B, K, N = nbr.shape
    C = feat.shape[1] if layout == BCN else feat.shape[2]
    if (feat.shape[2] if layout == BCN else feat.shape[1]) != N:
        raise ValueError("feat and nbr disagree about N")
    out = torch.empty_like(feat)
    argmax = torch.empty(feat.shape, dtype=torch.int32, device=feat.device)
    _check(lib().flexpool_fwd_planned(_ptr(feat), _ptr(nbr), _ptr(out), _ptr(argmax), _ptr(plan), plan.numel(),
                                      B, N, K, C, layout, _stream()), "flexpool_fwd_planned")
    return out, argmax


def flexpool_bwd_planned(grad_out, argmax, in_edges, plan, layout=BCN):
    """Flex-max-pooling backward through the static gather plan: the result of flexpool_bwd(..., in_edges=...), bit
    for bit.  Returns grad_feat."""
    layout = _layout(layout)
    _dev(grad_out, torch.float32, "grad_out"); _dev(argmax, torch.int32, "argmax")
    if grad_out.dim() != 3 or grad_out.shape != argmax.shape:
        raise ValueError("grad_out and argmax must be 3-D and equal in shape")
    B = grad_out.shape[0]
    C, N = (grad_out.shape[1], grad_out.shape[2]) if layout == BCN else (grad_out.shape[2], grad_out.shape[1])
    off, src = in_edges
    _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src"); _dev(plan, torch.uint8, "plan")
    if off.numel() != B * N + 1 or src.numel() % (B * N) != 0:
        raise ValueError("in_edges do not match the tensors")
    K = src.numel() // (B * N)
    gf = torch.empty_like(grad_out)
    _check(lib().flexpool_bwd_planned(_ptr(grad_out), _ptr(argmax), _ptr(gf), _ptr(off), _ptr(src), _ptr(plan),
                                      plan.numel(), B, N, K, C, layout, _stream()), "flexpool_bwd_planned")
    return gf


def flexconv_compose_1x1(W, theta, bias):
    """Parameters of the flex-convolution that equals `1x1 convolution W [Dmid,Din0] (no bias), then
    flexconv(theta [3,Dmid,Dout], bias [Dmid,Dout])` (Sec. 4.3 block).  Returns (theta_c [3,Din0,Dout], bias_c [Din0,Dout])."""
    _dev(W, torch.float32, "W"); _dev(theta, torch.float32, "theta"); _dev(bias, torch.float32, "bias")
    Dmid, Din0 = W.shape
    if theta.dim() != 3 or theta.shape[0] != 3 or theta.shape[1] != Dmid or tuple(bias.shape) != (Dmid, theta.shape[2]):
        raise ValueError("theta must be [3,Dmid,Dout] and bias [Dmid,Dout] for W [Dmid,Din0]")
    Dout = theta.shape[2]
    W, theta, bias = W.contiguous(), theta.contiguous(), bias.contiguous()
    tc = torch.empty((3, Din0, Dout), dtype=torch.float32, device=W.device)
    bc = torch.empty((Din0, Dout), dtype=torch.float32, device=W.device)
    _check(lib().flexconv_compose_1x1(_ptr(W), _ptr(theta), _ptr(bias), _ptr(tc), _ptr(bc), Din0, Dmid, Dout, _stream()),
           "flexconv_compose_1x1")
    return tc, bc


def flexconv_compose_1x1_bwd(W, theta, bias, grad_theta_c, grad_bias_c):
    """Gradients of (W, theta, bias) from those of the composed parameters.  Returns (grad_W, grad_theta, grad_bias)."""
    for t, n in ((W, "W"), (theta, "theta"), (bias, "bias"), (grad_theta_c, "grad_theta_c"), (grad_bias_c, "grad_bias_c")):
        _dev(t, torch.float32, n)
    Dmid, Din0 = W.shape
    Dout = theta.shape[2]
    if tuple(theta.shape) != (3, Dmid, Dout) or tuple(bias.shape) != (Dmid, Dout) or \
            tuple(grad_theta_c.shape) != (3, Din0, Dout) or tuple(grad_bias_c.shape) != (Din0, Dout):
        raise ValueError("shapes do not match W [Dmid,Din0]")
    W, theta, bias = W.contiguous(), theta.contiguous(), bias.contiguous()
    grad_theta_c, grad_bias_c = grad_theta_c.contiguous(), grad_bias_c.contiguous()
    gW, gt, gb = torch.empty_like(W), torch.empty_like(theta), torch.empty_like(bias)
    _check(lib().flexconv_compose_1x1_bwd(_ptr(W), _ptr(theta), _ptr(bias), _ptr(grad_theta_c), _ptr(grad_bias_c),
                                          _ptr(gW), _ptr(gt), _ptr(gb), Din0, Dmid, Dout, _stream()),
           "flexconv_compose_1x1_bwd")
    return gW, gt, gb


def flex_knn(pos, K, workspace=None):
    """Exact K nearest neighbours of every point of pos [B,3,N] (itself included), ordered by (distance, index).
    Returns nbr int32 [B,K,N]."""
    _dev(pos, torch.float32, "pos")
    if pos.dim() != 3 or pos.shape[1] != 3:
        raise ValueError("pos must be [B,3,N]")
    B, _, N = pos.shape
    nbr = torch.empty((B, int(K), N), dtype=torch.int32, device=pos.device)
    need = workspace_bytes(OP_KNN, B, N, int(K), 1, 1, BCN)
    if need == 0:
        raise ValueError(f"flex_knn does not take B={B}, N={N}, K={K}")
    ws, ws_bytes = _ws_arg(workspace, pos.device, need)
    _check(lib().flex_knn(_ptr(pos.contiguous()), _ptr(nbr), B, N, int(K), _ptr(ws), ws_bytes, _stream()), "flex_knn")
    return nbr


def flex_idiss_phi(pos, nbr):
    """phi [B,N]: sum of the distances from every point to its K neighbours (Sec. 3.2)."""
    _dev(pos, torch.float32, "pos"); _dev(nbr, torch.int32, "nbr")
    B, K, N = nbr.shape
    if tuple(pos.shape) != (B, 3, N):
        raise ValueError("pos must be [B,3,N]")
    phi = torch.empty((B, N), dtype=torch.float32, device=pos.device)
    _check(lib().flex_idiss_phi(_ptr(pos.contiguous()), _ptr(nbr), _ptr(phi), B, N, K, _stream()), "flex_idiss_phi")
    return phi


def flex_idiss_sample(phi, u, workspace=None):
    """Ns = u.shape[1] points per cloud drawn proportionally to phi [B,N] from the random words u (an int32 or
    uint32-valued tensor [B,Ns], taken bit for bit).  Returns sel int32 [B,Ns], ascending."""
    _dev(phi, torch.float32, "phi")
    if not u.is_cuda or u.dtype not in (torch.int32, torch.uint32) or u.dim() != 2:
        raise TypeError("u must be a CUDA int32 / uint32 tensor [B,Ns]")
    B, N = phi.shape
    Ns = u.shape[1]
    if u.shape[0] != B:
        raise ValueError("u must be [B,Ns]")
    sel = torch.empty((B, Ns), dtype=torch.int32, device=phi.device)
    need = workspace_bytes(OP_IDISS, B, N, 1, 1, 1, BCN)
    ws, ws_bytes = _ws_arg(workspace, phi.device, need)
    _check(lib().flex_idiss_sample(_ptr(phi.contiguous()), _ptr(u.contiguous()), _ptr(sel), B, N, Ns, _ptr(ws),
                                   ws_bytes, _stream()), "flex_idiss_sample")
    return sel


def flex_selection_make_distinct(sel, N, workspace=None):
    """In place: an ascending selection int32 [B,Ns] with repeats becomes distinct (a repeated entry moves to the
    next free index).  Returns sel."""
    _dev(sel, torch.int32, "sel")
    if sel.dim() != 2 or not sel.is_contiguous():
        raise ValueError("sel must be a contiguous [B,Ns] tensor")
    B, Ns = sel.shape
    need = workspace_bytes(OP_IDISS, B, N, 1, 1, 1, BCN)
    ws, ws_bytes = _ws_arg(workspace, sel.device, need)
    _check(lib().flex_selection_make_distinct(_ptr(sel), B, int(N), Ns, _ptr(ws), ws_bytes, _stream()),
           "flex_selection_make_distinct")
    return sel


def flexpool_sub_fwd(feat, nbr, sel, layout=BCN):
    """Flex-max-pooling with subsampling (Sec. 4.1 / 5): the pooled rows of the kept centres sel [B,Ns]
    only.  Returns (out, argmax int32), shaped [B,C,Ns] / [B,Ns,C]; argmax indexes the N input points."""
    layout = _layout(layout)
    _dev(feat, torch.float32, "feat"); _dev(nbr, torch.int32, "nbr"); _dev(sel, torch.int32, "sel")
    B, N, K, C = _dims(feat, nbr, layout)
    if sel.dim() != 2 or sel.shape[0] != B:
        raise ValueError("sel must be [B,Ns]")
    Ns = sel.shape[1]
    shape = (B, C, Ns) if layout == BCN else (B, Ns, C)
    out = torch.empty(shape, dtype=torch.float32, device=feat.device)
    arg = torch.empty(shape, dtype=torch.int32, device=feat.device)
    _check(lib().flexpool_sub_fwd(_ptr(feat), _ptr(nbr), _ptr(sel), _ptr(out), _ptr(arg), B, N, Ns, K, C, layout,
                                  _stream()), "flexpool_sub_fwd")
    return out, arg


def flex_inedges_build_sub(nbr, sel, workspace=None):
    """Transposed neighbour lists over the kept centres sel [B,Ns] of nbr [B,K,N]: (in_off [B*N+1],
    in_src [B*K*Ns]) for flexpool_sub_bwd.  Static per layer: build once."""
    _dev(nbr, torch.int32, "nbr"); _dev(sel, torch.int32, "sel")
    B, K, N = nbr.shape
    if sel.dim() != 2 or sel.shape[0] != B:
        raise ValueError("sel must be [B,Ns]")
    Ns = sel.shape[1]
    off = torch.empty(B * N + 1, dtype=torch.int32, device=nbr.device)
    src = torch.empty(B * K * Ns, dtype=torch.int32, device=nbr.device)
    need = workspace_bytes(OP_INEDGES, B, N, K, 1, 1, BCN)
    ws, ws_bytes = _ws_arg(workspace, nbr.device, need)
    _check(lib().flex_inedges_build_sub(_ptr(nbr), _ptr(sel), B, N, Ns, K, _ptr(off), _ptr(src), _ptr(ws),
                                        ws_bytes, _stream()), "flex_inedges_build_sub")
    return off, src


def flexpool_sub_bwd(grad_out, argmax, N, layout=BCN, in_edges=None):
    """Backward of flexpool_sub_fwd.  Returns grad_feat [B,C,N] / [B,N,C].  in_edges = (in_off, in_src) from
    flex_inedges_build_sub(nbr, sel) selects the atomic-free gather form."""
    layout = _layout(layout)
    _dev(grad_out, torch.float32, "grad_out"); _dev(argmax, torch.int32, "argmax")
    if grad_out.dim() != 3 or grad_out.shape != argmax.shape:
        raise ValueError("grad_out and argmax must be 3-D and equal in shape")
    B = grad_out.shape[0]
    C, Ns = (grad_out.shape[1], grad_out.shape[2]) if layout == BCN else (grad_out.shape[2], grad_out.shape[1])
    off = src = None
    k = 1
    if in_edges is not None:
        off, src = in_edges
        _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src")
        if off.numel() != B * N + 1 or src.numel() % (B * Ns) != 0:
            raise ValueError("in_edges do not match the tensors")
        k = src.numel() // (B * Ns)
    gf = torch.empty((B, C, N) if layout == BCN else (B, N, C), dtype=torch.float32, device=grad_out.device)
    _check(lib().flexpool_sub_bwd(_ptr(grad_out), _ptr(argmax), _ptr(off), _ptr(src), _ptr(gf),
                                  B, N, Ns, k, C, layout, _stream()), "flexpool_sub_bwd")
    return gf


def _up_dims(small, sel, layout):
    if small.dim() != 3 or sel.dim() != 2:
        raise ValueError("the smaller layer's tensor must be 3-D and sel 2-D")
    B, Ns = sel.shape
    C = small.shape[1] if layout == BCN else small.shape[2]
    want = (B, C, Ns) if layout == BCN else (B, Ns, C)
    if tuple(small.shape) != want:
        raise ValueError(f"tensor shape {tuple(small.shape)} does not match sel {tuple(sel.shape)} in this layout")
    return B, Ns, C


def flexupsample_fwd(feat_small, sel, nbr, layout=BCN, workspace=None):
    """Flex-upsampling forward (Sec. 4.1): copy the smaller layer's features to their points sel
    [B,Ns] of the larger layer, zero elsewhere, flex-max-pool over nbr [B,K,Nf].
    Returns (out, argmax int32), shaped [B,C,Nf] / [B,Nf,C]."""
    layout = _layout(layout)
    _dev(feat_small, torch.float32, "feat_small"); _dev(sel, torch.int32, "sel"); _dev(nbr, torch.int32, "nbr")
    B, Ns, C = _up_dims(feat_small, sel, layout)
    if nbr.dim() != 3 or nbr.shape[0] != B:
        raise ValueError("nbr must be [B,K,Nf]")
    K, Nf = nbr.shape[1], nbr.shape[2]
    shape = (B, C, Nf) if layout == BCN else (B, Nf, C)
    out = torch.empty(shape, dtype=torch.float32, device=feat_small.device)
    arg = torch.empty(shape, dtype=torch.int32, device=feat_small.device)
    need = workspace_bytes(OP_UPSAMPLE, B, Nf, K, C, 1, layout)
    ws, ws_bytes = _ws_arg(workspace, feat_small.device, need)
    _check(lib().flexupsample_fwd(_ptr(feat_small), _ptr(sel), _ptr(nbr), _ptr(out), _ptr(arg), B, Ns, Nf, K, C,
                                  layout, _ptr(ws), ws_bytes, _stream()), "flexupsample_fwd")
    return out, arg


def flexupsample_bwd(grad_out, argmax, sel, in_edges, layout=BCN):
    """Flex-upsampling backward.  in_edges = (in_off, in_src) of the larger layer's nbr.
    Returns grad_small shaped [B,C,Ns] / [B,Ns,C]."""
    layout = _layout(layout)
    _dev(grad_out, torch.float32, "grad_out"); _dev(argmax, torch.int32, "argmax"); _dev(sel, torch.int32, "sel")
    if grad_out.dim() != 3 or grad_out.shape != argmax.shape or sel.dim() != 2:
        raise ValueError("grad_out and argmax must be 3-D and equal in shape, sel 2-D")
    B, Ns = sel.shape
    C, Nf = (grad_out.shape[1], grad_out.shape[2]) if layout == BCN else (grad_out.shape[2], grad_out.shape[1])
    off, src = in_edges
    _dev(off, torch.int32, "in_off"); _dev(src, torch.int32, "in_src")
    if grad_out.shape[0] != B or off.numel() != B * Nf + 1 or src.numel() % (B * Nf) != 0:
        raise ValueError("in_edges do not match the tensors")
    k = src.numel() // (B * Nf)
    gs = torch.empty((B, C, Ns) if layout == BCN else (B, Ns, C), dtype=torch.float32, device=grad_out.device)
    _check(lib().flexupsample_bwd(_ptr(grad_out), _ptr(argmax), _ptr(sel), _ptr(off), _ptr(src), _ptr(gs),
                                  B, Ns, Nf, k, C, layout, _stream()), "flexupsample_bwd")
    return gs


def flex_validate_selection(sel, Nf, workspace=None):
    """Number of entries of sel [B,Ns] outside [0,Nf) or repeating another entry of their cloud (synchronises)."""
    _dev(sel, torch.int32, "sel")
    B, Ns = sel.shape
    bad = torch.zeros(1, dtype=torch.int32, device=sel.device)
    need = workspace_bytes(OP_UPSAMPLE, B, Nf, 1, 1, 1, BCN)
    ws, ws_bytes = _ws_arg(workspace, sel.device, need)
    _check(lib().flex_validate_selection(_ptr(sel), B, Ns, Nf, _ptr(bad), _ptr(ws), ws_bytes, _stream()),
           "flex_validate_selection")
    return int(bad.item())


def flex_validate_neighbors(nbr):
    """Number of entries of nbr [B,K,N] outside [0,N) (synchronises)."""
    _dev(nbr, torch.int32, "nbr")
    B, K, N = nbr.shape
    bad = torch.zeros(1, dtype=torch.int32, device=nbr.device)
    _check(lib().flex_validate_neighbors(_ptr(nbr), B, N, K, _ptr(bad), _stream()), "flex_validate_neighbors")
    return int(bad.item())


def flex_calibrate_copy(src, dst):
    """Measurement aid: dst = src by a plain copy kernel (time it with events)."""
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()) or \
            src.numel() * src.element_size() != dst.numel() * dst.element_size():
        raise ValueError("src and dst must be contiguous CUDA tensors of equal byte size")
    _check(lib().flex_calibrate_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()),
           "flex_calibrate_copy")
    return dst


def flex_calibrate_mfma_f16(iters, sink):
    """Measurement aid: a pure f16 matrix-op loop on every compute unit; returns the launch's flop count."""
    _dev(sink, torch.float32, "sink")
    flop = ctypes.c_double(0.0)
    _check(lib().flex_calibrate_mfma_f16(int(iters), _ptr(sink), ctypes.byref(flop), _stream()),
           "flex_calibrate_mfma_f16")
    return float(flop.value)


def has_fast_path(Din, Dout):
    """True if flexconv_fwd / flexconv_bwd run these widths on the matrix-core kernels (natively, as block passes or
    zero-padded) rather than on the direct-form kernels."""
    return bool(lib().flexconv_has_fast_path(int(Din), int(Dout)))
