"""The allocation-free forward entry point (flexconv_fwd_noalloc: the library's static device scratch instead of a
caller workspace) against flexconv_fwd, through the C ABI: two calls in a row, the second with a smaller input, then
other widths and layouts, the size limit, and the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1803_07289_amd as fx
from gpu_util import TOL, dev, to_layout, from_layout, say
from helpers import rel_err
from test_gpu_parity import random_problem

pytestmark = pytest.mark.gpu


def call_noalloc_raw(feat, pos, nbr, theta, bias, out, B, N, K, Din, Dout, layout):
    """Straight through the C ABI: plain pointers and sizes."""
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return fx.lib().flexconv_fwd_noalloc(p(feat), p(pos), p(nbr), p(theta), p(bias), p(out), B, N, K, Din, Dout,
                                         layout, stream)


def one_case(seed, B, N, K, Din, Dout, layout):
    pos, nbr, feat, theta, bias, _ = random_problem(seed, B, N, K, Din, Dout)
    a = (to_layout(feat, layout), dev(pos), dev(nbr), dev(theta), dev(bias))
    want = fx.flexconv_fwd(*a, layout=layout)                     # the existing entry point, caller workspace
    got = torch.full_like(want, float("nan"))
    mem = torch.cuda.memory_allocated()
    st = call_noalloc_raw(*a, got, B, N, K, Din, Dout, layout)
    assert st == 0, fx.lib().flex_status_string(st)
    assert torch.cuda.memory_allocated() == mem                   # nothing came from torch's allocator either
    torch.cuda.synchronize()
    assert torch.equal(got, want)                                 # same kernels, same arithmetic: bit for bit
    ref = oracle.flexconv_fwd(feat, pos, nbr, theta, bias)
    assert rel_err(from_layout(got, layout), ref) <= TOL


def test_two_calls_in_a_row_the_second_smaller():
    say("noalloc: 3000 points 64->64, then 500 points 32->32")
    one_case(1, 1, 3000, 8, 64, 64, fx.BNC)
    one_case(2, 1, 500, 8, 32, 32, fx.BNC)       # smaller input, smaller plan: the scratch still holds the first call's bytes
    one_case(3, 2, 777, 16, 64, 64, fx.BNC)


@pytest.mark.parametrize("B,N,K,Din,Dout,layout", [
    (1, 1000, 8, 128, 128, fx.BNC),       # two passes, parameter blocks extracted in the scratch
    (1, 400, 8, 256, 256, fx.BNC),        # block passes: all packed parameter blocks (1.06 MB)
    (2, 300, 9, 64, 32, fx.BCN),          # channel-major: transposed copy in the scratch
    (1, 250, 8, 5, 7, fx.BCN),            # zero-padded widths: padded copies in the scratch
    (1, 257, 8, 9, 64, fx.BNC),
])
def test_other_plans_fit_the_static_scratch(B, N, K, Din, Dout, layout):
    say(f"noalloc: B={B} N={N} K={K} Din={Din} Dout={Dout} layout={layout}")
    assert fx.workspace_bytes(fx.OP_CONV_FWD, B, N, K, Din, Dout, layout) <= (2 << 20)
    one_case(10 + N, B, N, K, Din, Dout, layout)


def test_calls_beyond_the_static_scratch_are_refused_before_any_launch():
    B, N, K, Din, Dout = 1, 20000, 8, 64, 64
    assert fx.workspace_bytes(fx.OP_CONV_FWD, B, N, K, Din, Dout, fx.BCN) > (2 << 20)      # the transposed copy alone is 5 MB
    pos, nbr, feat, theta, bias, _ = random_problem(5, B, N, K, Din, Dout)
    a = (to_layout(feat, fx.BCN), dev(pos), dev(nbr), dev(theta), dev(bias))
    out = torch.full((B, Dout, N), 7.0, device="cuda")
    assert call_noalloc_raw(*a, out, B, N, K, Din, Dout, fx.BCN) == 6
    with pytest.raises(fx.FlexError, match="static buffer"):
        fx.flexconv_fwd_noalloc(*a, out, layout=fx.BCN)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                                # nothing was launched
    # the same layer point-major needs the packed parameters only
    out2 = torch.empty((B, N, Dout), device="cuda")
    fx.flexconv_fwd_noalloc(to_layout(feat, fx.BNC), *a[1:], out2, layout=fx.BNC)
    assert torch.equal(out2, fx.flexconv_fwd(to_layout(feat, fx.BNC), *a[1:], layout=fx.BNC))
    # 512 x 512: the packed parameter blocks alone exceed the buffer
    assert fx.lib().flexconv_fwd_noalloc(*[ctypes.c_void_p(256)] * 6, 1, 4096, 8, 512, 512, 1, None) == 6
    assert fx.lib().flexconv_fwd_noalloc(None, *[ctypes.c_void_p(256)] * 5, 1, 4096, 8, 64, 64, 1, None) == 1
    assert fx.lib().flexconv_fwd_noalloc(*[ctypes.c_void_p(256)] * 6, 1, 4, 8, 64, 64, 1, None) == 2


def test_replays_inside_a_hip_graph():
    # what the entry point is for: captured once (after a first eager call resolved the scratch address), replayed
    # with eager work in between; every replay equals the eager result
    B, N, K, Din, Dout = 1, 2000, 8, 64, 64
    pos, nbr, feat, theta, bias, _ = random_problem(9, B, N, K, Din, Dout)
    a = [to_layout(feat, fx.BNC), dev(pos), dev(nbr), dev(theta), dev(bias)]
    out = torch.empty((B, N, Dout), device="cuda")
    fx.flexconv_fwd_noalloc(*a, out, layout=fx.BNC)
    want = out.clone()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fx.flexconv_fwd_noalloc(*a, out, layout=fx.BNC)
    torch.cuda.synchronize()
    for r in range(3):
        out.fill_(float("nan"))
        one_case(20 + r, 1, 300 + 50 * r, 8, 32, 64, fx.BNC)      # eager work that overwrites the scratch
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {r}"
