"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every
declared symbol, and rejects host-visible errors before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "flexconv.h")


@pytest.fixture(scope="module")
def L():
    import paper_1803_07289_amd as fx
    if not os.path.exists(fx.LIB_PATH):
        from paper_1803_07289_amd import build
        build.build()
    return fx.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flex[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert {"flexconv_fwd", "flexconv_bwd", "flexpool_fwd", "flexpool_bwd", "flex_inedges_build",
            "flexconv_workspace_bytes", "flex_validate_neighbors", "flex_status_string",
            "flexconv_has_fast_path", "flexupsample_fwd", "flexupsample_bwd", "flex_validate_selection",
            "flexconv_bwd_pos", "flexpool_sub_fwd", "flexpool_sub_bwd", "flex_inedges_build_sub",
            "flexconv_compose_1x1", "flexconv_compose_1x1_bwd", "flex_idiss_phi", "flex_idiss_sample", "flex_knn",
            "flex_selection_make_distinct", "flexpool_plan_bytes", "flexpool_plan_build",
            "flexpool_bwd_planned", "flexpool_fwd_plan_build", "flexpool_fwd_planned"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings(L):
    assert L.flex_status_string(0) == b"ok"
    for s in range(1, 6):
        assert len(L.flex_status_string(s)) > 0
    assert L.flex_status_string(99) == b"unknown status"


def test_null_and_shape_errors_precede_any_launch(L):
    one = ctypes.c_void_p(256)      # never dereferenced: validation fails first
    none = None
    # null pointers
    assert L.flexconv_fwd(none, one, one, one, one, one, 1, 8, 2, 4, 4, 0, one, 1 << 20, None) == 1
    assert L.flexpool_fwd(one, none, one, one, 1, 8, 2, 4, 0, None) == 1
    assert L.flexpool_bwd(one, one, none, none, none, 1, 8, 1, 4, 0, None) == 1
    assert L.flexpool_bwd(one, one, one, one, none, 1, 8, 1, 4, 0, None) == 1
    assert L.flexconv_bwd(one, one, one, one, one, none, one, one, one, none, none, 1, 8, 2, 4, 4, 0, one, 1 << 20, None) == 1
    # grad_theta without grad_bias, in_off without in_src
    assert L.flexconv_bwd(one, one, one, one, one, one, one, one, none, none, none, 1, 8, 2, 4, 4, 0, one, 1 << 20, None) == 1
    assert L.flexconv_bwd(one, one, one, one, one, one, one, one, one, one, none, 1, 8, 2, 4, 4, 0, one, 1 << 20, None) == 1
    # sizes: zero, K > N, bad layout, B*N too large
    assert L.flexconv_fwd(one, one, one, one, one, one, 0, 8, 2, 4, 4, 0, one, 1 << 20, None) == 2
    assert L.flexconv_fwd(one, one, one, one, one, one, 1, 8, 9, 4, 4, 0, one, 1 << 20, None) == 2
    assert L.flexconv_fwd(one, one, one, one, one, one, 1, 8, 2, 4, 4, 7, one, 1 << 20, None) == 2
    assert L.flexconv_fwd(one, one, one, one, one, one, 1 << 12, 1 << 20, 2, 4, 4, 0, one, 1 << 20, None) == 2
    assert L.flexpool_fwd(one, one, one, one, 1, 8, 2, 0, 0, None) == 2
    assert L.flexpool_bwd(one, one, one, none, none, 1, 8, 1, 4, 3, None) == 2
    # workspace: missing, misaligned, too small (tiled shape needs > 256 bytes)
    assert L.flexconv_fwd(one, one, one, one, one, one, 1, 64, 2, 64, 64, 1, none, 0, None) == 4
    assert L.flexconv_fwd(one, one, one, one, one, one, 1, 64, 2, 64, 64, 1, ctypes.c_void_p(260), 1 << 20, None) == 4
    assert L.flexconv_fwd(one, one, one, one, one, one, 1, 64, 2, 64, 64, 1, one, 512, None) == 4


def test_pooling_plan_size_and_errors_precede_any_launch(L):
    one, none = ctypes.c_void_p(256), None
    up = lambda x: (x + 255) // 256 * 256
    for B, N, K in ((1, 1, 1), (2, 33, 8), (1, 7_000_000, 8), (3, 4097, 16)):
        tiles = B * ((N + 31) // 32)
        # a header, distinct-row counts, 128 row places per tile of 32 points, one 16-bit place per list entry
        # ... and 2 KB of tile counters for the kernel
        assert L.flexpool_plan_bytes(B, N, K) == 256 + up(4 * tiles) + up(4 * tiles * 128) + up(2 * B * K * N) + 2048
    assert L.flexpool_plan_bytes(1, 8, 9) == 0 and L.flexpool_plan_bytes(0, 8, 1) == 0
    need = L.flexpool_plan_bytes(1, 64, 2)
    assert L.flexpool_plan_build(none, one, 1, 64, 2, one, need, None) == 1
    assert L.flexpool_plan_build(one, one, 1, 64, 2, none, need, None) == 1
    assert L.flexpool_plan_build(one, one, 1, 64, 65, one, need, None) == 2
    assert L.flexpool_plan_build(one, one, 1, 64, 2, one, need - 1, None) == 4
    assert L.flexpool_plan_build(one, one, 1, 64, 2, ctypes.c_void_p(260), need, None) == 4
    assert L.flexpool_bwd_planned(one, one, one, one, one, none, need, 1, 64, 2, 64, 1, None) == 1
    assert L.flexpool_bwd_planned(one, one, none, one, one, one, need, 1, 64, 2, 64, 1, None) == 1
    assert L.flexpool_bwd_planned(one, one, one, one, one, one, need, 1, 64, 2, 64, 5, None) == 2
    assert L.flexpool_bwd_planned(one, one, one, one, one, one, need, 1, 64, 2, 0, 1, None) == 2
    assert L.flexpool_bwd_planned(one, one, one, one, one, one, need - 1, 1, 64, 2, 64, 1, None) == 4
    assert L.flexpool_bwd_planned(one, one, one, one, one, ctypes.c_void_p(260), need, 1, 64, 2, 64, 1, None) == 4
    # flexpool_fwd_plan_build(nbr, B, N, K, plan, plan_bytes, stream)
    assert L.flexpool_fwd_plan_build(none, 1, 64, 2, one, need, None) == 1
    assert L.flexpool_fwd_plan_build(one, 1, 64, 2, none, need, None) == 1
    assert L.flexpool_fwd_plan_build(one, 1, 64, 65, one, need, None) == 2
    assert L.flexpool_fwd_plan_build(one, 1, 64, 2, one, need - 1, None) == 4
    assert L.flexpool_fwd_plan_build(one, 1, 64, 2, ctypes.c_void_p(260), need, None) == 4
    # flexpool_fwd_planned(feat, nbr, out, argmax, plan, plan_bytes, B, N, K, C, layout, stream)
    assert L.flexpool_fwd_planned(one, one, one, one, none, need, 1, 64, 2, 64, 1, None) == 1
    assert L.flexpool_fwd_planned(one, one, none, one, one, need, 1, 64, 2, 64, 1, None) == 1
    assert L.flexpool_fwd_planned(one, one, one, one, one, need, 1, 64, 2, 64, 5, None) == 2
    assert L.flexpool_fwd_planned(one, one, one, one, one, need, 1, 64, 2, 0, 1, None) == 2
    assert L.flexpool_fwd_planned(one, one, one, one, one, need - 1, 1, 64, 2, 64, 1, None) == 4
    assert L.flexpool_fwd_planned(one, one, one, one, ctypes.c_void_p(260), need, 1, 64, 2, 64, 1, None) == 4


def test_upsampling_and_location_gradient_errors_precede_any_launch(L):
    one, none = ctypes.c_void_p(256), None
    big = 1 << 30
    # flexupsample_fwd(feat_small, sel, nbr, out, argmax, B, Ns, Nf, K, C, layout, ws, ws_bytes, stream)
    assert L.flexupsample_fwd(one, none, one, one, one, 1, 4, 16, 2, 8, 0, one, big, None) == 1
    assert L.flexupsample_fwd(one, one, one, one, one, 1, 17, 16, 2, 8, 0, one, big, None) == 2    # Ns > Nf
    assert L.flexupsample_fwd(one, one, one, one, one, 1, 0, 16, 2, 8, 0, one, big, None) == 2
    assert L.flexupsample_fwd(one, one, one, one, one, 1, 4, 16, 2, 8, 2, one, big, None) == 2     # layout
    assert L.flexupsample_fwd(one, one, one, one, one, 1, 4, 16, 2, 8, 0, none, 0, None) == 4
    assert L.flexupsample_fwd(one, one, one, one, one, 1, 4, 1 << 20, 2, 8, 0, one, 1024, None) == 4
    # flexupsample_bwd(grad_out, argmax, sel, in_off, in_src, grad_small, B, Ns, Nf, K, C, layout, stream)
    assert L.flexupsample_bwd(one, one, one, none, one, one, 1, 4, 16, 2, 8, 0, None) == 1          # lists are required
    assert L.flexupsample_bwd(one, one, one, one, one, one, 1, 4, 16, 2, 0, 0, None) == 2
    # flexconv_compose_1x1(W, theta, bias, theta_c, bias_c, Din0, Dmid, Dout, stream)
    assert L.flexconv_compose_1x1(one, one, none, one, one, 8, 8, 8, None) == 1
    assert L.flexconv_compose_1x1(one, one, one, one, one, 0, 8, 8, None) == 2
    assert L.flexconv_compose_1x1_bwd(one, one, one, one, one, one, one, none, 8, 8, 8, None) == 1
    assert L.flexconv_compose_1x1_bwd(one, one, one, one, one, one, one, one, 8, 1 << 20, 8, None) == 2
    # flex_idiss_phi(pos, nbr, phi, B, N, K, stream); flex_idiss_sample(phi, u, sel, B, N, Ns, ws, ws_bytes, stream)
    assert L.flex_idiss_phi(one, none, one, 1, 16, 4, None) == 1
    assert L.flex_idiss_phi(one, one, one, 1, 16, 17, None) == 2
    assert L.flex_idiss_sample(one, one, none, 1, 16, 4, one, big, None) == 1
    assert L.flex_idiss_sample(one, one, one, 1, 16, 17, one, big, None) == 2
    assert L.flex_idiss_sample(one, one, one, 1, (1 << 25) + 1, 4, one, big, None) == 2
    assert L.flex_idiss_sample(one, one, one, 1, 4096, 4, one, 1024, None) == 4
    assert L.flexconv_workspace_bytes(7, 1, 4096, 1, 1, 1, 0) == 8 * 4096 + 256 + 256
    # flex_selection_make_distinct(sel, B, N, Ns, ws, ws_bytes, stream)
    assert L.flex_selection_make_distinct(none, 1, 16, 4, one, big, None) == 1
    assert L.flex_selection_make_distinct(one, 1, 16, 17, one, big, None) == 2
    assert L.flex_selection_make_distinct(one, 1, 16, 4, none, 0, None) == 4
    # flex_knn(pos, nbr, B, N, K, ws, ws_bytes, stream)
    assert L.flex_knn(one, none, 1, 100, 8, one, big, None) == 1
    assert L.flex_knn(one, one, 1, 100, 11, one, big, None) == 2           # K without a kernel
    assert L.flex_knn(one, one, 1, 4, 8, one, big, None) == 2              # K > N
    assert L.flex_knn(one, one, 1, 100, 8, one, 64, None) == 4
    assert L.flexconv_workspace_bytes(8, 1, 100, 8, 1, 1, 0) > 100 * 16
    assert L.flexconv_workspace_bytes(8, 1, 100, 11, 1, 1, 0) == 0
    # flexpool_sub_fwd(feat, nbr, sel, out, argmax, B, N, Ns, K, C, layout, stream)
    assert L.flexpool_sub_fwd(one, one, none, one, one, 1, 16, 4, 2, 8, 0, None) == 1
    assert L.flexpool_sub_fwd(one, one, one, one, one, 1, 16, 17, 2, 8, 0, None) == 2               # Ns > N
    assert L.flexpool_sub_fwd(one, one, one, one, one, 1, 16, 4, 2, 8, 5, None) == 2                # layout
    # flexpool_sub_bwd(grad_out, argmax, in_off, in_src, grad_feat, B, N, Ns, K, C, layout, stream)
    assert L.flexpool_sub_bwd(one, one, one, none, one, 1, 16, 4, 2, 8, 0, None) == 1               # in_off without in_src
    assert L.flexpool_sub_bwd(one, one, none, none, none, 1, 16, 4, 2, 8, 0, None) == 1
    assert L.flexpool_sub_bwd(one, one, none, none, one, 1, 16, 0, 2, 8, 0, None) == 2
    # flex_inedges_build_sub(nbr, sel, B, N, Ns, K, in_off, in_src, ws, ws_bytes, stream)
    assert L.flex_inedges_build_sub(one, none, 1, 16, 4, 2, one, one, one, big, None) == 1
    assert L.flex_inedges_build_sub(one, one, 1, 16, 17, 2, one, one, one, big, None) == 2
    assert L.flex_inedges_build_sub(one, one, 1, 16, 4, 2, one, one, one, 16, None) == 4
    # flex_validate_selection(sel, B, Ns, Nf, bad, ws, ws_bytes, stream)
    assert L.flex_validate_selection(one, 1, 4, 16, none, one, big, None) == 1
    assert L.flex_validate_selection(one, 1, 4, 16, one, one, 16, None) == 4
    # flexconv_bwd_pos(feat, nbr, theta, grad_out, in_off, in_src, grad_pos, B, N, K, Din, Dout, layout, ws, ws_bytes, stream)
    assert L.flexconv_bwd_pos(one, one, none, one, none, none, one, 1, 8, 2, 4, 4, 0, one, big, None) == 1
    assert L.flexconv_bwd_pos(one, one, one, one, one, none, one, 1, 8, 2, 4, 4, 0, one, big, None) == 1   # in_off without in_src
    assert L.flexconv_bwd_pos(one, one, one, one, none, none, one, 1, 8, 9, 4, 4, 0, one, big, None) == 2  # K > N
    assert L.flexconv_bwd_pos(one, one, one, one, none, none, one, 1, 64, 8, 64, 64, 1, one, 256, None) == 4
    w = L.flexconv_workspace_bytes
    assert w(4, 2, 1000, 1, 1, 1, 0) == 8192                   # inverse map: 4 bytes per larger-layer point, 256-aligned
    assert w(6, 1, 4096, 8, 64, 64, 1) > w(5, 1, 4096, 8, 64, 64, 1) > 256    # lists built inside the call cost workspace
    # other widths: packed 64 x 64 parameter block (both orientations, 6 f16 planes + exponent slot each), its fp32
    # source, and one zero-padded 64-channel column block of each tensor
    assert w(5, 1, 4096, 8, 5, 7, 1) == 2 * (6 * 64 * 64 * 2 + 256) + 3 * 64 * 64 * 4 + 2 * 4096 * 64 * 4


def test_workspace_sizes(L):
    w = L.flexconv_workspace_bytes
    # parameters (fp32 form = both f16 halves) + 64 column exponents + 256 depth scales
    packed = 4 * 64 * 64 * 4 + 64 * 4 + 256 * 4
    assert w(0, 1, 4096, 8, 64, 64, 1) == packed                                 # packed parameters only
    assert w(0, 1, 4096, 8, 64, 64, 0) == packed + 4096 * 64 * 4                 # + transposed features
    # widths without a kernel of their own: padded copies of the features, the parameters and the output + the 9 -> 64 plan
    assert w(0, 1, 4096, 8, 5, 7, 0) == 4096 * 9 * 4 + 4 * 9 * 64 * 4 + 4096 * 64 * 4 + w(0, 1, 4096, 8, 9, 64, 1)
    assert w(2, 1, 4096, 8, 64, 64, 1) > w(1, 1, 4096, 8, 64, 64, 1) > 0
    assert w(0, 0, 4096, 8, 64, 64, 1) == 0 and w(9, 1, 4096, 8, 64, 64, 1) == 0
    assert w(0, 1, 4096, 8, 64, 64, 5) == 0
    assert L.flexconv_has_fast_path(64, 64) == 1 and L.flexconv_has_fast_path(256, 512) == 1
    assert L.flexconv_has_fast_path(5, 7) == 2 and L.flexconv_has_fast_path(200, 300) == 2


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_1803_07289_amd as fx
    t = torch.zeros(1, 4, 8)
    with pytest.raises(TypeError):
        fx.flexpool_fwd(t, torch.zeros(1, 2, 8, dtype=torch.int32))


# ---- the route a call takes and the workspace it is planned for (host queries, child processes per switch) ----
def _query(env_extra, calls):
    """Run flexconv_kernel_route / flexconv_workspace_bytes in a fresh interpreter with extra environment
    (the switches are read once per process).  calls: list of (fn, args); returns the list of results."""
    import json
    import subprocess
    import sys
    code = (
        "import json, sys; sys.path.insert(0, %r)\n"
        "import paper_1803_07289_amd as fx\n"
        "L = fx.lib()\n"
        "calls = json.loads(%r)\n"
        "print(json.dumps([int(getattr(L, f)(*a)) for f, a in calls]))\n" % (ROOT, json.dumps(calls)))
    env = dict(os.environ)
    env.update(env_extra)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, check=True)
    return json.loads(r.stdout.strip().splitlines()[-1])


ROUTE_SINGLE, ROUTE_STAGED, ROUTE_LEAN, ROUTE_SPLIT128, ROUTE_WIDE, ROUTE_PADDED, ROUTE_LEAN_FUSED = 1, 2, 3, 4, 5, 6, 7


def _align256(x):
    return (x + 255) // 256 * 256


@pytest.mark.parametrize("env", [{}, {"FLEX_CONTRACT": "f32"}, {"FLEX_PRODUCER": "staged"}, {"FLEX_SPLIT": "0"}])
def test_channel_major_128_backward_is_planned_for_the_route_it_takes(L, env):
    # The channel-major 128 -> 128 backward pass runs as block passes only where those kernels apply; anywhere
    # else it is the single-pass tiled path on transposed copies, and the workspace must hold THAT path's
    # per-workgroup partial sums (256 workgroups x [4*128 x 128] floats), not the block passes' smaller ones.
    N, K = 1_000_000, 8
    tiled_partials = 256 * 4 * 128 * 128 * 4
    transposed = 2 * _align256(N * 128 * 4)
    r_bcn, r_bnc, w_bcn, w_bnc, w_small = _query(env, [
        ("flexconv_kernel_route", [1, 1, N, K, 128, 128, 0]),
        ("flexconv_kernel_route", [1, 1, N, K, 128, 128, 1]),
        ("flexconv_workspace_bytes", [1, 1, N, K, 128, 128, 0]),
        ("flexconv_workspace_bytes", [1, 1, N, K, 128, 128, 1]),
        ("flexconv_workspace_bytes", [1, 1, 300, 16, 128, 128, 0]),
    ])
    if not env:
        assert r_bcn == ROUTE_WIDE and r_bnc == ROUTE_SPLIT128
    else:
        assert r_bcn != ROUTE_WIDE and r_bnc != ROUTE_SPLIT128
        # same single-pass plan in both layouts, plus the two transposed copies
        assert w_bcn == w_bnc + transposed
        assert w_bcn >= tiled_partials + transposed
        # the small parity shape (300 points, 19 tiles of 16): one partial per tile-owning workgroup
        assert w_small >= 16 * 4 * 128 * 128 * 4


def test_block_passes_stop_where_byte_offsets_leave_32_bits(L):
    # N * 128 * 4 = 2^32 at N = 8 388 608 points per cloud: the block passes (32-bit byte offsets inside a cloud)
    # hand over to the single-pass kernels, and the plan follows.
    K = 8
    below, at = 8_388_607, 8_388_608
    r = _query({}, [("flexconv_kernel_route", [op, 1, n, K, 128, 128, lay])
                    for op in (0, 1) for n in (below, at) for lay in (0, 1)])
    assert r == [ROUTE_WIDE, ROUTE_SPLIT128, ROUTE_SINGLE, ROUTE_SINGLE,
                 ROUTE_WIDE, ROUTE_SPLIT128, ROUTE_SINGLE, ROUTE_SINGLE]
    w_at_bcn, w_at_bnc = _query({}, [("flexconv_workspace_bytes", [1, 1, at, K, 128, 128, 0]),
                                     ("flexconv_workspace_bytes", [1, 1, at, K, 128, 128, 1])])
    assert w_at_bcn == w_at_bnc + 2 * _align256(at * 128 * 4)
    assert w_at_bnc >= 256 * 4 * 128 * 128 * 4


def test_one_pass_backward_is_planned_only_where_it_runs():
    # plan and route agree, the switch restores the two separate kernels, the plan holds the flag's 256 bytes
    N, K = 100_000, 8
    q = [("flexconv_kernel_route", [1, 1, N, K, 64, 64, 1]), ("flexconv_workspace_bytes", [1, 1, N, K, 64, 64, 1]),
         ("flexconv_kernel_route", [1, 1, N, K, 64, 64, 0]), ("flexconv_kernel_route", [1, 1, N, K, 32, 32, 1]),
         ("flexconv_kernel_route", [1, 1, N, 12, 64, 64, 1])]
    r_on, w_on, r_bcn, r32, r_k12 = _query({}, q)
    r_off, w_off, _, _, _ = _query({"FLEX_FUSED_BWD": "0"}, q)
    assert r_on == ROUTE_LEAN_FUSED and r_bcn == ROUTE_LEAN_FUSED and r_k12 == ROUTE_LEAN_FUSED and r32 == ROUTE_LEAN
    assert r_off == ROUTE_LEAN and w_on == w_off + 4 * (64 + 128 * 1024)      # flag block + 1024 workgroup records
    for env in ({"FLEX_CONTRACT": "f32"}, {"FLEX_PRODUCER": "staged"}):
        assert _query(env, q[:1])[0] != ROUTE_LEAN_FUSED


def test_lean_kernels_stop_where_byte_offsets_leave_32_bits(L):
    # the lean producers address rows with 32-bit byte offsets from a per-cloud base: N * width * 4 < 2^32
    route = L.flexconv_kernel_route
    lim64, lim32 = (1 << 32) // (64 * 4), (1 << 32) // (32 * 4)
    for op in (0, 1):
        lean64 = ROUTE_LEAN_FUSED if op == 1 else ROUTE_LEAN    # 64 -> 64 backward: one pass for all gradients
        assert route(op, 1, lim64 - 1, 8, 64, 64, 1) == lean64
        assert route(op, 1, lim64, 8, 64, 64, 1) == ROUTE_STAGED
        assert route(op, 1, lim32 - 1, 8, 32, 32, 1) == ROUTE_LEAN
        assert route(op, 1, lim32, 8, 32, 32, 1) == ROUTE_STAGED
        assert route(op, 4, lim64 - 1, 8, 64, 64, 1) == lean64              # the limit is per cloud, not per batch
    # the gathered width decides: forward gathers Din-wide rows, the feature gradient Dout-wide ones
    assert route(0, 1, lim64, 8, 32, 64, 1) == ROUTE_LEAN and route(1, 1, lim64, 8, 32, 64, 1) == ROUTE_STAGED
    assert route(0, 1, lim64, 8, 64, 32, 1) == ROUTE_STAGED and route(1, 1, lim64, 8, 64, 32, 1) == ROUTE_LEAN
    # K too large for the staged producers' 64 entries per wave and no lean kernel: single-role kernels
    assert route(0, 1, lim64, 24, 64, 64, 1) == ROUTE_SINGLE
    assert route(0, 1, 4096, 8, 5, 7, 1) == ROUTE_PADDED and route(0, 1, 4096, 8, 256, 512, 1) == ROUTE_WIDE
    assert route(0, 0, 4096, 8, 64, 64, 1) == -1 and route(3, 1, 4096, 8, 64, 64, 1) == -1
