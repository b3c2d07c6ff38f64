#!/usr/bin/env python3
"""Benchmark of the flex-convolution hot path on one MI355X.

One step = flexconv_fwd + flexconv_bwd + flexpool_fwd + flexpool_bwd over the
7M-point hall workload (config 4: B=1, N=7,000,000, K=8, Din=Dout=64, fp32),
inputs resident in HBM, neighbourhoods (and their transposed lists) static.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--n N] [--layout bnc|bcn]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense f16 / bf16 matrix
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "flexconv_cfg4_hbm_traffic.md")
DTYPE = "f32 (HBM tensors and accumulation fp32; contractions as split f16 / three-piece bf16 matrix ops)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash():
    """sha256 over the HIP sources of the library: ties a counter measurement to the kernels it was taken on."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_1803_07289_amd", "csrc")
    for name in sorted(os.listdir(src)):
        h.update(name.encode())
        h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()


def measured_traffic():
    """HBM bytes per launch of each entry point's kernel on the default workload, as measured with
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and recorded in the profile summary together with the hash of the
    kernel sources it was measured on.  ({}, why) when there is no record or the sources have changed since."""
    try:
        text = open(TRAFFIC_PROFILE).read()
        rec = json.loads(text.split("traffic-json:", 1)[1].splitlines()[0])
    except (OSError, IndexError, ValueError):
        return {}, "no machine-readable record in profiles/flexconv_cfg4_hbm_traffic.md"
    if rec.get("kernel_source_sha256") != kernel_source_hash():
        return {}, "kernel sources changed since the counters were read (profiles/flexconv_cfg4_hbm_traffic.md)"
    return {k: float(v) for k, v in rec["traffic_bytes"].items()}, "profiles/flexconv_cfg4_hbm_traffic.md"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--n", type=int, default=None, help="override N (smaller trial runs)")
    ap.add_argument("--k", type=int, default=None, help="override K (neighbourhood-size sweeps)")
    ap.add_argument("--din", type=int, default=None, help="override the input feature length (deeper-stage shapes)")
    ap.add_argument("--dout", type=int, default=None, help="override the output feature length")
    ap.add_argument("--layout", default="bnc", choices=["bnc", "bcn"])
    ap.add_argument("--order", default="morton", choices=["morton", "generator", "shuffled"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default=None,
                    help="comma list of ops to run (fwd,bwd,pool_fwd,pool_bwd; bwd_params / bwd_feat = flexconv_bwd asked "
                         "for the parameter gradients / the feature gradient alone; upsample = flex-upsampling from a "
                         "quarter of the points, bwd_pos = location gradient, pool_sub = pooling with subsampling to a "
                         "quarter of the points, idiss = importance sub-sampling of a quarter of the points, knn = the "
                         "neighbour search, pool_bwd_list = flexpool_bwd over the in-edge lists alone, pool_fwd_plain = flexpool_fwd "
                         "without its gather plan; none of them is part "
                         "of the default step)")
    ap.add_argument("--no-pool-plan", action="store_true",
                    help="flexpool_fwd and flexpool_bwd without their static gather plans (neighbour lists / in-edge "
                         "lists alone)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step into a HIP graph and time its replays (graph_ms_per_step)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain device copies of the feature tensor (known size) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run can be scaled against them")
    ap.add_argument("--no-calibrate", action="store_true",
                    help="skip the two microbenchmarks (plain copy, pure f16 matrix-op loop) whose results give "
                         "every roofline entry its fraction of the MEASURED peak beside the published one")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no multi-GPU path exists); use --gpus 1")

    import numpy as np
    import torch
    import paper_1803_07289_amd as fx
    from workloads import CONFIGS, make_inputs

    fx.lib()   # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    layout = fx.BNC if args.layout == "bnc" else fx.BCN
    ops = set((args.only or "fwd,bwd,pool_fwd,pool_bwd").split(","))

    cfg = CONFIGS[args.config]
    if args.k is not None:
        cfg = type(cfg)(**{**cfg.__dict__, "K": int(args.k), "name": cfg.name + f"_K{args.k}"})
    if args.din is not None or args.dout is not None:
        di, do = int(args.din or cfg.Din), int(args.dout or cfg.Dout)
        cfg = type(cfg)(**{**cfg.__dict__, "Din": di, "Dout": do, "name": cfg.name + f"_{di}x{do}"})
    t0 = time.time()
    x = make_inputs(cfg, order=args.order, n_override=args.n)
    cfg = x.cfg
    B, N, K, Din, Dout = cfg.B, cfg.N, cfg.K, cfg.Din, cfg.Dout
    log(f"[bench] inputs for {cfg.name} (N={N}) drawn in {time.time() - t0:.1f}s")

    def dev(a, transpose=False):
        t = torch.from_numpy(a).cuda()
        if transpose and layout == fx.BNC:
            t = t.transpose(1, 2).contiguous()
        return t

    feat, g = dev(x.feat, True), dev(x.grad_out, True)
    pos, nbr, theta, bias = dev(x.pos), dev(x.nbr), dev(x.theta), dev(x.bias)
    if Din != Dout:
        gpool = torch.randn(feat.shape, device="cuda", generator=torch.Generator("cuda").manual_seed(cfg.seed))
    else:
        gpool = g
    torch.cuda.synchronize()

    # static preprocessing of the neighbourhoods: transposed lists, built once
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    in_edges = fx.flex_inedges_build(nbr)
    torch.cuda.synchronize()
    ev0.record()
    in_edges = fx.flex_inedges_build(nbr)
    ev1.record()
    torch.cuda.synchronize()
    inedges_ms = ev0.elapsed_time(ev1)
    # and the gather plan of the pooling backward pass (which rows a tile of 32 points needs): also once per cloud
    pool_plan, pool_plan_ms = None, None
    if "pool_bwd" in ops and not args.no_pool_plan:
        pool_plan = fx.flexpool_plan_build(in_edges, B, N)
        torch.cuda.synchronize()
        ev0.record()
        pool_plan = fx.flexpool_plan_build(in_edges, B, N)
        ev1.record()
        torch.cuda.synchronize()
        pool_plan_ms = ev0.elapsed_time(ev1)
    # ... and of the pooling forward pass (the same over the neighbour lists themselves)
    pool_fwd_plan, pool_fwd_plan_ms = None, None
    if ("pool_fwd" in ops or "pool_bwd" in ops) and not args.no_pool_plan:
        pool_fwd_plan = fx.flexpool_fwd_plan_build(nbr)
        torch.cuda.synchronize()
        ev0.record()
        pool_fwd_plan = fx.flexpool_fwd_plan_build(nbr)
        ev1.record()
        torch.cuda.synchronize()
        pool_fwd_plan_ms = ev0.elapsed_time(ev1)

    names = [n for n in ("fwd", "bwd", "pool_fwd", "pool_bwd", "upsample", "bwd_pos", "pool_sub") if n in ops]
    state = {}
    OPS = ("fwd", "bwd", "pool_fwd", "pool_bwd", "upsample_fwd", "upsample_bwd", "bwd_pos",
           "pool_sub_fwd", "pool_sub_bwd", "idiss_phi", "idiss_sample", "knn", "bwd_params", "bwd_feat",
           "pool_bwd_list", "pool_fwd_plain")
    if "idiss" in ops:
        # random words for the stratified draw of a quarter of the points (Sec. 3.2), drawn once
        u_words = torch.from_numpy(np.random.default_rng([cfg.seed, 400]).integers(
            0, 2 ** 32, size=(B, max(1, N // 4)), dtype=np.uint64).astype(np.uint32).view(np.int32)).cuda()
    if "upsample" in ops or "pool_sub" in ops:
        # the smaller layer: a seeded quarter of the points (a decoder stage raises the resolution 4x)
        Ns = max(1, N // 4)
        sel_np = np.stack([np.sort(np.random.default_rng([cfg.seed, 300 + b]).permutation(N)[:Ns]) for b in range(B)])
        sel = torch.from_numpy(sel_np.astype(np.int32)).cuda()
        idx = sel.long()[:, :, None].expand(B, Ns, Din) if layout == fx.BNC else sel.long()[:, None, :].expand(B, Din, Ns)
        feat_small = torch.gather(feat, 1 if layout == fx.BNC else 2, idx).contiguous()
        g_small = torch.gather(gpool, 1 if layout == fx.BNC else 2, idx).contiguous()
        sub_edges = fx.flex_inedges_build_sub(nbr, sel) if "pool_sub" in ops else None

    def step(events=None):
        """One pass of the hot path: flexconv_fwd, flexconv_bwd (all three gradients, one call), flexpool_fwd,
        flexpool_bwd; then whatever --only added."""
        slot = [0]

        def mark():
            if events is not None:
                events[slot[0]].record()
            slot[0] += 1
        mark()
        if "fwd" in ops:
            state["out"] = fx.flexconv_fwd(feat, pos, nbr, theta, bias, layout=layout, out=state.get("out"))
        mark()
        if "bwd" in ops:
            state["grads"] = fx.flexconv_bwd(feat, pos, nbr, theta, bias, g, layout=layout, in_edges=in_edges)
        mark()
        if "pool_fwd" in ops or "pool_bwd" in ops or "pool_bwd_list" in ops:
            if pool_fwd_plan is not None:
                state["pool"] = fx.flexpool_fwd_planned(feat, nbr, pool_fwd_plan, layout=layout)
            else:
                state["pool"] = fx.flexpool_fwd(feat, nbr, layout=layout)
        mark()
        if "pool_bwd" in ops:
            if pool_plan is not None:
                state["pool_grad"] = fx.flexpool_bwd_planned(gpool, state["pool"][1], in_edges, pool_plan, layout=layout)
            else:
                state["pool_grad"] = fx.flexpool_bwd(gpool, state["pool"][1], layout=layout, in_edges=in_edges)
        mark()
        if "upsample" in ops:
            state["up"] = fx.flexupsample_fwd(feat_small, sel, nbr, layout=layout)
        mark()
        if "upsample" in ops:
            state["up_grad"] = fx.flexupsample_bwd(gpool, state["up"][1], sel, in_edges, layout=layout)
        mark()
        if "bwd_pos" in ops:
            state["grad_pos"] = fx.flexconv_bwd_pos(feat, nbr, theta, g, layout=layout, in_edges=in_edges)
        mark()
        if "pool_sub" in ops:
            state["pool_sub"] = fx.flexpool_sub_fwd(feat, nbr, sel, layout=layout)
        mark()
        if "pool_sub" in ops:
            state["pool_sub_grad"] = fx.flexpool_sub_bwd(g_small, state["pool_sub"][1], N, layout=layout,
                                                         in_edges=sub_edges)
        mark()
        if "idiss" in ops:
            state["phi"] = fx.flex_idiss_phi(pos, nbr)
        mark()
        if "idiss" in ops:
            state["sel"] = fx.flex_selection_make_distinct(fx.flex_idiss_sample(state["phi"], u_words), N)
        mark()
        if "knn" in ops:
            state["knn"] = fx.flex_knn(pos, K)
        mark()
        # the two halves of flexconv_bwd as calls of their own (each runs its stand-alone kernel)
        if "bwd_params" in ops:
            state["gp"] = fx.flexconv_bwd(feat, pos, nbr, theta, bias, g, layout=layout, in_edges=in_edges,
                                          need_feat=False)
        mark()
        if "bwd_feat" in ops:
            state["gfeat"] = fx.flexconv_bwd(feat, pos, nbr, theta, bias, g, layout=layout, in_edges=in_edges,
                                             need_params=False)
        mark()
        # the pooling backward pass over the lists alone, beside the planned form of the step
        if "pool_bwd_list" in ops:
            state["pool_grad_list"] = fx.flexpool_bwd(gpool, state["pool"][1], layout=layout, in_edges=in_edges)
        mark()
        if "pool_fwd_plain" in ops:
            state["pool_plain"] = fx.flexpool_fwd(feat, nbr, layout=layout)
        mark()

    # ---- measured peaks of this device: plain copy kernel, pure f16 matrix-op loop ----------
    measured_peaks = None
    if not args.no_calibrate:
        src_buf = feat if feat.numel() * 4 >= (1 << 28) else torch.empty(1 << 26, device="cuda")   # >= 256 MB
        dst_buf = torch.empty_like(src_buf)
        sink = torch.zeros(1, device="cuda")
        nbytes = src_buf.numel() * 4
        best_copy = best_mfma = 0.0
        for it in range(6):
            c0, c1, c2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            c0.record()
            fx.flex_calibrate_copy(src_buf, dst_buf)
            c1.record()
            flop = fx.flex_calibrate_mfma_f16(20000, sink)
            c2.record()
            torch.cuda.synchronize()
            if it > 0:         # the first round warms up
                best_copy = max(best_copy, 2 * nbytes / (c0.elapsed_time(c1) * 1e-3) / 1e9)
                best_mfma = max(best_mfma, flop / (c1.elapsed_time(c2) * 1e-3) / 1e12)
        measured_peaks = {"copy_GBs": best_copy, "copy_bytes_each_way": nbytes, "mfma_f16_TFLOPs": best_mfma,
                          "how": "flex_calibrate_copy (bytes read + written / time) and flex_calibrate_mfma_f16 "
                                 "(16 waves per CU, 4 chains of v_mfma_f32_16x16x32_f16), best of 5"}
        del dst_buf, sink
        log(f"[bench] measured peaks: copy {best_copy:.0f} GB/s, f16 matrix ops {best_mfma:.0f} TFLOP/s")

    if args.calibrate_copy:
        scratch = torch.empty_like(feat)
        for _ in range(3):
            scratch.copy_(feat)          # reads and writes feat.numel()*4 bytes, contiguous
        torch.cuda.synchronize()
        del scratch

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    per_step_events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(OPS) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(per_step_events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps

    op_ms = {}
    for j, name in enumerate(OPS):
        ts = [ev[j].elapsed_time(ev[j + 1]) for ev in per_step_events]
        op_ms[name] = {"mean": float(np.mean(ts)), "min": float(np.min(ts)), "median": float(np.median(ts))}
    pts = B * N

    # ---- rooflines (algorithmic figures: every array touched once) ----------
    # Every kernel of the path is bound by HBM: the contractions run on the f16 / bf16 matrix cores in
    # split form (3 resp. 6 matrix ops per fp32-equivalent product), whose time at the published dense
    # peak (2.5 PFLOP/s) stays below the time the touched-once bytes need at 8 TB/s.
    conv_flop_pt = 8 * K * Din + 2 * 4 * Din * Dout          # factored form, fp32-equivalent
    route_bwd = fx.kernel_route(fx.OP_CONV_BWD, B, N, K, Din, Dout, layout)
    fused_bwd = route_bwd == 7          # FLEX_ROUTE_LEAN_FUSED: one pass over the in-edge lists for all gradients
    issued_matrix_flop_pt = {"fwd": 3 * 2 * 4 * Din * Dout, "bwd_params": 6 * 2 * 4 * Din * Dout,
                             "bwd_feat": 3 * 2 * 4 * Din * Dout,
                             "bwd": (3 + 3 if fused_bwd else 6 + 3) * 2 * 4 * Din * Dout}
    fp32_flop_pt = {"fwd": conv_flop_pt, "bwd_params": conv_flop_pt, "bwd_feat": conv_flop_pt,
                    # one aggregate and two contractions when fused, else two of each
                    "bwd": (8 * K * Dout + 2 * 2 * 4 * Din * Dout) if fused_bwd else 2 * conv_flop_pt}
    bytes_pt = {"fwd": 4 * Din + 12 + 4 * K + 4 * Dout,
                # every array of the call touched once: features, upstream gradient, feature gradient, positions,
                # in-edge lists (fused: the neighbour tensor is not read; separate kernels: it is, + 4 K)
                "bwd": 4 * Din + 4 * Dout + 4 * Din + 12 + 4 * (K + 1) + (0 if fused_bwd else 4 * K),
                "bwd_params": 4 * Din + 12 + 4 * K + 4 * Dout,
                "bwd_feat": 4 * Dout + 12 + 4 * (K + 1) + 4 * Din,
                "pool_fwd": 4 * Din + 4 * K + 8 * Din,
                "pool_bwd": 8 * Din + 4 * (K + 1) + 4 * Din,
                "pool_bwd_list": 8 * Din + 4 * (K + 1) + 4 * Din,
                "pool_fwd_plain": 4 * Din + 4 * K + 8 * Din,
                # per point of the larger layer, smaller layer = a quarter of it: rows of the smaller layer,
                # sel, inverse map (written, read), ids, out + winners / gradient + winners, lists, smaller rows
                "upsample_fwd": Din + 1 + 8 + 4 * K + 8 * Din,
                "upsample_bwd": 8 * Din + 1 + 4 * (K + 1) + Din,
                # two passes: each reads features and upstream gradient once, ids / lists, writes 3 floats
                "bwd_pos": 2 * (4 * Din + 4 * Dout) + 4 * K + 4 * (K + 1) + 12 + 24,
                # per point before subsampling, a quarter kept: the features once (every row is somebody's
                # neighbour), ids of the kept centres, sel, out + winners of the kept / their gradient +
                # winners, lists over the kept centres, the full-size gradient written
                "pool_sub_fwd": 4 * Din + K + 1 + 2 * Din,
                "pool_sub_bwd": 2 * Din + (K + 4) + 4 * Din}
    kernel_of = {"fwd": "gather_contract_lean_kernel (flexconv_fwd)",
                 "bwd": ("bwd_fused_lean_kernel (flexconv_bwd: feature and parameter gradients in one pass)" if fused_bwd
                         else "grad_theta kernel + grad_feat kernel (flexconv_bwd)"),
                 "bwd_params": "grad_theta_lean_kernel (flexconv_bwd, parameter gradients)",
                 "bwd_feat": "grad_feat_lean_kernel (flexconv_bwd, feature gradient)",
                 "pool_fwd": ("pool_fwd_planned64_kernel (flexpool_fwd_planned)"
                              if pool_fwd_plan is not None and layout == fx.BNC and Din in (64, 128, 256) and K <= 10 and B * N >= (1 << 18)
                              else "pool_fwd_bnc4_kernel (flexpool_fwd)"),
                 "pool_fwd_plain": "pool_fwd_bnc4_kernel (flexpool_fwd)",
                 "pool_bwd": ("pool_bwd_planned64_kernel (flexpool_bwd_planned)"
                              if pool_plan is not None and layout == fx.BNC and Din in (64, 128, 256) and K <= 10 and B * N >= (1 << 18)
                              else "pool_bwd_gather_row16_kernel (flexpool_bwd)"),
                 "upsample_fwd": "upsample_fwd_bnc4_kernel (flexupsample_fwd)",
                 "upsample_bwd": "upsample_bwd_bnc4_kernel (flexupsample_bwd)",
                 "bwd_pos": "grad_pos_kernel x2 (flexconv_bwd_pos: centre term, neighbour term)",
                 "pool_sub_fwd": "pool_fwd_bnc4_kernel<true> (flexpool_sub_fwd)",
                 "pool_bwd_list": "pool_bwd_gather_row16_kernel (flexpool_bwd)",
                 "pool_sub_bwd": "pool_bwd_gather_row16_kernel<2> (flexpool_sub_bwd)"}
    # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy
    # (profiles/flexconv_cfg4_hbm_traffic.md); only known for the default workload
    traffic_rec, traffic_src = measured_traffic()
    default_workload = (cfg.index == 4 and N == 7_000_000 and K == 8 and layout == fx.BNC and x.order == "morton")

    def roof(name):
        ms = op_ms[name]["mean"]
        if ms <= 0:
            return None
        traffic = traffic_rec.get(name) if default_workload else None
        gbs = bytes_pt[name] * pts / (ms * 1e-3) / 1e9
        r = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
             "traffic": traffic, "traffic_source": traffic_src if default_workload else "not the default workload",
             "kernel": kernel_of[name], "kernel_ms": ms}
        if measured_peaks:
            r["frac_of_measured_peak"] = gbs / measured_peaks["copy_GBs"]
        if name in issued_matrix_flop_pt:
            r["fp32_equivalent_TFLOPs"] = fp32_flop_pt[name] * pts / (ms * 1e-3) / 1e12
            r["issued_matrix_TFLOPs"] = issued_matrix_flop_pt[name] * pts / (ms * 1e-3) / 1e12
            r["issued_matrix_frac_of_f16_peak"] = r["issued_matrix_TFLOPs"] / MFMA_F16_PEAK_TFLOPS
            if measured_peaks:
                r["issued_matrix_frac_of_measured_f16_peak"] = r["issued_matrix_TFLOPs"] / measured_peaks["mfma_f16_TFLOPs"]
        return r

    rooflines = {n: roof(n) for n in OPS if n in ops and n in bytes_pt and op_ms[n]["mean"] > 1e-2}
    dominant = max(rooflines, key=lambda n: rooflines[n]["kernel_ms"]) if rooflines else None
    roofline = rooflines.get(dominant)
    fwd_ms = op_ms["fwd"]["mean"] if "fwd" in ops else 0.0
    bwd_ms = op_ms["bwd"]["mean"] if "bwd" in ops else 0.0

    # ---- sampled parity at this size, in this launch configuration -------------
    parity = None
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.default_rng(0)
        starts = sorted({0, max(0, N - 300), *(int(s) for s in rng.integers(0, max(1, N - 300), size=2))})
        if "fwd" in ops:
            out = state["out"]
            worst = 0.0
            for s0 in starts:
                s1 = min(N, s0 + 300)
                ref = oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias, l_range=(s0, s1))
                got = (out[:, s0:s1, :].transpose(1, 2) if layout == fx.BNC else out[:, :, s0:s1]).cpu().numpy()
                den = np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)))
                worst = max(worst, float(np.max(np.abs(got - ref) / den)))
            parity = {"fwd_sampled_max_rel_err": worst, "points": 300 * len(starts)}
        if "bwd" in ops and "grads" in state and hasattr(oracle, "flexconv_grad_feat_at"):
            # feature-gradient rows of the timed call at sampled points (the oracle evaluates single rows)
            targets = np.unique(rng.integers(0, B * N, size=2000)).astype(np.int64)
            ref = oracle.flexconv_grad_feat_at(x.pos, x.nbr, x.theta, x.bias, x.grad_out, targets)
            gfeat = state["grads"][0]
            rows_g = (gfeat.reshape(B * N, Din) if layout == fx.BNC
                      else gfeat.transpose(1, 2).reshape(B * N, Din))[torch.from_numpy(targets).cuda()].cpu().numpy()
            den = np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)))
            parity = dict(parity or {}, grad_feat_sampled_max_rel_err=float(np.max(np.abs(rows_g - ref) / den)),
                          grad_feat_rows=int(targets.size))

        if pool_fwd_plan is not None and "pool" in state:
            # the planned pooling forward of the timed call against the plain kernel (which the full-size GPU tests
            # compare with the oracle element by element): the same comparisons in the same order, so the same bits
            plain = fx.flexpool_fwd(feat, nbr, layout=layout)
            parity = dict(parity or {}, pool_fwd_planned_equals_plain=bool(
                torch.equal(plain[0].view(torch.int32), state["pool"][0].view(torch.int32))
                and torch.equal(plain[1], state["pool"][1])))
            del plain
        if "pool_bwd" in ops and pool_plan is not None and "pool_grad" in state:
            # the planned pooling backward of the timed call against the list form (which the full-size GPU tests
            # compare with the oracle element by element): the same sums in the same order, so the same bits
            listed = fx.flexpool_bwd(gpool, state["pool"][1], layout=layout, in_edges=in_edges)
            parity = dict(parity or {}, pool_bwd_planned_equals_list_form=bool(
                torch.equal(listed.view(torch.int32), state["pool_grad"].view(torch.int32))))
            del listed

        # ---- CPU baseline: the oracle on a bounded slice of the same workload ----
        def oracle_pass(l0, l1):
            t = time.perf_counter()
            oracle.flexconv_fwd(x.feat, x.pos, x.nbr, x.theta, x.bias, l_range=(l0, l1))
            oracle.flexconv_bwd(x.feat, x.pos, x.nbr, x.theta, x.bias, x.grad_out, l_range=(l0, l1))
            o, a = oracle.flexpool_fwd(x.feat, x.nbr, l_range=(l0, l1))
            a_full = np.zeros(x.feat.shape, np.int32)          # pages are only touched inside the slice
            a_full[:, :, l0:l1] = a
            oracle.flexpool_bwd(x.grad_out if Din == Dout else x.feat, a_full, l_range=(l0, l1))
            return time.perf_counter() - t

        # two short probes size the slice so that the timed pass is about 15 s of CPU work (the first one is
        # dominated by thread start-up and cold pages, so it only sizes the second)
        probe = min(N, 20000)
        per_pt = max(oracle_pass(0, probe) / probe, 1e-9)
        probe = int(min(N, max(probe, 2.0 / per_pt)))
        per_pt = max(oracle_pass(0, probe) / probe, 1e-9)
        n_slice = int(min(N, max(probe, 15.0 / per_pt)))
        t_slice = oracle_pass(0, n_slice)
        cpu_baseline = {"value": n_slice * B / t_slice, "unit": "points/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "sample": f"centre points [0,{n_slice}) of each cloud of the same "
                        f"workload, all four ops, {t_slice:.1f}s", "os_cpu_count": os.cpu_count()}

    graph_ms = None
    if args.graph:
        # the entry points only enqueue kernels, so a step can be captured whole; replays skip the launch path
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            step()
        for _ in range(args.warmup):
            gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            gr.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    direct_flop_pt = 8 * K * Din * Dout
    result = {
        "metric": "flex-conv fwd+bwd (+ flex-max-pool fwd+bwd) points/sec at N=7M,K=8",
        "value": pts / (ms_per_step * 1e-3),
        "unit": "points/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": DTYPE,
        "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}", "B": B, "N": N, "K": K, "Din": Din,
                   "Dout": Dout, "layout": args.layout, "point_order": x.order, "ops": names,
                   "in_edges": "prebuilt once (static neighbourhoods)",
                   "pool_plan": ("prebuilt once (static neighbourhoods)" if pool_plan is not None else "not used"),
                   "pool_fwd_plan": ("prebuilt once (static neighbourhoods)" if pool_fwd_plan is not None else "not used")},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "measured_peaks": measured_peaks,
        "kernel_source_sha256": kernel_source_hash(),
        "rooflines_all": rooflines,
        "op_ms": {n: v for n, v in op_ms.items() if n in ops},      # entry points outside this run's step are not listed
        "inedges_build_ms": inedges_ms,
        "pool_plan_build_ms": pool_plan_ms,
        "pool_plan_bytes": int(pool_plan.numel()) if pool_plan is not None else None,
        "pool_fwd_plan_build_ms": pool_fwd_plan_ms,
        "pool_fwd_plan_bytes": int(pool_fwd_plan.numel()) if pool_fwd_plan is not None else None,
        "graph_ms_per_step": graph_ms,
        "fwd_points_per_s": pts / (fwd_ms * 1e-3) if fwd_ms > 0 else None,
        "fwd_effective_GFLOPs_direct_form": direct_flop_pt * pts / (fwd_ms * 1e-3) / 1e9 if fwd_ms > 0 else None,
        "fwd_bwd_points_per_s": pts / ((fwd_ms + bwd_ms) * 1e-3) if fwd_ms > 0 and bwd_ms > 0 else None,
        "parity": parity,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
