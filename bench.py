#!/usr/bin/env python3
"""Benchmark of the hybrid SpMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--no-modes] [--no-cold] [--no-cpu]

One "step" is one `hcspmm_spmm` call (Y = A X on the hybrid plan: every window goes through the
path its selector flag names) on the named synthetic workload, with the CSR, X, Y and the plan
already resident in HBM; the plan is built once beforehand, as the method prescribes
(preprocessing is a one-time cost that is reported separately, in `prepare_ms`).

Prints ONE JSON line:
  metric/value   SpMM GFLOP/s = 2 nnz d / t over the K timed steps
  roofline       dominant kernel of the step: algorithmic HBM bytes of its share of the work
                 divided by its average duration (HIP events on the launch stream), vs 8 TB/s
                 (plus gather_floor_ms / gather_ceiling_frac: the bare gather of X rows along the same column
                 stream, the floor of any kernel that fetches one row per non-zero, and the step relative to it)
  t_cold_ms      median time of a step with cold caches (512 MiB flush before every repetition)
  modes          the same workload on the all-CSR and all-MFMA plans, next to the hybrid plan
  cpu_baseline   the CPU oracle (plain CSR triple loop, fp64) timed on this machine's host cores
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# rocprofv3 summaries of the dominant kernel per workload (HBM-side bytes per launch from FETCH_SIZE / WRITE_SIZE runs,
# each with the full command that produced it).  Counters cannot be read from inside this process, so the bench line
# carries "traffic": null and names the summary instead.
TRAFFIC_PROFILE = {
    ("C4", "k_csr"): "profiles/k_csr_C4_large_powerlaw.md",
    ("C5", "k_mfma_wg"): "profiles/k_mfma_wg_C5_dense_powerlaw.md",
    ("C2", "k_csr"): "profiles/k_csr_C2_C3.md",
    ("C3", "k_csr"): "profiles/k_csr_C2_C3.md",
}

WORKLOAD_TEXT = {
    "C1": "C1 small power-law: N=2,708, 10,556 edges + self-loops, values 1, X 2708x32 fp32 U[-1,1]",
    "C2": "C2 medium power-law: N=169,343, 2.3M edges + self-loops, GCN-normalised, X Nx128 fp32 N(0,1)",
    "C3": "C3 community SBM: N=131,072 (2,048 blocks of 64), p_in 0.25, inter degree 4, values 1, X Nx64 fp32 N(0,1)",
    "C4": "C4 large power-law: N=2,449,029, 123.7M edges + self-loops, GCN-normalised, X Nx32 fp32 U[-1,1]",
    "C5": "C5 dense-ish power-law, SpMM stage of the GCN layer: N=232,965, 114.6M edges + self-loops, T Nx128 fp32",
    "C6": "C6 mixed (not in the baseline's list): 131,072 nodes in blocks of 64 at 75 % fill + 169,343 power-law nodes "
          "(C2's recipe), disjoint, GCN-normalised, X Nx128 fp32 N(0,1)",
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C4", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--modes", action="store_true", help="(default; kept for old command lines) time the all-CSR and all-MFMA plans too")
    ap.add_argument("--no-modes", action="store_true", help="skip the all-CSR and all-MFMA plans")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache timing (512 MiB flush before every repetition)")
    ap.add_argument("--no-gather-probe", action="store_true", help="skip the bare-gather floor of the scalar path")
    ap.add_argument("--gather-ceiling", action="store_true",
                    help="also time the bare gather on uniform indices and on the hub / cold bands of the column stream")
    ap.add_argument("--x-dtype", default="f32", choices=["f32", "bf16", "f16"], help="storage type of X")
    ap.add_argument("--y-dtype", default="f32", choices=["f32", "bf16", "f16"], help="storage type of Y (one rounding when stored)")
    ap.add_argument("--layer", action="store_true",
                    help="C5 only: time the whole GCN layer Y = ReLU(A (X W)) (GEMM + hybrid SpMM) instead of the SpMM")
    ap.add_argument("--t-dtype", default="f32", choices=["f32", "bf16", "f16"],
                    help="with --layer: storage type of the intermediate X W (f32 is the headline layer)")
    ap.add_argument("--matrix-kernels", default="auto", choices=["auto", "per_window", "runs"],
                    help="kernels of the matrix path: per window (what auto picks), or runs of four windows sharing X rows in LDS")
    ap.add_argument("--sel-coef", default=None, help="three comma-separated integers overriding the shipped selector")
    ap.add_argument("--agg-update", type=int, default=None, metavar="D_OUT",
                    help="also time the aggregate-then-update layer Y = ReLU((A X) W) with a d x D_OUT W, with the "
                         "update stage fused into the SpMM kernels and as SpMM + GEMM")
    ap.add_argument("--backward", type=int, default=0, metavar="D_IN",
                    help="also time the layer's backward pass (S = A G, dX = S W^T, dW = X^T S) for a D_IN x d W")
    ap.add_argument("--update", action="store_true",
                    help="also time hcspmm_plan_update for 1, 10^3 and 10^5 changed rows against a preparation from scratch")
    ap.add_argument("--graph", type=int, default=0, metavar="N",
                    help="also capture N back-to-back SpMM calls in a HIP graph and time its replays "
                         "(separates launch latency from kernel time on the small configs)")
    ap.add_argument("--scramble", action="store_true",
                    help="relabel the vertices at random first (a layout with no locality)")
    ap.add_argument("--loa", type=int, default=None, metavar="VW",
                    help="reformat the layout first (Section V-B) with a vertices window of VW")
    ap.add_argument("--calib", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2412_08902_amd.binding as hc
    from workloads import make_config, dense_normal, CONFIGS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    name = args.workload
    t0 = time.time()
    g, X, Wm = make_config(name, with_dense=(name != "C5" or args.layer))
    layout = None
    if args.scramble or args.loa is not None:
        from workloads import random_relabel, CSRGraph
        layout = {"scrambled": bool(args.scramble), "loa_vw": args.loa}
        if args.scramble:
            g = random_relabel(g, seed=777)
        if args.loa is not None:
            t1 = time.perf_counter()
            order, before, after = hc.hcspmm_loa_order_checked(g.n_rows, g.n_cols, g.rowptr, g.colind, args.loa)
            layout["loa_order_ms"] = round((time.perf_counter() - t1) * 1e3, 1)
            layout["total_ncols_before"], layout["total_ncols_after"] = before, after
            layout["applied"] = bool(after < before)
            if after < before:                       # the regrouping can scatter a layout that already had locality
                t1 = time.perf_counter()
                rp2, ci2, va2 = hc.hcspmm_permute_csr(g.n_rows, g.rowptr, g.colind, g.vals, order)
                layout["permute_ms"] = round((time.perf_counter() - t1) * 1e3, 1)
                g = CSRGraph(g.n_rows, g.n_cols, rp2, ci2, va2)
        log("layout: %s" % layout)
    X_in = X
    if name == "C5":                      # SpMM stage of the layer: T = X W has the layer's output width
        X = dense_normal(g.n_rows, CONFIGS["C5"]["d"], seed=1)
    d = X.shape[1]
    from workloads import to_bf16_bits, to_f16_bits
    x_bits = None
    if args.x_dtype != "f32":
        x_bits = to_bf16_bits(X) if args.x_dtype == "bf16" else to_f16_bits(X)
    log("generated %s: N=%d nnz=%d d=%d in %.1fs" % (name, g.n_rows, g.nnz, d, time.time() - t0))
    rp = torch.from_numpy(g.rowptr).to(dev)
    ci = torch.from_numpy(g.colind).to(dev)
    va = torch.from_numpy(g.vals).to(dev)
    if x_bits is None:
        Xd = torch.from_numpy(X).to(dev)
    else:
        Xd = torch.from_numpy(x_bits.view(np.int16)).to(dev).view(torch.bfloat16 if args.x_dtype == "bf16" else torch.float16)
    y_torch = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.y_dtype]
    Yd = torch.empty((g.n_rows, d), dtype=y_torch, device=dev)
    sy = 4 if args.y_dtype == "f32" else 2
    mfma_dtype = {"f32": hc.HCSPMM_F32, "bf16": hc.HCSPMM_BF16, "f16": hc.HCSPMM_F16}[args.x_dtype]
    sx = 4 if x_bits is None else 2
    flops = 2.0 * g.nnz * d

    sel_coef = [int(v) for v in args.sel_coef.split(",")] if args.sel_coef else None

    def prepare(mode):
        torch.cuda.synchronize()
        t = time.perf_counter()
        plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=d, sel_coef=sel_coef,
                                 mfma_dtype=mfma_dtype,
                                 matrix_kernels={"auto": 0, "per_window": 1, "runs": 2}[args.matrix_kernels])
        torch.cuda.synchronize()
        return plan, (time.perf_counter() - t) * 1e3

    plan, _ = prepare(hc.HCSPMM_ROUTE_HYBRID)          # first call also pays one-time runtime set-up
    plan.destroy()
    plan, prepare_ms = prepare(hc.HCSPMM_ROUTE_HYBRID)
    info = hc.hcspmm_plan_info(plan)
    log("plan: %d windows, %d on the matrix path (%d nnz), prepare %.2f ms" %
        (info["n_windows"], info["n_mfma_windows"], info["nnz_mfma"], prepare_ms))

    ms = time_steps(lambda: hc.hcspmm_spmm(plan, Xd, Yd), args.steps, args.warmup, torch)
    gflops = flops / (ms * 1e-3) / 1e9
    log("hybrid: %.3f ms/step, %.1f GFLOP/s" % (ms, gflops))

    # per-stage durations (HIP events on the launch stream), averaged over the same number of launches
    stage_sum = {}
    for _ in range(args.steps):
        st = hc.hcspmm_spmm_timed(plan, Xd, Yd)
        for k, v in st.items():
            stage_sum[k] = stage_sum.get(k, 0.0) + v
    stage_ms = {k: v / args.steps for k, v in stage_sum.items()}
    log("stages (ms): " + ", ".join("%s=%.4f" % (k[3:], v) for k, v in stage_ms.items()))

    # share of the work per stage -> algorithmic bytes of the dominant kernel
    nnz_mfma = info["nnz_mfma"]
    nnz_csr = g.nnz - nnz_mfma
    rows_mfma = min(info["n_mfma_windows"] * 16, g.n_rows)
    rows_csr = g.n_rows - rows_mfma
    share = {
        "ms_csr": dict(kernel="k_csr", rows=rows_csr, nnz=nnz_csr, extra_per_nnz=0),
        # the matrix path also reads 4 B per non-zero (condensed column + row) and 4 B per condensed column
        "ms_mfma_small": dict(kernel="k_mfma_small", rows=rows_mfma, nnz=nnz_mfma, extra_per_nnz=4),
        "ms_mfma_big": dict(kernel="k_mfma_wg", rows=rows_mfma, nnz=nnz_mfma, extra_per_nnz=4),
    }
    dom = max(share, key=lambda k: stage_ms.get(k, 0.0))
    s = share[dom]
    # B_min of the kernel's share: rowptr + (colind, val) + X read once + its Y rows written once
    alg_bytes = 4.0 * (s["rows"] + 1) + (8.0 + s["extra_per_nnz"]) * s["nnz"] + g.n_cols * d * sx + s["rows"] * d * float(sy)
    achieved = alg_bytes / (stage_ms[dom] * 1e-3) / 1e9
    whole_bytes = 4.0 * (g.n_rows + 1) + 8.0 * g.nnz + g.n_cols * d * sx + g.n_rows * d * float(sy)
    roofline = dict(bound="hbm", kernel=s["kernel"], achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=None,
                    traffic_profile=TRAFFIC_PROFILE.get((name, s["kernel"])),
                    algorithmic_bytes=int(alg_bytes), kernel_ms=round(stage_ms[dom], 5),
                    whole_step_frac=round(whole_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))

    out = dict(metric="spmm_gflops (2*nnz*d/t)", value=round(gflops, 2), unit="GFLOP/s", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(ms, 5), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype=args.x_dtype, y_dtype=args.y_dtype, data="synthetic",
               config=dict(workload=WORKLOAD_TEXT[name], name=name, n=g.n_rows, nnz=g.nnz, d=d, route_mode="hybrid",
                           n_windows=info["n_windows"], mfma_windows=info["n_mfma_windows"],
                           nnz_on_matrix_path=nnz_mfma, sel_coef=info["sel_coef"], matrix_kernels=args.matrix_kernels,
                           total_ncols=info["total_ncols"], n_runs=info["n_runs"], run_union_cols=info["run_union_cols"]),
               roofline=roofline, prepare_ms=round(prepare_ms, 3),
               stage_ms={k: round(v, 5) for k, v in stage_ms.items()})

    if layout is not None:
        layout["computing_intensity"] = round(g.nnz / max(1, info["total_ncols"]), 4)      # Eq. 5 over all windows
        out["layout"] = layout

    Y_hybrid = Yd.float().cpu().numpy()              # output of the timed SpMM, checked against the oracle below

    if args.layer and name == "C5":
        Xin_d = torch.from_numpy(X_in).to(dev)
        Wd = torch.from_numpy(Wm).to(dev)
        ws = torch.empty(hc.hcspmm_gcn_workspace_bytes(plan, X_in.shape[1], d), dtype=torch.uint8, device=dev)
        Tg = torch.empty((g.n_rows, d), dtype=torch.float32, device=dev)
        ms_gemm = time_steps(lambda: hc.hcspmm_gemm_f32(Xin_d, Wd, Tg), args.steps, args.warmup, torch)
        ms_layer = time_steps(lambda: hc.hcspmm_gcn_layer_ex(plan, Xin_d, Wd, Yd, ws), args.steps, args.warmup, torch)
        if args.t_dtype != "f32":
            code = hc.HCSPMM_BF16 if args.t_dtype == "bf16" else hc.HCSPMM_F16
            plan16 = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, d_hint=d, mfma_dtype=code)
            ms16 = time_steps(lambda: hc.hcspmm_gcn_layer_ex(plan16, Xin_d, Wd, Yd, ws, t_dtype=code), args.steps,
                              args.warmup, torch)
            plan16.destroy()
            log("layer with %s intermediate: %.3f ms" % (args.t_dtype, ms16))
        gemm_flops = 2.0 * g.n_rows * X_in.shape[1] * d
        out["layer"] = dict(ms_per_layer=round(ms_layer, 5), ms_gemm=round(ms_gemm, 5),
                            **({"ms_per_layer_%s_intermediate" % args.t_dtype: round(ms16, 5)} if args.t_dtype != "f32" else {}),
                            gemm_tflops=round(gemm_flops / (ms_gemm * 1e-3) / 1e12, 2),
                            gemm_frac_of_fp32_mfma_peak=round(gemm_flops / (ms_gemm * 1e-3) / 157.3e12, 4),
                            total_gflops=round((gemm_flops + flops) / (ms_layer * 1e-3) / 1e9, 1))
        log("layer: %.3f ms (gemm alone %.3f ms = %.1f TFLOP/s)" % (ms_layer, ms_gemm, out["layer"]["gemm_tflops"]))
        del Xin_d, Wd, ws, Tg

    if args.graph > 0:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            hc.hcspmm_spmm(plan, Xd, Yd)                       # every lazy allocation happens before the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(args.graph):
                hc.hcspmm_spmm(plan, Xd, Yd)
        reps = max(3, args.steps // 10)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / (reps * args.graph)
        same = bool(np.array_equal(Yd.float().cpu().numpy(), Y_hybrid))
        out["graph_replay"] = dict(calls_per_graph=args.graph, replays=reps, ms_per_call=round(ms_graph, 5),
                                   bitwise_equal_to_eager=same)
        log("graph replay: %.5f ms per SpMM call (eager %.5f), same bits: %s" % (ms_graph, ms, same))
        del graph

    if args.agg_update:
        from workloads import glorot_uniform
        d_out = args.agg_update
        Wd = torch.from_numpy(glorot_uniform(d, d_out, seed=4242)).to(dev)
        ws = torch.empty(hc.hcspmm_aggregate_update_workspace_bytes(plan, d, d_out), dtype=torch.uint8, device=dev)
        Y2 = torch.empty((g.n_rows, d_out), dtype=torch.float32, device=dev)
        Zt = torch.empty((g.n_rows, d), dtype=torch.float32, device=dev)
        ms_fused = time_steps(lambda: hc.hcspmm_aggregate_update(plan, Xd, Wd, Y2, ws), args.steps, args.warmup, torch)
        Y_fused = Y2.clone()
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_SPLIT)
        ms_split = time_steps(lambda: hc.hcspmm_aggregate_update(plan, Xd, Wd, Y2, ws), args.steps, args.warmup, torch)
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_AUTO)
        ms_gemm = time_steps(lambda: hc.hcspmm_gemm_f32(Zt, Wd, Y2), args.steps, args.warmup, torch)
        out["aggregate_update"] = dict(d_in=d, d_out=d_out, ms_fused=round(ms_fused, 5), ms_spmm_then_gemm=round(ms_split, 5),
                                       ms_gemm_alone=round(ms_gemm, 5), ms_spmm_alone=round(ms, 5),
                                       max_abs_diff_fused_vs_split=float((Y_fused - Y2).abs().max().item()) if False else None)
        hc.hcspmm_aggregate_update(plan, Xd, Wd, Y2, ws)
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_SPLIT)
        Y3 = torch.empty_like(Y2)
        hc.hcspmm_aggregate_update(plan, Xd, Wd, Y3, ws)
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_AUTO)
        torch.cuda.synchronize()
        out["aggregate_update"]["max_abs_diff_fused_vs_split"] = float((Y2 - Y3).abs().max().item())
        log("aggregate-update: fused %.4f ms, spmm+gemm %.4f ms (gemm alone %.4f)" % (ms_fused, ms_split, ms_gemm))
        del Wd, ws, Y2, Y3, Zt, Y_fused

    if args.backward:
        # backward pass of a layer with a D_IN x d weight matrix: G is n x d (d = the workload's width), X is n x D_IN
        from workloads import glorot_uniform
        d_in = args.backward
        Wb = torch.from_numpy(glorot_uniform(d_in, d, seed=4343)).to(dev)
        Xb = torch.from_numpy(dense_normal(g.n_rows, d_in, seed=4344)).to(dev)
        Gb = Xd if args.x_dtype == "f32" else torch.from_numpy(dense_normal(g.n_cols, d, seed=4345)).to(dev)
        Yf = torch.from_numpy(dense_normal(g.n_cols, d, seed=4346)).to(dev)
        wsb = torch.empty(hc.hcspmm_layer_backward_workspace_bytes(plan, d_in, d), dtype=torch.uint8, device=dev)
        dXb = torch.empty((g.n_rows, d_in), dtype=torch.float32, device=dev)
        dWb = torch.empty((d_in, d), dtype=torch.float32, device=dev)
        bw = lambda **kw: hc.hcspmm_layer_backward(plan, Gb, Xb, Wb, dXb, dWb, wsb, **kw)
        ms_b = time_steps(lambda: bw(), args.steps, args.warmup, torch)
        ms_b_mask = time_steps(lambda: bw(Y_fwd=Yf), args.steps, args.warmup, torch)
        ms_b_emask = time_steps(lambda: bw(mask_dx_by_x=True), args.steps, args.warmup, torch)
        ms_dx = time_steps(lambda: hc.hcspmm_layer_backward(plan, Gb, Xb, Wb, dXb, None, wsb), args.steps, args.warmup, torch)
        ms_dw = time_steps(lambda: hc.hcspmm_layer_backward(plan, Gb, Xb, Wb, None, dWb, wsb), args.steps, args.warmup, torch)
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_SPLIT)
        ms_b_split = time_steps(lambda: bw(), args.steps, args.warmup, torch)
        hc.hcspmm_plan_set_update_fusion(plan, hc.HCSPMM_UPDATE_AUTO)
        out["layer_backward"] = dict(d_in=d_in, d_out=d, ms=round(ms_b, 5), ms_with_activation_mask=round(ms_b_mask, 5),
                                     ms_with_dx_masked_in_epilogue=round(ms_b_emask, 5),
                                     ms_unfused=round(ms_b_split, 5), ms_dx_only=round(ms_dx, 5), ms_dw_only=round(ms_dw, 5),
                                     ms_spmm_alone=round(ms, 5),
                                     dw_stream_gbps=round((g.n_rows * (d_in + d) * 4) / max(ms_dw - ms, 1e-6) / 1e6, 1))
        log("layer backward: %.4f ms (unfused %.4f; dX only %.4f, dW only %.4f, with mask pass %.4f, with dX masked in "
            "the epilogue %.4f; spmm alone %.4f)" % (ms_b, ms_b_split, ms_dx, ms_dw, ms_b_mask, ms_b_emask, ms))
        del Wb, Xb, Yf, wsb, dXb, dWb

    if args.update:
        # structural change without moving the arrays: the last column index of each chosen row is raised by one (rows
        # stay sorted and duplicate-free); successive calls alternate between the two versions of the column array
        rng = np.random.default_rng(4711)
        lens = np.diff(g.rowptr)
        res = {"prepare_from_scratch_ms": round(prepare_ms, 3)}
        for n_changed in (1, 1000, 100000):
            rows = np.unique(rng.choice(g.n_rows, min(n_changed, g.n_rows), replace=False)).astype(np.int32)
            last = g.rowptr[rows + 1].astype(np.int64) - 1
            ok = (lens[rows] > 0) & (g.colind[np.maximum(last, 0)] < g.n_cols - 1)
            rows, last = rows[ok], last[ok]
            ci2 = ci.clone()
            ci2[torch.from_numpy(last).to(dev)] += 1
            ts = []
            for rep in range(6):
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                hc.hcspmm_plan_update(plan, rp, ci2 if rep % 2 == 0 else ci, va, rows)
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t1) * 1e3)
            res["update_ms_%d_rows" % n_changed] = round(float(np.median(ts[1:])), 3)
            res["windows_touched_%d_rows" % n_changed] = int(np.unique(rows // 16).shape[0])
            del ci2
        out["plan_update"] = res
        log("plan update: %s" % res)

    if not args.no_cold:
        # cold caches: a 512 MiB write between repetitions evicts the L2s and the memory-side cache
        flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(min(args.steps, 100)):
            flush.fill_(1)
            e0.record()
            hc.hcspmm_spmm(plan, Xd, Yd)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        out["t_cold_ms"] = round(float(np.median(ts)), 5)
        out["t_cold_reps"] = len(ts)
        roofline["whole_step_frac_cold"] = round(whole_bytes / (out["t_cold_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        del flush

    if not args.no_gather_probe and args.x_dtype == "f32" and d % 4 == 0 and d <= 256:
        # Floor of the scalar path: the bare gather of X rows along the same column stream (no row structure, no
        # values, no output).  A kernel that fetches one X row per non-zero cannot run faster than this.
        def probe_ms(index, reps):
            buf = torch.empty(hc.hcspmm_probe_gather_out_bytes(index.numel(), d), dtype=torch.uint8, device=dev)
            return time_steps(lambda: hc.hcspmm_probe_gather(index, Xd, buf, d=d), reps, 3, torch)
        reps = max(5, min(args.steps, 20))
        g_ms = probe_ms(ci, reps)
        roofline["gather_floor_ms"] = round(g_ms, 5)
        # what the whole step achieves relative to that floor (1.0 = the memory system's rate for this access pattern)
        roofline["gather_ceiling_frac"] = round(g_ms / ms, 4)
        log("bare gather of the column stream: %.3f ms (%.2f TB/s of X rows); hybrid step = %.3f of that rate" %
            (g_ms, g.nnz * d * 4 / (g_ms * 1e-3) / 1e12, g_ms / ms))
        if args.gather_ceiling:
            gen = torch.Generator(device=dev)
            gen.manual_seed(99)
            uni = torch.randint(0, g.n_cols, (g.nnz,), dtype=torch.int32, device=dev, generator=gen)
            res = {"column_stream_ms": round(g_ms, 5), "uniform_ms": round(probe_ms(uni, reps), 5)}
            del uni
            for band in (4096, 32768, 262144):
                if band >= g.n_cols:
                    continue
                hot = ci[ci < band]
                cold = ci[ci >= band]
                res["band_%d" % band] = dict(hot_share=round(hot.numel() / g.nnz, 4), hot_ms=round(probe_ms(hot, reps), 5),
                                             cold_ms=round(probe_ms(cold, reps), 5))
                del hot, cold
            out["gather_ceiling"] = res
            log("gather ceiling: %s" % res)

    if args.calib:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)          # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 2.0, out=dst)          # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        out["calib_copy_bytes"] = int(src.numel() * 4)
        del src, dst

    if not args.no_modes:
        modes = {}
        for label, mode in (("all_csr", hc.HCSPMM_ROUTE_ALL_CSR), ("all_mfma", hc.HCSPMM_ROUTE_ALL_MFMA)):
            p2, pm = prepare(mode)
            steps = args.steps if label == "all_csr" else max(3, args.steps // 5)
            m2 = time_steps(lambda: hc.hcspmm_spmm(p2, Xd, Yd), steps, min(args.warmup, 3), torch)
            modes[label] = dict(ms_per_step=round(m2, 5), gflops=round(flops / (m2 * 1e-3) / 1e9, 2),
                                prepare_ms=round(pm, 3))
            log("%s: %.3f ms/step" % (label, m2))
            p2.destroy()
        # the hybrid plan once more, under the same conditions as the two pure plans (the headline figure above is
        # timed first, on a GPU that a sub-millisecond workload has not yet brought up to its clocks)
        m2 = time_steps(lambda: hc.hcspmm_spmm(plan, Xd, Yd), args.steps, min(args.warmup, 3), torch)
        modes["hybrid"] = dict(ms_per_step=round(m2, 5), gflops=round(flops / (m2 * 1e-3) / 1e9, 2),
                               ms_per_step_headline=round(ms, 5))
        out["modes"] = modes
    plan.destroy()

    if not args.no_cpu:
        import oracle
        # bounded sample: whole windows spread evenly over the matrix, at most 5e10 multiply-adds
        budget = 5.0e10
        total_fma = float(g.nnz) * d
        W = (g.n_rows + 15) // 16
        stride = max(1, int(np.ceil(total_fma / budget)))
        wins = np.arange(0, W, stride)
        rows = (wins[:, None] * 16 + np.arange(16)[None, :]).reshape(-1)
        rows = rows[rows < g.n_rows]
        t1 = time.perf_counter()
        x_or, code = (X, None) if x_bits is None else (x_bits, oracle.DT_BF16 if args.x_dtype == "bf16" else oracle.DT_F16)
        ref = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, x_or, code)
        cpu_s = time.perf_counter() - t1
        lens = np.diff(g.rowptr.astype(np.int64))[rows]
        cpu_gflops = 2.0 * float(lens.sum()) * d / cpu_s / 1e9
        bound = oracle.spmm_rows(rows, g.rowptr, g.colind, g.vals, x_or, code, use_abs=True)
        err = np.abs(Y_hybrid[rows].astype(np.float64) - ref)
        gate = (1e-5 if x_bits is None else 2e-2) + {"f32": 0.0, "bf16": 2.0 ** -8, "f16": 2.0 ** -11}[args.y_dtype]
        ok = bool(np.all(err <= gate * bound + (2.0 ** -25 if args.y_dtype == "f16" else 1e-30)))
        out["cpu_baseline"] = dict(value=round(cpu_gflops, 3), unit="GFLOP/s", cores=oracle.num_threads(), kind="oracle",
                                   sample="every %d-th 16-row window (%d rows, %d non-zeros), %.1f s" %
                                          (stride, rows.shape[0], int(lens.sum()), cpu_s))
        out["parity_on_sample"] = ok
        # largest error relative to the componentwise magnitude bound |A| |X| (the gate is 1e-5, or 2e-2 for 16-bit X)
        out["parity_max_err_over_bound"] = float(np.max(err / (bound + 1e-300)))
        log("cpu oracle: %.2f GFLOP/s on %d threads; GPU rows match oracle: %s" % (cpu_gflops, oracle.num_threads(), ok))
        # the same oracle on one thread, on every 8th window of that sample
        n_thr = oracle.num_threads()
        sub = rows.reshape(-1, 16)[::8].reshape(-1) if rows.shape[0] % 16 == 0 and rows.shape[0] >= 128 else rows
        try:
            oracle.set_num_threads(1)
            t1 = time.perf_counter()
            oracle.spmm_rows(sub, g.rowptr, g.colind, g.vals, x_or, code)
            one_s = time.perf_counter() - t1
        finally:
            oracle.set_num_threads(n_thr)
        sub_nnz = float(np.diff(g.rowptr.astype(np.int64))[sub].sum())
        out["cpu_baseline"]["one_thread_value"] = round(2.0 * sub_nnz * d / max(one_s, 1e-9) / 1e9, 3)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
