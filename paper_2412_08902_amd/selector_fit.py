"""Offline fitting of the window selector on the GPU at hand (procedure of Section IV-C).

    python -m paper_2412_08902_amd.selector_fit --d 64 [--windows 8192] [--share 0,0.5,1] [--out sweep.md]

1. Generate synthetic matrices whose 16-row windows all have the same number of non-zero columns
   c (2..16384) and the same number of non-zeros (c .. 15c, every column non-empty: one entry per
   column at a random row, the rest at random free cells) -- the paper's recipe, replicated over
   many windows so that one launch fills the GPU.  With --share f, each group of four consecutive
   windows (64 rows) has the fraction f of its columns in common, as the windows of a community
   do; f = 0 is the paper's recipe (a window shares nothing with its neighbours).
2. Time the deployed SpMM kernels on each matrix with every window forced to the scalar path and
   with every window forced to the matrix path.
3. Label a sample 1 when the scalar path is faster and fit a logistic regression on
   (ncols, sparsity); print w1, w2, b and their integer encoding for `hcspmm_options.sel_coef`.

4. --block-model instead times both paths on community graphs (2,048 blocks of 64 nodes, intra-block
   fill 0.25 .. 1, four inter-block edges per node; the generator of the benchmark's community
   configuration) at d = 32, 64, 128 in fp32 and bf16: the check of a fitted row on windows that
   mix a dense and a sparse half, which the sweep's homogeneous windows do not contain.

The script only drives the library through its binding and fits with scikit-learn; it is not part
of the SpMM path.
"""
from __future__ import annotations

import argparse
import json
import math
import sys

import numpy as np


def make_matrix(torch, W, c, nnz_w, n_cols, seed, dev, share=0.0):
    """CSR with W windows of 16 rows, each with exactly c distinct columns and nnz_w non-zeros; the first
    round(share * c) columns of a window are those of its group of four windows."""
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    cs = int(round(share * c))
    G = (W + 3) // 4
    gbase = torch.randint(0, n_cols, (G, 1), generator=g, device=dev)
    gstride = torch.randint(0, n_cols // 2, (G, 1), generator=g, device=dev) * 2 + 1
    base = torch.randint(0, n_cols, (W, 1), generator=g, device=dev)
    stride = torch.randint(0, n_cols // 2, (W, 1), generator=g, device=dev) * 2 + 1   # odd: distinct mod 2^k
    ar = torch.arange(c, device=dev).view(1, c)
    own = (base + stride * ar) % n_cols
    if cs > 0:
        grp = torch.arange(W, device=dev) // 4
        common = (gbase[grp] + gstride[grp] * ar) % n_cols
        cols = torch.where(ar < cs, common, own)      # (a private column may repeat a common one: rare, harmless)
    else:
        cols = own
    cols, _ = torch.sort(cols, dim=1)
    keys = torch.rand((W, 16, c), generator=g, device=dev)
    first_row = torch.randint(0, 16, (W, 1, c), generator=g, device=dev)
    keys.scatter_(1, first_row, -1.0)                      # one guaranteed entry per column
    flat = keys.view(W, 16 * c)
    kth = torch.kthvalue(flat, nnz_w, dim=1, keepdim=True).values
    mask = (flat <= kth).view(W, 16, c)
    per_row = mask.sum(dim=2).view(-1)
    rowptr = torch.zeros(W * 16 + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(per_row, 0)
    w_idx, _, j_idx = torch.nonzero(mask, as_tuple=True)   # row-major: (window, row, column) ascending
    colind = cols[w_idx, j_idx].to(torch.int32)
    vals = torch.rand(colind.numel(), generator=g, device=dev) + 0.5
    return rowptr.to(torch.int32), colind.contiguous(), vals


def time_mode(torch, hc, n_rows, n_cols, rp, ci, va, X, Y, mode, reps, mfma_dtype=0):
    plan = hc.hcspmm_prepare(n_rows, n_cols, rp, ci, va, route_mode=mode, mfma_dtype=mfma_dtype)
    for _ in range(3):
        hc.hcspmm_spmm(plan, X, Y)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        hc.hcspmm_spmm(plan, X, Y)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    plan.destroy()
    return ms


def selector_time(rows, coef, H=16):
    """Summed time when every sample takes the path the integer selector picks."""
    t = 0.0
    for r in rows:
        z = coef[0] * H * r["ncols"] ** 2 + coef[1] * (H * r["ncols"] - r["nnzw"]) + coef[2] * H * r["ncols"]
        t += r["ms_mfma"] if z < 0 else r["ms_csr"]
    return t


def grid_search(rows):
    """Within the same linear family z = w1*ncols + w2*sparsity + b, with w1, w2 >= 0 > b (the
    directions Section IV-B establishes), pick the integer coefficients that minimise the summed
    measured time of the sweep.  The samples are weighted by their own duration, so this is the
    objective the selector exists for; classification accuracy is only a proxy for it."""
    best = None
    B = 1 << 20
    ncol_cuts = [0] + [2 ** k for k in range(5, 16)] + [3 * 2 ** k for k in range(4, 14)]     # ncols where z(s=0) = 0
    slopes = [0.0, 0.25, 0.5, 0.75, 0.9, 1.0, 1.1, 1.25, 1.5, 2.0, 3.0, 4.0, 8.0]             # w2 / |b|
    for cut in ncol_cuts:
        w1 = 0 if cut == 0 else int(round(B / cut))
        for sl in slopes:
            coef = [w1, int(round(sl * B)), -B]
            t = selector_time(rows, coef)
            if best is None or t < best[0] - 1e-12:
                best = (t, coef)
    t_csr = sum(r["ms_csr"] for r in rows)
    if t_csr <= best[0]:
        best = (t_csr, [0, 0, 1])                      # the scalar path everywhere
    return best[1], best[0]


def block_model_table(out):
    """Both pure plans on block-model graphs of rising intra-block fill; prints (and writes) one line per case."""
    import time
    import torch
    from . import binding as hc
    from workloads import sbm_graph
    dev = torch.device("cuda:0")
    lines = ["| intra-block fill | window sparsity | d | X | scalar path ms | matrix path ms | scalar / matrix |", "|---|---|---|---|---|---|---|"]
    for p_in in (0.25, 0.5, 0.75, 1.0):
        g = sbm_graph(2048, 64, p_in, 4.0, seed=31)
        rp, ci, va = [torch.from_numpy(a).to(dev) for a in (g.rowptr, g.colind, g.vals)]
        plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=hc.HCSPMM_ROUTE_ALL_MFMA)
        info = hc.hcspmm_plan_info(plan)
        plan.destroy()
        sparsity = 1.0 - g.nnz / (16.0 * info["total_ncols"])
        for d in (32, 64, 128):
            for name, dt, md in (("f32", torch.float32, hc.HCSPMM_F32), ("bf16", torch.bfloat16, hc.HCSPMM_BF16)):
                X = torch.randn(g.n_cols, d, device=dev).to(dt)
                Y = torch.empty(g.n_rows, d, device=dev)
                ms = []
                for mode in (hc.HCSPMM_ROUTE_ALL_CSR, hc.HCSPMM_ROUTE_ALL_MFMA):
                    plan = hc.hcspmm_prepare(g.n_rows, g.n_cols, rp, ci, va, route_mode=mode, d_hint=d, mfma_dtype=md)
                    for _ in range(10):
                        hc.hcspmm_spmm(plan, X, Y)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(100):
                        hc.hcspmm_spmm(plan, X, Y)
                    torch.cuda.synchronize()
                    ms.append((time.perf_counter() - t0) * 10.0)
                    plan.destroy()
                lines.append("| %.2f | %.3f | %d | %s | %.4f | %.4f | %.3f |" % (p_in, sparsity, d, name, ms[0], ms[1], ms[0] / ms[1]))
                print(lines[-1], flush=True)
    if out:
        with open(out, "w") as f:
            f.write("# Both paths on block-model graphs (2,048 blocks of 64, four inter-block edges per node)\n\n"
                    "Command: `python -m paper_2412_08902_amd.selector_fit --block-model`\n\n" + "\n".join(lines) + "\n")
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--d", type=int, default=64)
    ap.add_argument("--windows", type=int, default=8192)
    ap.add_argument("--n-cols", type=int, default=1 << 18)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--x-dtype", default="f32", choices=["f32", "bf16", "f16"], help="storage type of X")
    ap.add_argument("--share", default="0", help="comma-separated fractions of a window's columns that the four windows "
                                                 "of a 64-row group have in common (0 = the paper's recipe)")
    ap.add_argument("--shipped", default=None, help="w1,w2,b of a table row to score on the same samples")
    ap.add_argument("--coarse", action="store_true", help="every other width and density (a third of the samples)")
    ap.add_argument("--out", default=None, help="write a markdown summary here")
    ap.add_argument("--json", default=None, help="write all samples and fits here")
    ap.add_argument("--block-model", action="store_true", help="time both paths on community graphs instead of the sweep")
    args = ap.parse_args()
    if args.block_model:
        return block_model_table(args.out)

    import torch
    from sklearn.linear_model import LogisticRegression
    from . import binding as hc

    dev = torch.device("cuda:0")
    d, W, n_cols = args.d, args.windows, args.n_cols
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.x_dtype]
    mfma_dtype = {"f32": hc.HCSPMM_F32, "bf16": hc.HCSPMM_BF16, "f16": hc.HCSPMM_F16}[args.x_dtype]
    X = torch.randn((n_cols, d), device=dev).to(tdt)
    Y = torch.empty((W * 16, d), device=dev)
    cs = [2, 4, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 2048, 4096, 8192, 16384]
    fills = [1, 1.5, 2, 3, 4, 6, 8, 11, 15]                # non-zeros per column: sparsity 15/16 .. 1/16
    if args.coarse:
        cs, fills = cs[1::2] + [16384], [1, 1.5, 2, 4, 8, 15]
    shares = [float(v) for v in args.share.split(",")]
    rows = []
    for share in shares:
        for c in cs:
            # fewer windows for wide ones (bounded matrix size); the widest come a few at a time, as
            # they do in real graphs, where a window is one workgroup's serial work on the matrix path
            Wc = max(256, min(W, (1 << 22) // c)) if c <= 4096 else 32
            for f in fills:
                nnz_w = int(min(15 * c, max(c, round(c * f))))
                rp, ci, va = make_matrix(torch, Wc, c, nnz_w, n_cols, seed=1000 * c + int(10 * f), dev=dev, share=share)
                t_csr = time_mode(torch, hc, Wc * 16, n_cols, rp, ci, va, X, Y, hc.HCSPMM_ROUTE_ALL_CSR, args.reps, mfma_dtype)
                t_mfma = time_mode(torch, hc, Wc * 16, n_cols, rp, ci, va, X, Y, hc.HCSPMM_ROUTE_ALL_MFMA, args.reps, mfma_dtype)
                sp = 1.0 - nnz_w / (16.0 * c)
                rows.append(dict(ncols=c, nnzw=nnz_w, sparsity=sp, share=share, ms_csr=t_csr, ms_mfma=t_mfma,
                                 label=int(t_csr < t_mfma)))
                print("share=%.2f c=%4d nnz=%5d sparsity=%.3f  csr %.4f ms  mfma %.4f ms  -> %s" %
                      (share, c, nnz_w, sp, t_csr, t_mfma, "scalar" if t_csr < t_mfma else "matrix"), flush=True)
    feats = np.array([[r["ncols"], r["sparsity"]] for r in rows], dtype=np.float64)
    labels = np.array([r["label"] for r in rows])
    result = dict(d=d, x_dtype=args.x_dtype, windows=W, n_cols=n_cols, samples=rows)
    if labels.min() == labels.max():
        # one path wins everywhere in the sampled region: encode "always" with the constant term only
        coef = [0, 0, 1 if labels[0] == 1 else -1]
        result.update(w=[0.0, 0.0, float(coef[2])], accuracy=1.0, sel_coef=coef)
    else:
        scale = np.array([1.0 / 4096.0, 1.0])
        # a sample counts by how much the choice matters: near-ties carry almost no weight
        weight = np.abs(np.log(np.array([r["ms_csr"] / r["ms_mfma"] for r in rows]))) + 1e-3
        clf = LogisticRegression(C=1e4, max_iter=10000).fit(feats * scale, labels, sample_weight=weight)
        w1, w2 = (clf.coef_[0] * scale).tolist()
        b = float(clf.intercept_[0])
        acc = float((clf.predict(feats * scale) == labels).mean())
        # integer encoding: common positive scale so that the largest coefficient is about 2^20
        k = (1 << 20) / max(abs(w1), abs(w2), abs(b))
        coef = [int(round(w1 * k)), int(round(w2 * k)), int(round(b * k))]
        H = 16
        agree = 0
        for r in rows:
            z = coef[0] * H * r["ncols"] ** 2 + coef[1] * (H * r["ncols"] - r["nnzw"]) + coef[2] * H * r["ncols"]
            agree += int((0 if z < 0 else 1) == r["label"])
        picked = sum(r["ms_mfma"] if (coef[0] * H * r["ncols"] ** 2 + coef[1] * (H * r["ncols"] - r["nnzw"]) +
                                          coef[2] * H * r["ncols"]) < 0 else r["ms_csr"] for r in rows)
        best = sum(min(r["ms_csr"], r["ms_mfma"]) for r in rows)
        result.update(w=[w1, w2, b], accuracy=acc, sel_coef=coef, integer_accuracy=agree / len(rows),
                      time_vs_best=picked / best, all_scalar_vs_best=sum(r["ms_csr"] for r in rows) / best,
                      all_matrix_vs_best=sum(r["ms_mfma"] for r in rows) / best)
    g_coef, g_time = grid_search(rows)
    best_time = sum(min(r["ms_csr"], r["ms_mfma"]) for r in rows)
    if args.shipped:
        shipped = [int(v) for v in args.shipped.split(",")]
        result.update(shipped_sel_coef=shipped, shipped_time_vs_best=selector_time(rows, shipped) / best_time)
    result.update(grid_sel_coef=g_coef, grid_time_vs_best=g_time / best_time,
                  all_scalar_vs_best=sum(r["ms_csr"] for r in rows) / best_time,
                  all_matrix_vs_best=sum(r["ms_mfma"] for r in rows) / best_time)
    print(json.dumps({k: v for k, v in result.items() if k != "samples"}))
    if args.json:
        with open(args.json, "w") as f:
            json.dump(result, f)
    if args.out:
        with open(args.out, "w") as f:
            f.write("# Selector sweep, X in %s, d = %d (up to %d windows per matrix, X %d x %d)\n\n" %
                    (args.x_dtype, d, W, n_cols, d))
            f.write("Command: `python -m paper_2412_08902_amd.selector_fit --d %d --x-dtype %s --windows %d --n-cols %d --share %s%s`\n\n" %
                    (d, args.x_dtype, W, n_cols, args.share, " --coarse" if args.coarse else ""))
            f.write("Fit: z = w1*ncols + w2*sparsity + b, w = %s, accuracy %.3f; sel_coef = %s\n\n" %
                    (result["w"], result["accuracy"], result["sel_coef"]))
            f.write("Time-minimising coefficients in the same family (w1, w2 >= 0 > b): sel_coef = %s, summed time %.3f x "
                    "the per-sample best\n\n" % (result["grid_sel_coef"], result["grid_time_vs_best"]))
            if "time_vs_best" in result:
                f.write("Summed time over the sweep relative to always picking the faster path: selector %.3f, "
                        "all-scalar %.3f, all-matrix %.3f\n\n" % (result["time_vs_best"], result["all_scalar_vs_best"],
                                                                   result["all_matrix_vs_best"]))
            if "shipped_time_vs_best" in result:
                f.write("Shipped row %s on these samples: %.3f x the per-sample best\n\n" %
                        (result["shipped_sel_coef"], result["shipped_time_vs_best"]))
            f.write("| shared | ncols | nnz/window | sparsity | scalar path ms | matrix path ms | faster |\n|---|---|---|---|---|---|---|\n")
            for r in rows:
                f.write("| %.2f | %d | %d | %.3f | %.4f | %.4f | %s |\n" % (r["share"], r["ncols"], r["nnzw"], r["sparsity"],
                                                                        r["ms_csr"], r["ms_mfma"], "scalar" if r["label"] else "matrix"))
    return 0


if __name__ == "__main__":
    sys.exit(main())
