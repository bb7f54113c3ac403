#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step is one complete pass of the hot path over one batch of synthetic input: one explanation
(extraction -> sampling -> masked GCN inference of every coalition -> weighted least squares) of the
workload's target, or, for the 64-target configuration, one ds_explain_batch call over all 64 targets.
Graph, features and weights are resident in HBM before the timed region. Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--others c2,c3,c5,c4b]

The headline workload is the largest single-GPU configuration (config 4: one million players, 400,000
coalitions, a 50 GB mask matrix). Short runs of the other configurations are reported under
"other_workloads", each with its own roofline. A step of config 4 takes seconds, so the warm-up is
cut short once it has taken `--warmup-budget-s` seconds (at least one warm-up step always runs; the
JSON states how many ran), and the extra workloads and the CPU baseline are skipped when the process
is about to run out of `--time-budget-s`.
"""
import argparse
import json
import os
import sys
import time

T_START = time.perf_counter()
ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
# plain integer/fp32 VALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
FP64_PEAK_TFLOPS = 78.6
FP32_PEAK_TFLOPS = 157.3


def inference_flops_per_coalition(ctx, cg, dims):
    """Algorithmic flops of one masked GCN evaluation of the target: aggregation over the entries
    that can reach the target (half of them active on average over a complementary pair, one
    multiply-add per feature) plus the per-coalition dense transforms of layers >= 2."""
    import numpy as np
    info = ctx.cgraph_info(cg)
    L = len(dims) - 1
    gid, hop = ctx.cgraph_nodes(cg)
    es, ed = ctx.cgraph_edges(cg)
    gid, hop = gid.cpu().numpy(), hop.cpu().numpy()
    order = np.argsort(gid)
    hs = hop[order][np.searchsorted(gid[order], es.cpu().numpy())]
    hd = hop[order][np.searchsorted(gid[order], ed.cpu().numpy())]
    flops = 0.0
    for l in range(1, L + 1):
        radius = min(L - l, info.hops)
        entries = int((hs <= radius).sum() + (hd <= radius).sum())     # directed entries into rows of that ball
        width = dims[1] if l == 1 else dims[l - 1]
        flops += 0.5 * entries * width * 2
        if l >= 2:
            flops += 2.0 * info.ball[radius] * dims[l - 1] * dims[l]
    return flops


def gat_flops_per_coalition(ctx, cg, model):
    """Algorithmic flops of one masked GAT evaluation of the target: per active entry of a needed row (half of
    them on average) one attention logit and one weighted accumulate per feature column (4 flop), plus the dense
    transform of layers >= 2 on the rows they read."""
    import numpy as np
    info = ctx.cgraph_info(cg)
    heads, widths = model["heads"], model["widths"]
    L = len(heads)
    gid, hop = ctx.cgraph_nodes(cg)
    es, ed = ctx.cgraph_edges(cg)
    gid, hop = gid.cpu().numpy(), hop.cpu().numpy()
    order = np.argsort(gid)
    hs = hop[order][np.searchsorted(gid[order], es.cpu().numpy())]
    hd = hop[order][np.searchsorted(gid[order], ed.cpu().numpy())]
    flops, din = 0.0, None
    for l in range(1, L + 1):
        radius = min(L - l, info.hops)
        entries = int((hs <= radius).sum() + (hd <= radius).sum())
        zw = heads[l - 1] * widths[l - 1]
        flops += 0.5 * entries * zw * 4
        if l >= 2:
            flops += 2.0 * info.ball[min(L - l + 1, info.hops)] * din * zw
        din = zw
    return flops


def cpu_baseline(w, gpu_iterations, budget_s=20.0):
    """The C oracle (OpenMP, one coalition per thread, fp64, every layer on every node) as it stands, timed on
    this machine's host cores on a bounded sample of the same workload: the first rows of the same mask matrix
    (rows 0/1 and whole complementary pairs, which ascend by size, so the sample is also spread over the sizes).
    Inference is timed on the sample; the solve is timed as one conjugate-gradient step on the sample's rows and
    scaled to all rows and to the number of steps the GPU run needed (config 3/4), or as the oracle's dense
    least-squares solve on the sample (small configs). Both are extrapolated linearly to one explanation."""
    import numpy as np
    from oracle import cfast, compgraph
    if w.gat is not None:
        return None
    target = w.targets[0]
    cg = compgraph.extract(w.row_ptr, w.col, target, w.num_layers)
    n = cg["num_players"]
    k = w.n_samples - w.n_samples % 2
    threads = cfast.threads()
    K1 = k // 2

    def rows_spread(count):
        per = max(count // 16, 1)                        # pairs per block; eight blocks spread over the pair index
        starts = np.unique(np.linspace(1, max(K1 - per, 1), 8).astype(np.int64))
        parts = [cfast.sample(n, w.n_samples, w.seed, target & 0xFFFFFFFF, pair_range=(0, 1))]
        parts += [cfast.sample(n, w.n_samples, w.seed, target & 0xFFFFFFFF, pair_range=(int(s), int(min(s + per, K1))))
                  for s in starts]
        return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])

    probe = 2 * threads
    Z, wt = rows_spread(probe)
    t0 = time.perf_counter()
    cfast.gcn_values(cg, w.features, w.weights, Z)
    per = (time.perf_counter() - t0) / len(Z)
    rows = int(max(probe, min(k, 0.7 * budget_s / max(per, 1e-9))))
    Z, wt = rows_spread(rows)
    t0 = time.perf_counter()
    y, _, _ = cfast.gcn_values(cg, w.features, w.weights, Z)
    t_inf = time.perf_counter() - t0
    evals_per_s = len(Z) / t_inf
    # one conjugate-gradient step = one product with Z and one with its transpose, whose cost is proportional to
    # the rows walked, plus vector work that is not: the step is timed on the sample repeated to a few thousand
    # rows and on four rows, and the difference is scaled to all k rows
    def step_seconds(Zr, wr, yr):
        t0 = time.perf_counter()
        cfast.cgls(n, Zr, wr, yr, tol=0.0, max_iter=1)
        t1 = time.perf_counter()
        cfast.cgls(n, Zr, wr, yr, tol=0.0, max_iter=3)
        return max((time.perf_counter() - t1) - (t1 - t0), 0.0) / 2.0
    reps = int(max(1, min(4000 // len(Z), (1 << 30) // max(Z.nbytes, 1))))
    Zr, wr, yr = np.tile(Z, (reps, 1)), np.tile(wt, reps), np.tile(y, reps)
    t_fixed = step_seconds(Z[:4], wt[:4], y[:4])
    t_rows = step_seconds(Zr, wr, yr)
    t_step = t_fixed + max(t_rows - t_fixed, 0.0) * (k / len(Zr))
    iters = gpu_iterations if gpu_iterations > 0 else 100.0   # direct-solver configs: a nominal 100 steps
    solve_s = t_step * iters
    e2e = k / evals_per_s + solve_s
    return {"value": evals_per_s, "unit": "coalition evals/s (masked inference)", "cores": threads, "kind": "oracle",
            "sec_per_explained_node_extrapolated": e2e,
            "sample": f"{len(Z)} rows (rows 0/1 and eight blocks of pairs spread evenly over the {K1 - 1} sampled pairs) of the same mask "
                      f"matrix: inference {t_inf:.1f} s measured; end to end = all {k} rows at that rate + "
                      f"{iters:.0f} conjugate-gradient steps ({'the count of the GPU run' if gpu_iterations > 0 else 'nominal: the GPU run solved directly'}) at {t_step:.2f} s each (a step timed on "
                      f"{len(Zr)} rows, the sample repeated, and scaled by rows)"}


def progress(msg):
    """Progress goes to stderr (stdout carries the one JSON line): a step of the large workloads takes seconds, and
    a run that prints nothing for minutes is taken to be hung."""
    print(f"[bench {time.perf_counter() - T_START:7.1f} s] {msg}", file=sys.stderr, flush=True)


def read_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload`, from the committed rocprofv3 --pmc summaries
    (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain copy of known
    size). None if no summary covers it."""
    pdir = os.path.join(ROOT, "profiles")
    try:
        for fn in sorted(os.listdir(pdir)):
            for line in open(os.path.join(pdir, fn)):
                parts = line.split()
                if len(parts) >= 4 and parts[0] == "traffic_bytes" and parts[1] == workload and parts[2] == kernel:
                    return float(parts[3])
    except OSError:
        pass
    return None


def run_workload(key, steps, warmup, warmup_budget_s, batch, copy_probe_mib=0, max_iter=0):
    """Time `steps` steps of workload `key`; returns (result dict, workload, mean CGLS iterations)."""
    import numpy as np
    import torch
    from paper_2506_22668_amd import Context, Options, DS_SOLVER_CGLS, DS_SOLVER_GRAM_CHOL, DS_BF16_IN_F32_ACC, DS_F32
    from synth import make_workload

    t_gen = time.perf_counter()
    progress(f"{key}: generating the workload")
    w = make_workload(key)
    t_gen = time.perf_counter() - t_gen
    progress(f"{key}: {w.name} generated in {t_gen:.1f} s; uploading, extracting")
    ctx = Context("cuda:0")
    ctx.set_graph(w.row_ptr, w.col)
    ctx.set_features(w.features)
    if w.gat is not None:
        ctx.set_gat(w.gat["W"], w.gat["a_src"], w.gat["a_dst"], w.gat["heads"], negative_slope=w.gat["slope"])
    else:
        ctx.set_gcn(w.weights, transform_dtype=DS_BF16_IN_F32_ACC if w.transform_dtype == "bf16" else DS_F32)
    opts = Options(solver=DS_SOLVER_CGLS if w.solver == "cgls" else DS_SOLVER_GRAM_CHOL, tol=w.tol,
                   max_iter=max_iter if max_iter > 0 else w.max_iter)
    targets = w.targets
    many = len(targets) > 1                      # the 64-target configuration: a step is one batch call
    flops_of, capacity = {}, 0      # algorithmic inference flops per coalition, per target
    for tgt in targets:
        cg = ctx.extract(tgt, opts)
        flops_of[ctx.cgraph_info(cg).num_players] = (gat_flops_per_coalition(ctx, cg, w.gat) if w.gat is not None
                                                      else inference_flops_per_coalition(ctx, cg, list(w.dims)))
        capacity += ctx.cgraph_info(cg).num_players
        ctx.cgraph_free(cg)

    def step():
        if many:
            return ctx.explain_batch(targets, w.n_samples, w.seed, opts, capacity=capacity)[5]
        return [ctx.explain(targets[0], w.n_samples, w.seed, opts, capacity=capacity, want_edges=False,
                            allow_not_converged=max_iter > 0)[3]]

    if copy_probe_mib > 0:
        ctx.copy_probe(copy_probe_mib << 20)
    warm_done, t0 = 0, time.perf_counter()
    for i in range(max(warmup, 1)):
        step()
        warm_done += 1
        progress(f"{key}: warm-up step {warm_done} done")
        if time.perf_counter() - t0 > warmup_budget_s:
            break
    torch.cuda.synchronize()
    reports = []
    t0 = time.perf_counter()
    t_last = t0
    for i in range(steps):
        reports.extend(step())
        if time.perf_counter() - t_last > 20.0:      # a line now and then; never inside a step
            t_last = time.perf_counter()
            progress(f"{key}: timed step {i + 1} of {steps} done")
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    progress(f"{key}: {steps} steps in {elapsed:.2f} s")

    k_total = sum(r.num_rows for r in reports)
    per_step = len(reports) // steps
    mean = lambda name: float(np.mean([getattr(r, name) for r in reports]))
    mean_of = lambda fn: float(np.mean([fn(r) for r in reports]))   # algorithmic work differs from game to game
    rep = max(reports[:per_step], key=lambda r: r.num_players)
    n, V, W64, rows = rep.num_players, rep.num_nodes, (rep.num_players + 63) // 64, rep.num_rows
    iters = mean("cgls_iterations")
    # per-kernel-group durations: HIP events recorded by the library on its own stream inside the timed region
    # (means over all explanations of the run); algorithmic work per explanation from the library's report
    stream_eval = mean("ms_k_stream") > 0              # long mask rows: streaming kernel + layers kernel
    eval_tflop = mean_of(lambda r: r.num_rows * flops_of[r.num_players]) / 1e12
    kernels = {
        "gram_popcount": {"ms": mean("ms_k_gram"), "bound": "alu",
                          # lower triangle of n^2 column pairs x 64-row words x (AND, popcount, weighted add)
                          "alg": mean_of(lambda r: 3.0 * (r.num_players * (r.num_players + 1) / 2) * ((r.num_rows + 63) // 64)) / 1e12
                          if mean("ms_k_gram") > 0 else 0.0, "peak": ALU_PEAK_TOPS, "unit": "Top/s"},
        "cholesky_fp64": {"ms": mean("ms_k_chol"), "bound": "mfma",
                          "alg": mean_of(lambda r: r.num_players ** 3 / 3.0) / 1e12 if mean("ms_k_chol") > 0 else 0.0,
                          "peak": FP64_PEAK_TFLOPS, "unit": "TFLOP/s"},
        # all iterations of the conjugate-gradient loop; per iteration the small member of every pair once for
        # Z u and once for Z^T r
        "cgls_loop": {"ms": mean("ms_k_cgls"), "bound": "hbm", "alg": mean("bytes_solve") / 1e9 if iters > 0 else 0.0,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "launches": max(int(round(iters)), 1)},
    }
    if stream_eval:
        # the kernel that streams the mask matrix (one member of every pair) against HBM, the layers on its compact
        # output (first layer on the fp32 matrix cores) against the fp32 matrix-core peak
        kernels["mask_stream"] = {"ms": mean("ms_k_stream"), "bound": "hbm", "alg": mean("bytes_eval") / 1e9,
                                  "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        kernels["masked_gcn_layers"] = {"ms": mean("ms_k_eval") - mean("ms_k_stream"), "bound": "mfma", "alg": eval_tflop,
                                        "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        # short mask rows (one coalition per lane, everything but the mask on chip): arithmetic-bound
        kernels["masked_gat_eval" if w.gat is not None else "masked_gcn_eval"] = {
            "ms": mean("ms_k_eval"), "bound": "alu", "alg": eval_tflop, "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s"}
    for v in kernels.values():
        v["achieved"] = (v["alg"] / (v["ms"] / 1e3)) if v["ms"] > 0 else 0.0
        v["frac"] = v["achieved"] / v["peak"]
    dom_name = max(kernels, key=lambda name: kernels[name]["ms"])
    dom = kernels[dom_name]
    launches = dom.get("launches", 1)
    out = {
        "value": k_total / elapsed,
        "ms_per_step": 1e3 * elapsed / steps,
        "steps": steps, "warmup": warm_done,
        "dtype": "f32" if w.transform_dtype != "bf16" else "bf16 per-coalition transforms, f32 accumulate",
        "config": {"workload": w.name, "graph_nodes": w.num_nodes, "players": int(n), "cg_nodes": int(V),
                   "coalitions": int(rows), "pairs_sampled": int(rep.num_pairs), "solver": w.solver,
                   **({"gat_heads": w.gat["heads"], "gat_head_widths": w.gat["widths"]} if w.gat is not None
                      else {"gcn_dims": list(w.dims)}),
                   "targets_per_step": per_step},
        "sec_per_explained_node": elapsed / len(reports),
        "inference_stage_evals_per_sec": rows / (mean("ms_eval") / 1e3) if mean("ms_eval") > 0 else None,
        "stage_ms": {s: mean("ms_" + s) for s in ("extract", "sample", "eval", "solve", "total")},
        "algorithmic_bytes": {s: mean("bytes_" + s) for s in ("sample", "eval", "solve")},
        "cgls_iterations": iters,
        "roofline": {"kernel": dom_name, "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                     "unit": dom["unit"], "frac": dom["frac"], "traffic": read_traffic(dom_name, w.name),
                     "avg_launch_ms": dom["ms"] / launches, "launches": launches},
        "kernels": {name: {kk: v[kk] for kk in ("ms", "bound", "achieved", "peak", "unit", "frac")}
                    for name, v in kernels.items()},
        "generation_s": t_gen,
    }
    if many:
        out["games_players_min_max"] = [int(min(r.num_players for r in reports)), int(max(r.num_players for r in reports))]
    # several explanations of one target in flight (ds_explain_batch keeps up to eight on worker contexts)
    if batch > 0 and not many:
        tg = [targets[0]] * batch
        ctx.explain_batch(tg, w.n_samples, w.seed, opts, capacity=capacity * batch)   # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps_b = 3
        for _ in range(reps_b):
            ctx.explain_batch(tg, w.n_samples, w.seed, opts, capacity=capacity * batch)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out["batch"] = {"targets_per_call": batch, "sec_per_explained_node": dt / (reps_b * batch),
                        "coalition_evals_per_sec": reps_b * batch * rows / dt}
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    return out, w, iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--others", default="c2,c3,c5,c4b",
                    help="comma-separated workloads timed briefly after the headline one (\"\" = none)")
    ap.add_argument("--other-steps", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch", type=int, default=16,
                    help="small workloads: also time ds_explain_batch on this many copies of the target (0 = skip)")
    ap.add_argument("--warmup-budget-s", type=float, default=12.0)
    ap.add_argument("--time-budget-s", type=float, default=480.0,
                    help="wall-clock budget of the process: optional parts are skipped when it is nearly spent")
    ap.add_argument("--profile-max-iter", type=int, default=0,
                    help="profiling runs only: stop the conjugate-gradient loop after this many steps (the result is "
                         "then not the converged one and the line is not a benchmark)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB first (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one GPU's share on one GPU; --gpus must be 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    small = args.workload in ("c1", "c2", "c2_small", "gat_c2", "gat_small", "c5_small", "c3_small", "c4_small")
    head, w, iters = run_workload(args.workload, args.steps, args.warmup, args.warmup_budget_s,
                                  args.batch if small else 0, args.copy_probe_mib, args.profile_max_iter)
    out = {
        "metric": ("masked-GAT" if w.gat is not None else "masked-GCN") +
                  " coalition evals/sec; end-to-end seconds per explained node",
        "value": head.pop("value"),
        "unit": "coalition evals/s (end to end: extraction + sampling + inference + solve)",
        "n_gpus": 1, "steps": head.pop("steps"), "warmup": head.pop("warmup"), "warmup_requested": args.warmup,
        "ms_per_step": head.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head.pop("dtype"), "data": "synthetic",
    }
    if args.profile_max_iter > 0:
        out["profiling_run_cgls_capped_at"] = args.profile_max_iter
    out.update(head)
    left = lambda: args.time_budget_s - (time.perf_counter() - T_START)
    others = {}
    # rough cost of a short run of each (generation + warm-up + steps), seconds
    cost = {"c2": 15, "c3": 50, "c5": 25, "c4": 80, "c4b": 15, "gat_c2": 15, "gat_rmat": 20}
    for key in [s for s in args.others.split(",") if s and s != args.workload]:
        need = cost.get(key, 30) + (0 if args.no_cpu_baseline else 35)
        if left() < need:
            others[key] = {"skipped": f"{left():.0f} s of the process's time budget left, about {need} s needed"}
            continue
        r, _, _ = run_workload(key, args.other_steps, 1, 5.0, args.batch if key in ("c2", "gat_c2") else 0)
        others[key] = r
    if others:
        out["other_workloads"] = others
    if not args.no_cpu_baseline:
        progress("CPU baseline (the C oracle on a sample of the same rows)")
        budget = min(20.0, max(5.0, left() - 15.0))
        out["cpu_baseline"] = cpu_baseline(w, iters, budget)
    out["wall_s"] = time.perf_counter() - T_START
    print(json.dumps(out))


if __name__ == "__main__":
    main()
