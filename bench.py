#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step is one complete explanation (extraction -> sampling -> masked GCN inference
of every coalition -> weighted least squares) of one target of the workload, with
the graph, features and weights already resident in HBM. Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]
"""
import argparse
import json
import os
import sys
import time

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
    hop_of = dict(zip(gid.tolist(), hop.tolist()))
    hs = np.array([hop_of[int(x)] for x in es.cpu().numpy()])
    hd = np.array([hop_of[int(x)] for x in ed.cpu().numpy()])
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
    hop_of = dict(zip(gid.cpu().numpy().tolist(), hop.cpu().numpy().tolist()))
    hs = np.array([hop_of[int(x)] for x in es.cpu().numpy()])
    hd = np.array([hop_of[int(x)] for x in ed.cpu().numpy()])
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


def cholesky_launches(n, block=64, fuse_rows=2048, super_cols=256):
    """Kernel launches of the blocked factorisation (the library's rules): while more than `fuse_rows` rows
    trail a super-panel of 256 columns, 4 panels + 3 narrow updates (each factorising the next diagonal block) +
    1 diagonal block (not the very first: that one is factorised when the system matrix is built, outside the
    timed group) + 1 wide update; afterwards one launch per full 64-column block that has columns behind it
    (panel solve, trailing update and the next diagonal block together, plus one copy of the panel before the
    first of them), and a panel launch for the last block; a diagonal block has a launch of its own only if
    the launch before it did not factorise it."""
    count, done, j0, panel_ready = 0, True, 0, False   # the first diagonal block is factorised with the system matrix
    while j0 < n:
        if (n + 1) - j0 - super_cols > fuse_rows and n - j0 >= super_cols + block:
            count += (0 if j0 == 0 else 1) + 4 + 3 + 1
            j0 += super_cols
            done = False
            continue
        nb = min(block, n - j0)
        count += 0 if done else 1
        done = False
        rest = n + 1 - j0 - nb
        if n - j0 - nb > 0 and rest <= fuse_rows:
            count += (0 if panel_ready else 1) + 1
            panel_ready, done = True, True
        else:
            count += 1
            if n - j0 - nb > 0:
                count += 1
        j0 += nb
    return count


def cpu_baseline(w, budget_s=20.0):
    """The oracle's masked inference, as it stands, on a bounded prefix of the same
    coalitions (rows of the same mask matrix), timed on this machine's host cores."""
    import numpy as np
    from oracle import compgraph, gat, gcn, sampling
    target = w.targets[0]
    cg = compgraph.extract(w.row_ptr, w.col, target, w.num_layers)
    n = cg["num_players"]
    if w.gat is not None:
        f = gat.ValueFunction(cg, w.features, w.gat)
    else:
        f = gcn.ValueFunction(cg, w.features, w.weights, bf16=(w.transform_dtype == "bf16"))
    probe = 64
    Z, wt, sz = sampling.sample(n, w.n_samples, w.seed, target & 0xFFFFFFFF, pair_range=(0, probe // 2))
    bits = sampling.unpack_rows(Z, n)
    f.batch(bits[:8])                       # first calls pay one-off costs
    t0, c0 = time.perf_counter(), time.process_time()
    f.batch(bits)
    per = (time.perf_counter() - t0) / probe
    rows = int(max(probe, min(w.n_samples, budget_s / max(per, 1e-9))))
    rows -= rows % 2
    Z, wt, sz = sampling.sample(n, w.n_samples, w.seed, target & 0xFFFFFFFF, pair_range=(0, rows // 2))
    bits = sampling.unpack_rows(Z, n)
    t0, c0 = time.perf_counter(), time.process_time()
    f.batch(bits)
    wall, cpu = time.perf_counter() - t0, time.process_time() - c0
    return {"value": rows / wall, "unit": "coalition evals/s", "cores": max(1, int(round(cpu / wall))),
            "kind": "oracle", "sample": f"first {rows} rows (pairs 0..{rows // 2 - 1}) of the same mask matrix, "
            f"masked inference only, {wall:.1f} s"}


def read_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload`, from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain copy of known
    size). None if no summary covers it."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 4 and parts[0] == "traffic_bytes" and parts[1] == workload and parts[2] == kernel:
                return float(parts[3])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch", type=int, default=16,
                    help="also time ds_explain_batch on this many targets (0 = skip); reported under \"batch\"")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB first (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one GPU's share on one GPU; --gpus must be 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_22668_amd import Context, Options, DS_SOLVER_CGLS, DS_SOLVER_GRAM_CHOL, DS_BF16_IN_F32_ACC, DS_F32
    from synth import make_workload

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    w = make_workload(args.workload)
    ctx = Context("cuda:0")
    ctx.set_graph(w.row_ptr, w.col)
    ctx.set_features(w.features)
    if w.gat is not None:
        ctx.set_gat(w.gat["W"], w.gat["a_src"], w.gat["a_dst"], w.gat["heads"], negative_slope=w.gat["slope"])
    else:
        ctx.set_gcn(w.weights, transform_dtype=DS_BF16_IN_F32_ACC if w.transform_dtype == "bf16" else DS_F32)
    opts = Options(solver=DS_SOLVER_CGLS if w.solver == "cgls" else DS_SOLVER_GRAM_CHOL, tol=w.tol,
                   max_iter=w.max_iter)
    targets = w.targets
    cg = ctx.extract(targets[0], opts)
    info = ctx.cgraph_info(cg)
    capacity = max(ctx.cgraph_info(c).num_players for c in [cg])
    eval_flops = (gat_flops_per_coalition(ctx, cg, w.gat) if w.gat is not None
                  else inference_flops_per_coalition(ctx, cg, list(w.dims)))
    ctx.cgraph_free(cg)
    if len(targets) > 1:
        caps = []
        for t in targets:
            c = ctx.extract(t, opts)
            caps.append(ctx.cgraph_info(c).num_players)
            ctx.cgraph_free(c)
        capacity = max(caps)

    def step(i):
        return ctx.explain(targets[i % len(targets)], w.n_samples, w.seed, opts, capacity=capacity,
                           want_edges=False)

    if args.copy_probe_mib > 0:
        ctx.copy_probe(args.copy_probe_mib << 20)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    reports = []
    t0 = time.perf_counter()
    for i in range(args.steps):
        reports.append(step(i)[3])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    k = sum(r.num_rows for r in reports)
    ms_per_step = 1e3 * elapsed / args.steps
    mean = lambda name: float(np.mean([getattr(r, name) for r in reports]))
    rep = reports[0]
    n, V, W64 = rep.num_players, rep.num_nodes, (rep.num_players + 63) // 64
    rows = rep.num_rows
    KW = (rows + 63) // 64
    # per-kernel durations (HIP events on the library's stream, recorded inside the timed region)
    kernels = {
        # small graphs (one coalition per lane, everything but the mask on chip): arithmetic-bound;
        # large ones stream the mask matrix: compulsory HBM bytes per coalition = its mask row in, one float out
        ("masked_gat_eval" if w.gat is not None else "masked_gcn_eval"): ({"ms": mean("ms_k_eval"), "bound": "alu", "alg": rows * eval_flops / 1e12,
                             "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s"} if (n <= 2048 or w.gat is not None) else
                            {"ms": mean("ms_k_eval"), "bound": "hbm", "alg": rows * (W64 * 8 + 4) / 1e9,
                             "peak": HBM_PEAK_GBS, "unit": "GB/s"}),
        "gram_popcount": {"ms": mean("ms_k_gram"), "bound": "alu",
                          # lower triangle of n^2 column pairs x KW 64-row words x (AND, popcount, weighted add)
                          "alg": 3.0 * (n * (n + 1) / 2) * KW / 1e12, "peak": ALU_PEAK_TOPS, "unit": "Top/s"},
        # the factorisation is a group of launches (per 64-column block: panel, then the trailing update that also
        # factorises the next diagonal block; the first diagonal block has a launch of its own)
        "cholesky_fp64": {"ms": mean("ms_k_chol"), "bound": "alu", "launches": cholesky_launches(n),
                          "alg": (n ** 3 / 3.0) / 1e12, "peak": FP64_PEAK_TFLOPS, "unit": "TFLOP/s"},
        "cgls_loop": {"ms": mean("ms_k_cgls"), "bound": "hbm",
                      # per iteration: the small member of every pair once, plus its transposed copy once
                      "alg": mean("cgls_iterations") * 2 * (rows // 2) * W64 * 8 / 1e9, "peak": HBM_PEAK_GBS,
                      "unit": "GB/s"},
    }
    for v in kernels.values():
        v["achieved"] = (v["alg"] / (v["ms"] / 1e3)) if v["ms"] > 0 else 0.0
        v["frac"] = v["achieved"] / v["peak"]
    dom_name = max(kernels, key=lambda name: kernels[name]["ms"])
    dom = kernels[dom_name]
    traffic = read_traffic(dom_name, w.name)
    out = {
        "metric": ("masked-GAT" if w.gat is not None else "masked-GCN") +
                  " coalition evals/sec; end-to-end seconds per explained node",
        "value": k / elapsed,
        "unit": "coalition evals/s (end to end: extraction + sampling + inference + solve)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.transform_dtype != "bf16" else "bf16 transforms, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": w.name, "graph_nodes": w.num_nodes, "players": int(n), "cg_nodes": int(V),
                   "coalitions": int(rows), "solver": w.solver,
                   **({"gat_heads": w.gat["heads"], "gat_head_widths": w.gat["widths"]} if w.gat is not None
                      else {"gcn_dims": list(w.dims)}),
                   "targets_cycled": len(targets)},
        "sec_per_explained_node": elapsed / args.steps,
        "inference_stage_evals_per_sec": rows / (mean("ms_eval") / 1e3) if mean("ms_eval") > 0 else None,
        "stage_ms": {s: mean("ms_" + s) for s in ("extract", "sample", "eval", "solve", "total")},
        "cgls_iterations": mean("cgls_iterations"),
        "roofline": {"kernel": dom_name, "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                     "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic,
                     "avg_launch_ms": dom["ms"], "launches": dom.get("launches", 1)},
        "kernels": {name: {kk: v[kk] for kk in ("ms", "bound", "achieved", "peak", "unit", "frac")}
                    for name, v in kernels.items()},
    }
    # several explanations in flight (ds_explain_batch runs up to eight at a time on worker contexts)
    if args.batch > 0:
        tg = [targets[i % len(targets)] for i in range(args.batch)]
        ctx.explain_batch(tg, w.n_samples, w.seed, opts, capacity=capacity * args.batch)   # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps_b = 3
        for _ in range(reps_b):
            ctx.explain_batch(tg, w.n_samples, w.seed, opts, capacity=capacity * args.batch)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out["batch"] = {"targets_per_call": args.batch, "sec_per_explained_node": dt / (reps_b * args.batch),
                        "coalition_evals_per_sec": reps_b * args.batch * rows / dt}
    ctx.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
