"""The stored target scans (synth/targets.json) equal a live scan."""
import json
import os

import numpy as np

from synth import graphs, workloads


def test_stored_target_scan_equals_a_live_scan():
    with open(workloads._TARGETS_FILE) as f:
        stored = json.load(f)
    name = "gat_rmat16_50k_edges"
    rng = workloads._rng(24)
    N, rp, ci = graphs.rmat(16, 16, rng)
    (_, v, m, sizes), = workloads.pick_targets(rp, ci, 2, 50_000, examine=400)
    assert [int(v), int(m), [int(x) for x in sizes]] == stored[name][0][1:]
    # and the workload built from the stored scan uses that target
    w = workloads.make_workload("gat_rmat")
    assert w.targets == [int(v)] and w.info["players"] == int(m)


def test_fan_out_capped_neighbourhood_of_a_hub():
    """The hub workload: every kept edge is one of the first F neighbours (CSR order) of a node reached earlier,
    the graph is symmetric, everything lies within three hops of the root, and the cap is the smallest that
    reaches the wanted number of edges."""
    rng = workloads._rng(16)
    _, rp, ci = graphs.rmat(13, 3, rng)
    hub = int(np.argmax(np.diff(rp)))
    N, srp, sci, root = graphs.fanout_capped_subgraph(rp, ci, hub, (5, 5, 5))
    rows = np.repeat(np.arange(N), np.diff(srp))
    fwd = set(zip(rows.tolist(), sci.tolist()))
    assert all((b, a) in fwd for a, b in fwd) and all(a != b for a, b in fwd)
    inside, sizes = graphs.khop_ball(srp, sci, root, 3)
    assert inside.all() and sizes[-1] == N
    # by hand: the same sampling, node by node, on the old ids
    seen, frontier, kept = {hub}, [hub], set()
    for _ in range(3):
        nxt = []
        for u in frontier:
            for v in ci[rp[u]:rp[u + 1]][:5].tolist():
                kept.add((min(u, v), max(u, v)))
                if v not in seen:
                    seen.add(v)
                    nxt.append(v)
        frontier = sorted(nxt)
    assert N == len(seen) and len(sci) // 2 == len(kept)
    old = np.array(sorted(seen))
    assert {(int(old[a]), int(old[b])) for a, b in fwd if a < b} == kept and old[root] == hub
    w = workloads.make_workload("c4b_small")
    assert w.info["players"] >= 1500 and w.num_nodes == len(w.row_ptr) - 1 and 0 <= w.targets[0] < w.num_nodes
    F = w.info["fan_out"]
    assert len(graphs.fanout_capped_subgraph(rp, ci, hub, (F - 1,) * 3)[2]) // 2 < 1500 <= w.info["players"]
