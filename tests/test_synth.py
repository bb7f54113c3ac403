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
