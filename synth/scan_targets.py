"""Run the target scans of the large workloads and store their results in targets.json
(`python -m synth.scan_targets [workload keys]`). The scan only counts edges of k-hop induced
sub-graphs; the stored (node, player count, ball sizes) tuples let `make_workload` skip it."""
import json
import os
import sys
import time

os.environ["DISTSHAP_SYNTH_RESCAN"] = "1"

from synth import workloads  # noqa: E402


def main(keys):
    out = {}
    if os.path.exists(workloads._TARGETS_FILE):
        with open(workloads._TARGETS_FILE) as f:
            out = json.load(f)
    for key in keys:
        t0 = time.time()
        w = workloads.WORKLOADS[key]()
        players, balls = w.info["players"], w.info["balls"]
        if not isinstance(players, list):
            players, balls = [players], [balls]
        out[w.name] = [[abs(m - w.info.get("want", m)), int(v), int(m), [int(x) for x in b]]
                       for v, m, b in zip(w.targets, players, balls)]
        print(f"{key}: {w.name} targets={w.targets[:4]}... {time.time() - t0:.1f} s", flush=True)
    with open(workloads._TARGETS_FILE, "w") as f:
        f.write("{\n" + ",\n".join(f" {json.dumps(k)}: {json.dumps(v, separators=(',', ':'))}"
                                    for k, v in sorted(out.items())) + "\n}\n")


if __name__ == "__main__":
    main(sys.argv[1:] or ["c3", "c4", "c5", "gat_rmat"])
