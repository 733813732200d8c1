#!/usr/bin/env python3
"""Routing report: what replication and the two routing policies do to traffic and load.

For a seeded synthetic workload, every virtual rank routes the same batch of
tokens through the library on one GPU (top-k gate, replica pick, send lists,
offsets) under three set-ups, the columns of the paper's ablation (Section 6.3,
Table 1): no replicas, replicas with weighted round-robin over all instances
(Section 4.3, first policy), replicas with locality-first routing (Algorithm 4).
Reported, summed over the source ranks and in tokens: rows each destination rank
receives (mean, max, standard deviation: the paper's load-balance metric),
cross-node and intra-node traffic with and without de-duplication (Section 5).
With --planner two more set-ups run on a table that the offline planner of this package builds
from the profiled expert loads and the primary groups (Equation 3: number of replicas and hot set
of the heaviest group; Equation 4: predicted loads -> integer polling weights), under both policies.
Prints one JSON object per set-up.  Inputs are synthetic (see workloads/).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="olmoe")
    ap.add_argument("--planner", action="store_true",
                    help="also route on the table planner.plan_layer builds (Equations 3 and 4)")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2509_25041_amd as grace
    from paper_2509_25041_amd import planner
    from workloads import CONFIGS, make_workload
    from workloads.generator import primary_group_sizes

    assert torch.cuda.is_available(), "routing_report.py needs a GPU"
    cfg = CONFIGS[args.workload]
    setups = [("no replicas", dataclasses.replace(cfg, n_hot=0), grace.GRACE_POLICY_TAR),
              ("replicas, weighted round-robin", cfg, grace.GRACE_POLICY_WRR),
              ("replicas, locality first", cfg, grace.GRACE_POLICY_TAR)]
    if args.planner:
        setups += [("planner table (Equations 3, 4), weighted round-robin", cfg, grace.GRACE_POLICY_WRR),
                   ("planner table (Equations 3, 4), locality first", cfg, grace.GRACE_POLICY_TAR)]
    for name, c, policy in setups:
        wl = make_workload(c)
        pl = wl.placement
        extra = {}
        if name.startswith("planner"):
            # the generator's contiguous primary groups and profiled loads are the planner's inputs
            groups, e = [], 0
            for sz in primary_group_sizes(c.E, c.R):
                groups.append(list(range(e, e + sz)))
                e += sz
            pl = planner.plan_layer(pl.profile_load, groups, c.nodes, c.gpus_per_node)
            extra = {"n_replica": int(pl.n_replica), "hot_experts": [int(h) for h in pl.hot],
                     "replica_ranks": [int(r) for r in pl.targets], "poll_weight": [int(w) for w in pl.poll_weight]}
        table = grace.GraceTable.from_placement(pl)
        logits = torch.from_numpy(wl.logits).cuda()
        rows = np.zeros(pl.R, np.int64)
        traffic = np.zeros(4, np.int64)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        send_ms = []
        for lr in range(pl.R):
            _, _, ti, _ = grace.grace_route(table, lr, logits, c.k, policy=policy)
            ev0.record()
            tr = grace.grace_send_lists(table, lr, ti)[5]
            ev1.record()
            roff = grace.grace_permute(table, ti, None)[3]
            torch.cuda.synchronize()
            send_ms.append(ev0.elapsed_time(ev1))
            rows += np.diff(roff.cpu().numpy().astype(np.int64))
            traffic += tr.cpu().numpy()
        print(json.dumps({
            "workload": c.name, "setup": name, "ranks": int(pl.R), "nodes": int(pl.N), "instances": int(pl.I),
            "tokens_per_rank": int(c.T), "top_k": int(c.k),
            "rows_per_rank": {"mean": float(rows.mean()), "max": int(rows.max()), "std": float(rows.std())},
            "cross_node_tokens": {"dedup": int(traffic[0]), "one_row_per_assignment": int(traffic[1])},
            "intra_node_tokens": {"dedup": int(traffic[2]), "flat_dispatch_rows": int(traffic[3])},
            "grace_send_lists_ms": float(np.median(send_ms)), **extra,
        }))
    return 0


if __name__ == "__main__":
    sys.exit(main())
