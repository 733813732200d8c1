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
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2509_25041_amd as grace
    from workloads import CONFIGS, make_workload

    assert torch.cuda.is_available(), "routing_report.py needs a GPU"
    cfg = CONFIGS[args.workload]
    setups = [("no replicas", dataclasses.replace(cfg, n_hot=0), grace.GRACE_POLICY_TAR),
              ("replicas, weighted round-robin", cfg, grace.GRACE_POLICY_WRR),
              ("replicas, locality first", cfg, grace.GRACE_POLICY_TAR)]
    for name, c, policy in setups:
        wl = make_workload(c)
        pl = wl.placement
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
            "grace_send_lists_ms": float(np.median(send_ms)),
        }))
    return 0


if __name__ == "__main__":
    sys.exit(main())
