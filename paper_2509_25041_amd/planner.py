"""Offline placement planner (host side, runs once per layer; not on the hot path).

Turns per-expert load statistics and a grouping into the placement / replica
table and the integer polling weights that the hot path consumes, following the
paper's dynamic replication (Section 4.2, Equation 3), load prediction
(Section 4.3, Equation 4) and the group-size window of the controlled
non-uniform grouping (Algorithm 2).  Affinity-based grouping itself (spectral
clustering on co-activation statistics) is outside this repository: groups are
an input.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np


def group_size_window(n_experts: int, n_groups: int, r: float = 0.15):
    """(num_min, num_max) of Algorithm 2: E = floor(N_e / D), delta = max(1, round(E * r))."""
    e = n_experts // n_groups
    delta = max(1, int(round(e * r)))
    return max(1, e - delta), e + delta


def n_replica(w_max: float, w_mean: float, n_gpu: int) -> int:
    """Equation 3: min(max(1, floor(W_max / W_mean)), n_gpu - 1)."""
    return int(min(max(1, int(np.floor(w_max / w_mean))), n_gpu - 1))


def hot_experts(loads: Sequence[float], experts: Sequence[int], w_max: float, n_rep: int) -> List[int]:
    """Section 4.2: inside the heaviest group, experts ranked by load (descending, ties to the lower
    id); the leading ones up to and including the first whose cumulative load exceeds
    W_max * n_rep / (1 + n_rep) (strictly: a cumulative load equal to the threshold does not end
    the hot set)."""
    order = sorted(experts, key=lambda e: (-loads[e], e))
    thr = w_max * n_rep / (1.0 + n_rep)
    out, cum = [], 0.0
    for e in order:
        out.append(e)
        cum += loads[e]
        if cum > thr:
            break
    return out


@dataclass
class Plan:
    E: int
    R: int
    N: int
    rank_node: np.ndarray
    poll_weight: np.ndarray
    inst_ptr: np.ndarray
    inst_rank: np.ndarray
    hot: List[int] = field(default_factory=list)
    n_replica: int = 0
    targets: List[int] = field(default_factory=list)
    predicted_load: Optional[np.ndarray] = None   # W' per rank (Equation 4)

    @property
    def I(self) -> int:
        return int(self.inst_ptr[-1])


def plan_layer(expert_load: Sequence[float], groups: Sequence[Sequence[int]], nodes: int, gpus_per_node: int,
               weight_scale: int = 8, literal_eq4: bool = False) -> Plan:
    """groups[r] = experts whose primary instance lives on rank r (ranks are node-major).
    Replicates the hot experts of the heaviest group on the n_replica least-loaded other ranks
    (primaries stay), predicts the post-replication rank loads and derives integer polling weights
    inversely proportional to them.

    literal_eq4: W_p = W_max / (n_replica + 1) exactly as printed; otherwise the load that is
    actually split, W_p = W_r / (n_replica + 1) (the even split the text describes)."""
    load = np.asarray(expert_load, dtype=np.float64)
    E, R = load.shape[0], nodes * gpus_per_node
    if len(groups) != R:
        raise ValueError("one group per rank expected")
    seen = sorted(e for g in groups for e in g)
    if seen != list(range(E)):
        raise ValueError("groups must partition the experts")
    rank_node = (np.arange(R) // gpus_per_node).astype(np.int32)
    w = np.array([load[list(g)].sum() for g in groups], dtype=np.float64)
    hosts: List[List[int]] = [[] for _ in range(E)]
    for r, g in enumerate(groups):
        for e in g:
            hosts[e].append(r)
    heavy = int(np.argmax(w))                       # ties: lowest rank
    w_max, w_mean = float(w[heavy]), float(w.mean())
    n_rep = n_replica(w_max, w_mean, R) if R > 1 and w_mean > 0 else 0
    hot: List[int] = []
    targets: List[int] = []
    pred = w.copy()
    if n_rep > 0:
        hot = hot_experts(load, list(groups[heavy]), w_max, n_rep)
        others = [r for r in range(R) if r != heavy]
        targets = sorted(others, key=lambda r: (w[r], r))[:n_rep]   # the most under-utilised GPUs
        for e in hot:
            hosts[e].extend(targets)
        w_r = float(load[hot].sum())
        w_p = (w_max if literal_eq4 else w_r) / (n_rep + 1.0)
        pred[heavy] = w_max - w_r + w_p               # Equation 4
        for r in targets:
            pred[r] = w[r] + w_p
    pos = np.maximum(pred, 1e-12)
    pw = np.clip(np.rint(weight_scale * pos.min() / pos), 1, weight_scale).astype(np.uint32)
    inst_ptr = np.zeros(E + 1, dtype=np.int32)
    inst_rank: List[int] = []
    for e in range(E):
        inst_rank.extend(sorted(hosts[e]))
        inst_ptr[e + 1] = len(inst_rank)
    return Plan(E=E, R=R, N=nodes, rank_node=rank_node, poll_weight=pw, inst_ptr=inst_ptr,
                inst_rank=np.asarray(inst_rank, dtype=np.int32), hot=hot, n_replica=n_rep, targets=targets,
                predicted_load=pred)


def rank_load_std(rank_off: Sequence[int]) -> float:
    """Standard deviation of the rows per rank (the paper's load-balance metric, Section 6.1),
    from the rank offsets of grace_permute."""
    rows = np.diff(np.asarray(rank_off, dtype=np.float64))
    return float(rows.std())
