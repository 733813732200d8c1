"""Seeded workload and placement-table generator.

Stands in for the routing traces the paper profiles on its datasets
(Section 6.1): per-expert logit biases follow a Zipf law so a few experts are
hot and most are cold (Section 1, Figure 3), and the expert placement table has
the shape the paper's offline phase emits (Section 4.1 hierarchical grouping:
node -> GPU -> expert list; Section 4.2 replicas of hot experts; Section 4.3
polling weights inversely proportional to predicted GPU load).

Nothing here computes any part of the MoE layer.  "Profiled" expert loads are
random draws (k distinct experts per profiling token, sampled without
replacement from the Zipf mass), not the output of a gating function.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------
# bf16 storage helpers (bit-level; inputs are produced once and handed to both
# the oracle and the GPU library as the same uint16 arrays)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bits (uint16) to the fp32 values they denote."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int                 # tokens resident on local_rank
    E: int                 # routed experts
    k: int                 # top-k
    d: int                 # d_model
    f: int                 # d_ff of one expert
    dtype: str             # "f32" | "bf16" (storage of x and weights)
    zipf_s: float          # exponent of the per-expert logit bias
    nodes: int             # virtual nodes N
    gpus_per_node: int     # virtual GPUs per node G (R = N * G ranks)
    n_hot: int             # number of hot experts that get replicas
    replica_mode: str      # "all" | "per_node" | "eq3"
    n_shared: int = 0      # always-on shared experts
    drift_block: int = 0   # >0: hotness permutation redrawn every this many tokens
    seed: int = 0
    local_rank: int = 0
    renorm: int = 1

    @property
    def R(self) -> int:
        return self.nodes * self.gpus_per_node


CONFIGS: Dict[str, LayerConfig] = {
    # BASELINE configs[0..4]
    "tiny": LayerConfig("tiny", T=256, E=8, k=2, d=128, f=256, dtype="f32", zipf_s=1.2,
                        nodes=2, gpus_per_node=2, n_hot=1, replica_mode="all", seed=0),
    "olmoe": LayerConfig("olmoe", T=4096, E=64, k=8, d=2048, f=1024, dtype="bf16", zipf_s=1.2,
                         nodes=2, gpus_per_node=2, n_hot=4, replica_mode="all", seed=1),
    "mixtral": LayerConfig("mixtral", T=8192, E=8, k=2, d=4096, f=14336, dtype="bf16", zipf_s=0.8,
                           nodes=2, gpus_per_node=4, n_hot=2, replica_mode="per_node", seed=2),
    "qwen": LayerConfig("qwen", T=16384, E=60, k=4, d=2048, f=1408, dtype="bf16", zipf_s=1.5,
                        nodes=4, gpus_per_node=2, n_hot=6, replica_mode="eq3", n_shared=4, seed=3),
    # decode-shaped steps (Section 6.1 workloads: batch 256 / 512 over 4-8 GPUs per decode step;
    # Appendix A.4: lighter batches 64 / 128): a few dozen to a few hundred tokens per rank
    "olmoe_decode64": LayerConfig("olmoe_decode64", T=64, E=64, k=8, d=2048, f=1024, dtype="bf16", zipf_s=1.2,
                                  nodes=2, gpus_per_node=2, n_hot=4, replica_mode="all", seed=5),
    "olmoe_decode512": LayerConfig("olmoe_decode512", T=512, E=64, k=8, d=2048, f=1024, dtype="bf16", zipf_s=1.2,
                                   nodes=2, gpus_per_node=2, n_hot=4, replica_mode="all", seed=6),
    # the paper's third model shape (Section 6.1: 128 experts, top-8): two experts per lane in the
    # wavefront top-k; 16 primaries per rank on 2 x 4 ranks, 8 hot experts replicated per node
    "qwen3moe": LayerConfig("qwen3moe", T=8192, E=128, k=8, d=2048, f=768, dtype="bf16", zipf_s=1.2,
                            nodes=2, gpus_per_node=4, n_hot=8, replica_mode="per_node", seed=7),
    "dsv2lite": LayerConfig("dsv2lite", T=32768, E=64, k=6, d=2048, f=1408, dtype="bf16", zipf_s=1.2,
                            nodes=4, gpus_per_node=8, n_hot=8, replica_mode="per_node", n_shared=2,
                            drift_block=4096, seed=4),
}


@dataclass
class Placement:
    """Placement / replica table (Sections 4.1-4.3) as plain host arrays.

    CSR over experts: the instances of expert e live on ranks
    inst_rank[inst_ptr[e] : inst_ptr[e+1]] (strictly ascending).
    """
    E: int
    R: int
    N: int
    rank_node: np.ndarray    # int32 [R], non-decreasing
    poll_weight: np.ndarray  # uint32 [R], >= 1
    inst_ptr: np.ndarray     # int32 [E+1]
    inst_rank: np.ndarray    # int32 [I]
    profile_load: np.ndarray = field(default_factory=lambda: np.zeros(0))
    hot: List[int] = field(default_factory=list)

    @property
    def I(self) -> int:
        return int(self.inst_ptr[-1])

    def experts_on(self, rank: int) -> List[int]:
        out = []
        for e in range(self.E):
            if rank in self.inst_rank[self.inst_ptr[e]:self.inst_ptr[e + 1]]:
                out.append(e)
        return out


def _zipf_bias(rng: np.random.Generator, E: int, s: float) -> Tuple[np.ndarray, np.ndarray]:
    """Hotness rank is a seeded permutation; bias_e = -s * ln(rank_e)."""
    perm = rng.permutation(E)
    rank = np.empty(E, dtype=np.int64)
    rank[perm] = np.arange(1, E + 1)
    return (-s * np.log(rank.astype(np.float64))).astype(np.float32), rank


def _profile_load(rng: np.random.Generator, rank: np.ndarray, s: float, k: int, n_tokens: int) -> np.ndarray:
    """Token counts per expert over a synthetic profiling batch (footnote of
    Section 1: load = number of tokens assigned).  Each profiling token draws k
    distinct experts without replacement with probability proportional to the
    Zipf mass rank^-s."""
    E = rank.shape[0]
    p = rank.astype(np.float64) ** (-s)
    p /= p.sum()
    load = np.zeros(E, dtype=np.int64)
    for _ in range(n_tokens):
        load[rng.choice(E, size=k, replace=False, p=p)] += 1
    return load


def primary_group_sizes(E: int, R: int) -> List[int]:
    """Contiguous primary groups.  Equal sizes when R divides E; otherwise sizes
    E0+1 for the first (E mod R) ranks and E0 for the rest, which stays inside
    the size window of the controlled non-uniform grouping (Algorithm 2:
    E0 = floor(E/R), delta = max(1, round(E0 * r)), sizes in [E0-delta, E0+delta])."""
    e0, rem = divmod(E, R)
    return [e0 + 1 if r < rem else e0 for r in range(R)]


def eq3_n_replica(w_max: float, w_mean: float, n_gpu: int) -> int:
    """Number of replicas from the load-skew factor rho = W_max / W_mean
    (Equation 3)."""
    rho = w_max / w_mean
    return int(min(max(1, int(np.floor(rho))), n_gpu - 1))


def make_placement(cfg: LayerConfig, profile_load: np.ndarray) -> Placement:
    E, R, N, G = cfg.E, cfg.R, cfg.nodes, cfg.gpus_per_node
    rank_node = (np.arange(R) // G).astype(np.int32)
    load = profile_load.astype(np.float64)

    hosts: List[List[int]] = [[] for _ in range(E)]   # ranks hosting each expert
    sizes = primary_group_sizes(E, R)
    e = 0
    for r, sz in enumerate(sizes):
        for _ in range(sz):
            hosts[e].append(r)
            e += 1
    assert e == E

    def rank_loads() -> np.ndarray:
        w = np.zeros(R, dtype=np.float64)
        for ee in range(E):
            for r in hosts[ee]:
                w[r] += load[ee] / len(hosts[ee])
        return w

    # hot set: largest profiled load, ties to the lower id
    order = sorted(range(E), key=lambda ee: (-load[ee], ee))
    hot = order[:cfg.n_hot]

    if cfg.replica_mode == "all":
        # one instance on every GPU (Section 4.2, Figure 1b; Equation 3 at its cap)
        for ee in hot:
            hosts[ee] = list(range(R))
    elif cfg.replica_mode == "per_node":
        # one instance in every node that lacks one, on that node's least-loaded rank
        for ee in hot:
            for n in range(N):
                if any(rank_node[r] == n for r in hosts[ee]):
                    continue
                w = rank_loads()
                cands = [r for r in range(R) if rank_node[r] == n]
                tgt = min(cands, key=lambda r: (w[r], r))
                hosts[ee].append(tgt)
    elif cfg.replica_mode == "eq3":
        # Equation 3 on the primary groups' loads; copies go to the least-loaded
        # ranks not yet hosting the expert (Section 4.2)
        w0 = rank_loads()
        n_rep = eq3_n_replica(float(w0.max()), float(w0.mean()), R)
        for ee in hot:
            for _ in range(n_rep):
                w = rank_loads()
                cands = [r for r in range(R) if r not in hosts[ee]]
                if not cands:
                    break
                tgt = min(cands, key=lambda r: (w[r], r))
                hosts[ee].append(tgt)
    else:
        raise ValueError(cfg.replica_mode)

    # predicted post-replication rank load (even split of each expert's own
    # load over its instances - the idea behind Equation 4), then integer
    # polling weights inversely proportional to it (Section 4.3)
    w = rank_loads()
    w = np.maximum(w, 1e-9)
    pw = np.clip(np.rint(8.0 * w.min() / w), 1, 8).astype(np.uint32)

    inst_ptr = np.zeros(E + 1, dtype=np.int32)
    inst_rank: List[int] = []
    for ee in range(E):
        rs = sorted(hosts[ee])
        inst_rank.extend(rs)
        inst_ptr[ee + 1] = len(inst_rank)
    return Placement(E=E, R=R, N=N, rank_node=rank_node, poll_weight=pw, inst_ptr=inst_ptr,
                     inst_rank=np.asarray(inst_rank, dtype=np.int32),
                     profile_load=profile_load.copy(), hot=list(hot))


@dataclass
class Workload:
    cfg: LayerConfig
    placement: Placement
    logits: np.ndarray          # float32 [T, E]
    x: np.ndarray               # float32 [T, d] (f32) or uint16 bf16 bits [T, d]

    def _store(self, a: np.ndarray) -> np.ndarray:
        return a if self.cfg.dtype == "f32" else f32_to_bf16_bits(a)

    def expert_weights(self, e: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """(w_gate [f,d], w_up [f,d], w_down [d,f]) of routed expert e in the
        storage dtype; each row holds one output feature, contiguous over the
        input feature.  Seeded per expert so any subset can be drawn."""
        c = self.cfg
        rng = np.random.default_rng([c.seed, 7001, e])
        wg = rng.standard_normal((c.f, c.d), dtype=np.float32) * np.float32(0.02)
        wu = rng.standard_normal((c.f, c.d), dtype=np.float32) * np.float32(0.02)
        wd = rng.standard_normal((c.d, c.f), dtype=np.float32) * np.float32(0.02)
        return self._store(wg), self._store(wu), self._store(wd)

    def stacked_weights(self, experts: List[int]):
        """Weights of the given experts stacked along a leading slot axis."""
        ws = [self.expert_weights(e) for e in experts]
        if not ws:
            c = self.cfg
            z = np.uint16 if c.dtype == "bf16" else np.float32
            return (np.zeros((0, c.f, c.d), z), np.zeros((0, c.f, c.d), z), np.zeros((0, c.d, c.f), z))
        return tuple(np.stack([w[i] for w in ws]) for i in range(3))

    def shared_weights(self) -> Optional[Tuple[np.ndarray, np.ndarray, np.ndarray]]:
        """(w_gate [n_shared,f,d], w_up [n_shared,f,d], w_down [n_shared,d,f])."""
        c = self.cfg
        if c.n_shared == 0:
            return None
        out = []
        for s in range(c.n_shared):
            rng = np.random.default_rng([c.seed, 9001, s])
            wg = rng.standard_normal((c.f, c.d), dtype=np.float32) * np.float32(0.02)
            wu = rng.standard_normal((c.f, c.d), dtype=np.float32) * np.float32(0.02)
            wd = rng.standard_normal((c.d, c.f), dtype=np.float32) * np.float32(0.02)
            out.append((self._store(wg), self._store(wu), self._store(wd)))
        return tuple(np.stack([w[i] for w in out]) for i in range(3))


def make_workload(cfg: LayerConfig, T: Optional[int] = None) -> Workload:
    """Draw logits, tokens and the placement table of one layer call."""
    if T is not None and T != cfg.T:
        cfg = LayerConfig(**{**cfg.__dict__, "T": T})
    rng = np.random.default_rng([cfg.seed, 1])
    block = cfg.drift_block if cfg.drift_block > 0 else max(cfg.T, 1)
    n_blocks = max(1, -(-cfg.T // block))
    logits = np.empty((cfg.T, cfg.E), dtype=np.float32)
    rank0 = None
    for b in range(n_blocks):
        bias, rank = _zipf_bias(rng, cfg.E, cfg.zipf_s)
        if b == 0:
            rank0 = rank
        lo, hi = b * block, min(cfg.T, (b + 1) * block)
        logits[lo:hi] = rng.standard_normal((hi - lo, cfg.E), dtype=np.float32) + bias[None, :]
    x = rng.standard_normal((cfg.T, cfg.d), dtype=np.float32)
    if cfg.dtype == "bf16":
        x = f32_to_bf16_bits(x)
    # offline "profile": the placement only ever sees block 0's hotness
    prng = np.random.default_rng([cfg.seed, 1000])
    load = _profile_load(prng, rank0, cfg.zipf_s, cfg.k, n_tokens=min(max(cfg.T, 256), 4096))
    return Workload(cfg=cfg, placement=make_placement(cfg, load), logits=logits, x=x)
