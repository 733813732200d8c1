"""Offline planner: Equation 3, the hot-set threshold, Equation 4 and Algorithm 2's window by hand;
every plan is a valid table; replication with locality-first routing flattens the rank loads."""
import numpy as np
import pytest

import oracle
import paper_2509_25041_amd as grace
from paper_2509_25041_amd import planner
from workloads import CONFIGS, make_workload


def test_closed_forms_by_hand():
    assert planner.n_replica(2.7, 1.0, 4) == 2 and planner.n_replica(0.9, 1.0, 4) == 1
    assert planner.n_replica(9.0, 1.0, 4) == 3
    assert planner.group_size_window(64, 4, 0.15) == (14, 18)       # E=16, delta=round(2.4)=2
    assert planner.group_size_window(60, 8, 0.15) == (6, 8)         # E=7, delta=max(1, round(1.05))=1
    # heaviest group loads 50, 30, 15, 5 (W_max = 100), n_replica = 2: threshold 66.7 -> the first two
    loads = {0: 50.0, 1: 30.0, 2: 15.0, 3: 5.0}
    assert planner.hot_experts(loads, [3, 1, 0, 2], 100.0, 2) == [0, 1]
    # threshold 50 is met exactly by the first expert: "exceeds" is strict, so the second one is hot as well
    assert planner.hot_experts(loads, [0, 1, 2, 3], 100.0, 1) == [0, 1]
    assert planner.hot_experts({0: 51.0, 1: 29.0, 2: 15.0, 3: 5.0}, [0, 1, 2, 3], 100.0, 1) == [0]   # 51 > 50 at once
    assert planner.hot_experts({0: 10.0, 1: 10.0}, [1, 0], 20.0, 3) == [0, 1]  # ties: lower id first


def test_equation_3_agrees_with_the_input_generator():
    """The workload generator applies Equation 3 when it lays out config 4's table (input data for both
    the HIP path and the oracle, so it cannot import the planner); the two must be the same function."""
    from workloads.generator import eq3_n_replica
    for n_gpu in (2, 4, 8, 32):
        for rho in (0.3, 0.99, 1.0, 1.5, 2.0, 2.7, 7.9, 8.0, 31.0, 40.0):
            assert planner.n_replica(rho * 3.0, 3.0, n_gpu) == eq3_n_replica(rho * 3.0, 3.0, n_gpu)


def test_plan_by_hand():
    # 1 node x 4 GPUs, 8 experts, two per rank; rank 0 holds the hot pair
    load = np.array([50, 30, 5, 5, 4, 3, 2, 1], dtype=float)     # group loads 80, 10, 7, 3 ; mean 25
    groups = [[0, 1], [2, 3], [4, 5], [6, 7]]
    p = planner.plan_layer(load, groups, nodes=1, gpus_per_node=4)
    assert p.n_replica == 3                                       # floor(80/25)=3, cap n_gpu-1=3
    assert p.hot == [0, 1]                                        # threshold 80*3/4 = 60: 50, then 80
    assert p.targets == [3, 2, 1]                                 # least loaded first
    # Equation 4 with W_r = 80: W_p = 20; W'_max = 80 - 80 + 20; W'_i = W_i + 20
    np.testing.assert_allclose(p.predicted_load, [20.0, 30.0, 27.0, 23.0])
    assert p.poll_weight.tolist() == [8, 5, 6, 7]                 # round(8 * 20 / W')
    assert p.inst_ptr.tolist() == [0, 4, 8, 9, 10, 11, 12, 13, 14]
    assert p.inst_rank.tolist() == [0, 1, 2, 3, 0, 1, 2, 3, 1, 1, 2, 2, 3, 3]
    lit = planner.plan_layer(load, groups, nodes=1, gpus_per_node=4, literal_eq4=True)
    np.testing.assert_allclose(lit.predicted_load, [20.0, 30.0, 27.0, 23.0])     # W_r == W_max here
    load2 = np.array([50, 30, 10, 5, 4, 3, 2, 1], dtype=float)
    groups2 = [[0, 1, 2], [3], [4, 5], [6, 7]]                   # W = 90, 5, 7, 3 ; mean 26.25 -> n_rep 3
    a = planner.plan_layer(load2, groups2, 1, 4)
    b = planner.plan_layer(load2, groups2, 1, 4, literal_eq4=True)
    assert a.hot == [0, 1]                                        # threshold 67.5
    np.testing.assert_allclose(a.predicted_load, [90 - 80 + 20, 25, 27, 23])
    np.testing.assert_allclose(b.predicted_load, [90 - 80 + 22.5, 27.5, 29.5, 25.5])


@pytest.mark.parametrize("name", ["olmoe", "qwen", "dsv2lite"])
def test_plans_are_valid_tables_and_flatten_load(name):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=min(cfg.T, 2048))
    base = wl.placement
    R = cfg.R
    sizes = np.diff(np.linspace(0, cfg.E, R + 1).astype(int))
    groups, e = [], 0
    for s in sizes:
        groups.append(list(range(e, e + s)))
        e += s
    plan = planner.plan_layer(base.profile_load, groups, cfg.nodes, cfg.gpus_per_node)
    grace.grace_table_validate(plan.E, plan.R, plan.N, plan.rank_node, plan.poll_weight, plan.inst_ptr, plan.inst_rank)
    assert plan.n_replica >= 1 and len(plan.hot) >= 1
    # the same table without the replicas
    noreps = planner.Plan(E=plan.E, R=R, N=plan.N, rank_node=plan.rank_node, poll_weight=np.ones(R, np.uint32),
                          inst_ptr=np.arange(plan.E + 1, dtype=np.int32),
                          inst_rank=np.array([r for r, g in enumerate(groups) for _ in g], np.int32))
    heavy = int(np.argmax([base.profile_load[g].sum() for g in groups]))
    # routed from a rank that holds no replica: the replicas take load off the heaviest rank
    src = [r for r in range(R) if r != heavy and r not in plan.targets]
    lr = src[0] if src else (heavy + 1) % R
    before = oracle.route_permute(wl.logits, noreps, cfg.k, lr, policy=1).perm.rank_off
    after = oracle.route_permute(wl.logits, plan, cfg.k, lr, policy=1).perm.rank_off
    rows_before, rows_after = np.diff(before), np.diff(after)
    assert rows_after[heavy] < rows_before[heavy]
    assert planner.rank_load_std(after) < planner.rank_load_std(before)
