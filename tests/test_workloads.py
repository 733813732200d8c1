"""The synthetic generator: closed forms of the offline rules it borrows from
the paper, determinism, and validity of every table it emits."""
import numpy as np
import pytest

from workloads import CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_workload
from workloads.generator import eq3_n_replica, primary_group_sizes


def test_eq3_by_hand():
    # Equation 3: n_replica = min(max(1, floor(rho)), n_gpu - 1)
    assert eq3_n_replica(2.7, 1.0, 4) == 2
    assert eq3_n_replica(0.9, 1.0, 4) == 1
    assert eq3_n_replica(9.0, 1.0, 4) == 3


def test_group_sizes_stay_in_algorithm2_window():
    # Algorithm 2: E0 = floor(E/D), delta = max(1, round(E0 * r)); r = 0.15 (Appendix A.1)
    for E, R in ((64, 4), (60, 8), (8, 8), (64, 32), (8, 4)):
        e0 = E // R
        delta = max(1, round(e0 * 0.15))
        sizes = primary_group_sizes(E, R)
        assert sum(sizes) == E
        assert all(max(1, e0 - delta) <= s <= e0 + delta for s in sizes)
    assert primary_group_sizes(60, 8) == [8, 8, 8, 8, 7, 7, 7, 7]


def test_bf16_round_trip_and_rounding():
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e-39], np.float32)
    b = f32_to_bf16_bits(a)
    back = bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[3] == -2.5
    assert back[1] == 1.0            # 1 + 2^-8 is a tie -> even mantissa
    assert back[2] == np.float32(1.015625)   # 1 + 3*2^-8 is a tie -> rounds up to even
    np.testing.assert_array_equal(f32_to_bf16_bits(back), b)


@pytest.mark.parametrize("name", list(CONFIGS))
def test_tables_are_valid_and_deterministic(name):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=min(cfg.T, 512))
    wl2 = make_workload(cfg, T=min(cfg.T, 512))
    np.testing.assert_array_equal(wl.logits, wl2.logits)
    np.testing.assert_array_equal(wl.x, wl2.x)
    pl = wl.placement
    np.testing.assert_array_equal(pl.inst_rank, wl2.placement.inst_rank)
    assert pl.R == cfg.nodes * cfg.gpus_per_node and pl.N == cfg.nodes
    assert (np.diff(pl.rank_node) >= 0).all()
    assert (pl.poll_weight >= 1).all() and (pl.poll_weight <= 8).all()
    for e in range(cfg.E):
        ranks = pl.inst_rank[pl.inst_ptr[e]:pl.inst_ptr[e + 1]]
        assert len(ranks) >= 1 and (np.diff(ranks) > 0).all()
        assert ranks.min() >= 0 and ranks.max() < pl.R
    assert len(pl.hot) == cfg.n_hot
    for e in pl.hot:
        n_inst = pl.inst_ptr[e + 1] - pl.inst_ptr[e]
        if cfg.replica_mode == "all":
            assert n_inst == pl.R
        elif cfg.replica_mode == "per_node":
            nodes = set(pl.rank_node[pl.inst_rank[pl.inst_ptr[e]:pl.inst_ptr[e + 1]]].tolist())
            assert nodes == set(range(pl.N))
        else:
            assert n_inst >= 2
    if cfg.d * cfg.f > 4 << 20:
        return
    wg, wu, wd = wl.expert_weights(0)
    assert wg.shape == (cfg.f, cfg.d) and wu.shape == (cfg.f, cfg.d) and wd.shape == (cfg.d, cfg.f)
