"""grace_route_permute_static (the entry point for callers that cannot allocate: its scratch is a
static device array) against grace_route_permute, through the C ABI: two calls in a row on the
same GPU, the second with a smaller input, every output bit for bit; sizes beyond the static
array are rejected with a clear error."""
import numpy as np
import pytest
import torch

import paper_2509_25041_amd as grace
from workloads import CONFIGS, LayerConfig, make_workload

pytestmark = pytest.mark.gpu


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def same(a, b):
    if a is None or b is None:
        return a is None and b is None
    if a.dtype == torch.bfloat16:
        a, b = a.view(torch.int16), b.view(torch.int16)
    if a.dtype == torch.float32:
        a, b = a.view(torch.int32), b.view(torch.int32)
    return torch.equal(a, b)


def run_both(table, cfg, wl, local_rank, rr_in=None, policy=0):
    logits, x = dev(wl.logits), dev(wl.x)
    T = wl.logits.shape[0]
    rin = None if rr_in is None else torch.from_numpy(rr_in.view(np.int32)).cuda()
    rout_a = torch.empty(cfg.E, dtype=torch.int32, device="cuda")
    rout_b = torch.empty(cfg.E, dtype=torch.int32, device="cuda")
    ref = grace.grace_route_permute(table, local_rank, logits, cfg.k, x, 1, rin, rout_a, policy=policy)
    got = grace.grace_route_permute_static(table, local_rank, logits, cfg.k, x, 1, rin, rout_b, policy=policy)
    torch.cuda.synchronize()
    names = ("topk_expert", "topk_weight", "topk_inst", "expert_count", "perm_pos", "perm_src", "inst_off", "rank_off",
             "node_off", "xp")
    for nm, a, b in zip(names, ref[0] + ref[1], got[0] + got[1]):
        assert same(a, b), f"T={T}: {nm} differs"
    assert torch.equal(rout_a, rout_b)
    assert int(got[1][2][-1]) == T * cfg.k


@pytest.mark.parametrize("name,sizes,local_rank", [
    ("olmoe", (4096, 1500), 0),          # larger batches: top-k, pick (+ permutation histograms), positions, scatter
    ("dsv2lite", (32768, 5000), 9),      # the largest config (2.3 MB of the 4 MiB array), then a smaller call
    ("olmoe_decode512", (512, 64), 0),   # decode-sized: the single-workgroup index kernel
    ("tiny", (256, 1), 2),               # fp32 rows
])
def test_static_scratch_matches_workspace_two_calls_in_a_row(name, sizes, local_rank):
    cfg = CONFIGS[name]
    table = grace.GraceTable.from_placement(make_workload(cfg, T=16).placement)
    rr = np.random.default_rng(1).integers(0, 2 ** 32, size=cfg.E, dtype=np.uint64).astype(np.uint32)
    for i, T in enumerate(sizes):        # the second, smaller call finds the first call's histograms in the scratch
        wl = make_workload(cfg, T=T)
        run_both(table, cfg, wl, local_rank, rr_in=rr if i else None, policy=i if name == "olmoe" else 0)


def test_static_scratch_rejects_sizes_beyond_the_array():
    cfg = LayerConfig("too_large", T=100000, E=128, k=8, d=8, f=16, dtype="f32", zipf_s=1.2, nodes=2, gpus_per_node=4,
                      n_hot=8, replica_mode="per_node", seed=41)
    wl = make_workload(cfg)
    table = grace.GraceTable.from_placement(wl.placement)
    logits, x = dev(wl.logits), dev(wl.x)
    with pytest.raises(grace.GraceError) as ei:
        grace.grace_route_permute_static(table, 0, logits, cfg.k, x)
    assert ei.value.status == -2 and "static buffer" in str(ei.value)
    # the workspace form takes the same call
    (te, tw, ti, cnt), perm = grace.grace_route_permute(table, 0, logits, cfg.k, x)
    torch.cuda.synchronize()
    assert int(perm[2][-1]) == cfg.T * cfg.k
