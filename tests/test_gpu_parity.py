"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same
seeded inputs.  Integer outputs bit-exact; gate weights within 1e-6 relative;
FFN / combine outputs within 2e-2 (bf16) / 1e-5 (fp32) by the metric
max |y - r| / max(|r|, rms(r))."""
import os
import sys
from types import SimpleNamespace

import numpy as np
import pytest
import torch

import oracle
import paper_2509_25041_amd as grace
from workloads import CONFIGS, LayerConfig, make_workload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    ref = ref.astype(np.float64)
    got = got.astype(np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def rel_err_rows(got: np.ndarray, ref: np.ndarray) -> float:
    """The same metric with the floor taken per row: max |y - r| / max(|r|, rms(row of r)).  For
    tensors whose rows differ in scale (the rank share of the combine output: a row is the sum over
    the token's LOCAL experts only, weighted by their gates, so rows range from one small-gate term to
    the whole token) the tensor-wide rms is no scale for the elements of a large row.  All-zero
    reference rows must be matched exactly."""
    ref = ref.astype(np.float64)
    got = got.astype(np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    zero = (rms[:, 0] == 0.0)
    if zero.any() and np.any(got[zero] != 0.0):
        return float("inf")
    den = np.maximum(np.abs(ref), np.maximum(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def dev(a: np.ndarray, dtype: str = None) -> torch.Tensor:
    """host array -> device tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a device"
    grace.load_library()


def run_route_permute(wl, pl, k, local_rank, rr_in=None, renorm=1, with_rows=True, policy=0, fold_limits=None):
    table = grace.GraceTable.from_placement(pl)
    if fold_limits is not None:
        table.set_fold_limits(*fold_limits)
    logits = dev(wl.logits)
    rin = None if rr_in is None else torch.from_numpy(rr_in.view(np.int32)).cuda()
    rout = torch.empty(pl.E, dtype=torch.int32, device="cuda")
    te, tw, ti, cnt = grace.grace_route(table, local_rank, logits, k, renorm, rin, rout, policy=policy)
    x = dev(wl.x) if with_rows else None
    pos, src, ioff, roff, noff, xp = grace.grace_permute(table, ti, x)
    torch.cuda.synchronize()
    return table, SimpleNamespace(te=te, tw=tw, ti=ti, cnt=cnt, rout=rout, pos=pos, src=src, ioff=ioff, roff=roff,
                                  noff=noff, xp=xp, x=x)


def check_route_permute(g, ref, wl, k):
    np.testing.assert_array_equal(host(g.te), ref.topk_expert)
    np.testing.assert_array_equal(host(g.ti), ref.topk_inst)
    np.testing.assert_array_equal(host(g.cnt), ref.expert_count)
    np.testing.assert_array_equal(host(g.rout).view(np.uint32), ref.rr_out)
    np.testing.assert_allclose(host(g.tw), ref.topk_weight, rtol=1e-6, atol=0)
    np.testing.assert_array_equal(host(g.pos), ref.perm.perm_pos)
    np.testing.assert_array_equal(host(g.src), ref.perm.perm_src)
    np.testing.assert_array_equal(host(g.ioff), ref.perm.inst_off)
    np.testing.assert_array_equal(host(g.roff), ref.perm.rank_off)
    np.testing.assert_array_equal(host(g.noff), ref.perm.node_off)
    if g.xp is not None:
        np.testing.assert_array_equal(host(g.xp), oracle.gather_rows(wl.x, ref.perm.perm_src, k))


# ------------------------------------------------------- routing + permutation --
@pytest.mark.parametrize("name,T,local_rank", [
    ("tiny", None, 0), ("tiny", None, 3), ("tiny", 1, 1), ("tiny", 63, 2), ("tiny", 65, 0), ("tiny", 1000, 1),
    ("olmoe", None, 0), ("olmoe", 777, 2),
    ("mixtral", 2048, 0), ("mixtral", 2048, 5),
    ("qwen", None, 0), ("qwen", 3001, 7),
    ("dsv2lite", None, 0), ("dsv2lite", 5000, 17),
    ("qwen3moe", None, 0), ("qwen3moe", 1111, 6),
])
def test_route_and_permute_bit_exact(name, T, local_rank):
    cfg = CONFIGS[name]
    with_rows = (T or cfg.T) * cfg.k * cfg.d <= 2 ** 27      # full-size rows are covered by the layer tests
    wl = make_workload(cfg, T=T)
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, local_rank)
    _, g = run_route_permute(wl, wl.placement, cfg.k, local_rank, with_rows=with_rows)
    check_route_permute(g, ref, wl, cfg.k)


@pytest.mark.parametrize("limits", [(-1, -1), (1 << 30, -1), (0, -1), (0, 0)])
def test_route_and_permute_many_chunks_every_prefix_algorithm(limits):
    """50 000 tokens (1563 routing chunks, 782 permutation chunks) through each way of turning the
    chunk histograms into prefix counts: the defaults (two-level sums at this size), one-level sums
    forced (every block adds thousands of rows), two-level forced, and the single-block scan kernels.
    Separate calls, the one-call dispatch and the send lists, all bit-exact."""
    cfg = LayerConfig("many_chunks", T=50000, E=128, k=8, d=8, f=16, dtype="f32", zipf_s=1.2, nodes=2,
                      gpus_per_node=4, n_hot=8, replica_mode="per_node", seed=31)
    wl = make_workload(cfg)
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, 3)
    sl = oracle.send_lists(ref.topk_inst, wl.placement, 3)
    table, g = run_route_permute(wl, wl.placement, cfg.k, 3, fold_limits=limits)     # the limits belong to the table
    check_route_permute(g, ref, wl, cfg.k)
    check_route_permute(run_fused(wl, wl.placement, cfg.k, 3, fold_limits=limits), ref, wl, cfg.k)   # the same as one call
    rp, rt, np_, nt, ex, tr = grace.grace_send_lists(table, 3, g.ti)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(rp), sl.rank_send_ptr)
    np.testing.assert_array_equal(host(rt)[:sl.rank_send_ptr[-1]], sl.rank_send_tok)
    np.testing.assert_array_equal(host(nt)[:sl.node_send_ptr[-1]], sl.node_send_tok)
    np.testing.assert_array_equal(host(ex), sl.expand)
    np.testing.assert_array_equal(host(tr), sl.traffic)


def test_route_rr_carry_and_no_renorm():
    cfg = CONFIGS["dsv2lite"]
    wl = make_workload(cfg, T=3000)
    rr_in = np.random.default_rng(5).integers(0, 2 ** 32, size=cfg.E, dtype=np.uint64).astype(np.uint32)
    rr_in[:8] = [0, 1, 2, 3, 4, 5, 2 ** 32 - 1, 2 ** 31]
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, 9, renorm=0, rr_in=rr_in)
    _, g = run_route_permute(wl, wl.placement, cfg.k, 9, rr_in=rr_in, renorm=0, with_rows=False)
    check_route_permute(g, ref, wl, cfg.k)


@pytest.mark.parametrize("name,local_rank", [("olmoe", 0), ("dsv2lite", 21), ("mixtral", 6)])
def test_route_wrr_policy_without_locality(name, local_rank):
    """The paper's first policy (weighted round-robin over all instances): bit-exact, and
    independent of the source rank."""
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=min(cfg.T, 6000))
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, local_rank, policy=1)
    _, g = run_route_permute(wl, wl.placement, cfg.k, local_rank, with_rows=False, policy=grace.GRACE_POLICY_WRR)
    check_route_permute(g, ref, wl, cfg.k)
    _, g0 = run_route_permute(wl, wl.placement, cfg.k, 0, with_rows=False, policy=grace.GRACE_POLICY_WRR)
    np.testing.assert_array_equal(host(g0.ti), host(g.ti))


@pytest.mark.parametrize("name,T,local_rank", [("tiny", None, 0), ("tiny", 1, 2), ("olmoe", None, 0), ("qwen", 3001, 5),
                                               ("dsv2lite", None, 0), ("dsv2lite", 5000, 13), ("mixtral", 2048, 6)])
def test_send_lists_bit_exact(name, T, local_rank):
    """De-duplicated per-rank / per-node send lists, expansion map and traffic counters."""
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=T)
    pl = wl.placement
    ref = oracle.route_permute(wl.logits, pl, cfg.k, local_rank)
    sl = oracle.send_lists(ref.topk_inst, pl, local_rank, ref.order)
    table = grace.GraceTable.from_placement(pl)
    te, tw, ti, cnt = grace.grace_route(table, local_rank, dev(wl.logits), cfg.k)
    rp, rt, np_, nt, ex, tr = grace.grace_send_lists(table, local_rank, ti)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(rp), sl.rank_send_ptr)
    np.testing.assert_array_equal(host(rt)[:sl.rank_send_ptr[-1]], sl.rank_send_tok)
    np.testing.assert_array_equal(host(np_), sl.node_send_ptr)
    np.testing.assert_array_equal(host(nt)[:sl.node_send_ptr[-1]], sl.node_send_tok)
    np.testing.assert_array_equal(host(ex), sl.expand)
    np.testing.assert_array_equal(host(tr), sl.traffic)
    assert (host(rt)[sl.rank_send_ptr[-1]:] == -1).all()      # nothing written past the lists


@pytest.mark.parametrize("case", ["case_from_larger_node", "case_from_smaller_node"])
def test_send_lists_nodes_of_unequal_size_golden(case):
    """The hand-worked example with nodes of 2 and 3 ranks (stage-1 peer = own index modulo the other node's size)."""
    import json
    with open(os.path.join(os.path.dirname(__file__), "golden", "send_lists_unequal_nodes.json")) as fh:
        g = json.load(fh)
    c = g[case]
    table = grace.GraceTable(g["E"], g["R"], g["N"], g["rank_node"], g["poll_weight"], g["inst_ptr"], g["inst_rank"])
    ti = torch.tensor(c["topk_inst"], dtype=torch.int32, device="cuda")
    rp, rt, np_, nt, ex, tr = grace.grace_send_lists(table, c["local_rank"], ti)
    torch.cuda.synchronize()
    assert host(rp).tolist() == c["rank_send_ptr"] and host(rt)[:len(c["rank_send_tok"])].tolist() == c["rank_send_tok"]
    assert host(np_).tolist() == c["node_send_ptr"] and host(nt)[:len(c["node_send_tok"])].tolist() == c["node_send_tok"]
    assert host(ex).tolist() == c["expand"]
    assert host(tr).tolist() == c["traffic"]


def run_fused(wl, pl, k, local_rank, rr_in=None, renorm=1, with_rows=True, policy=0, fold_limits=None):
    table = grace.GraceTable.from_placement(pl)
    if fold_limits is not None:
        table.set_fold_limits(*fold_limits)
    rin = None if rr_in is None else torch.from_numpy(rr_in.view(np.int32)).cuda()
    rout = torch.empty(pl.E, dtype=torch.int32, device="cuda")
    x = dev(wl.x) if with_rows else None
    (te, tw, ti, cnt), (pos, src, ioff, roff, noff, xp) = grace.grace_route_permute(
        table, local_rank, dev(wl.logits), k, x, renorm, rin, rout, policy=policy)
    torch.cuda.synchronize()
    return SimpleNamespace(te=te, tw=tw, ti=ti, cnt=cnt, rout=rout, pos=pos, src=src, ioff=ioff, roff=roff, noff=noff,
                           xp=xp, x=x)


@pytest.mark.parametrize("name,T,local_rank", [
    ("tiny", None, 0), ("tiny", 1, 1), ("tiny", 15, 3), ("tiny", 17, 2), ("tiny", 2048, 0),   # 2048: single kernel at k=2
    ("olmoe_decode64", None, 0), ("olmoe_decode512", None, 0), ("olmoe", 100, 2), ("olmoe", 513, 1),
    ("qwen", 200, 5), ("dsv2lite", 300, 17), ("mixtral", 1000, 6),
    # larger batches: the pick kernel also fills the permutation's chunk histograms
    ("olmoe", None, 0), ("qwen", 5001, 5), ("dsv2lite", None, 17), ("mixtral", None, 6), ("qwen3moe", 3000, 3),
])
def test_route_permute_single_call_bit_exact(name, T, local_rank):
    """grace_route_permute gives the outputs of the two calls, on the single-workgroup path
    (decode-sized batches) and on the path for larger batches alike."""
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=T)
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, local_rank)
    g = run_fused(wl, wl.placement, cfg.k, local_rank)
    check_route_permute(g, ref, wl, cfg.k)


def test_route_permute_single_call_carry_policy_and_wide_experts():
    cfg = CONFIGS["dsv2lite"]
    wl = make_workload(cfg, T=400)
    rr_in = np.random.default_rng(7).integers(0, 2 ** 32, size=cfg.E, dtype=np.uint64).astype(np.uint32)
    rr_in[:4] = [0, 2 ** 32 - 1, 2 ** 31, 5]
    for policy in (0, 1):
        ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, 11, renorm=0, rr_in=rr_in, policy=policy)
        g = run_fused(wl, wl.placement, cfg.k, 11, rr_in=rr_in, renorm=0, with_rows=False, policy=policy)
        check_route_permute(g, ref, wl, cfg.k)
    # more than one expert per lane, heavy ties, an instance table that still fits the single kernel
    rng = np.random.default_rng(3)
    E, k, T, R = 150, 5, 333, 4
    hosts = [sorted(rng.choice(R, size=rng.integers(1, 3), replace=False).tolist()) for _ in range(E)]
    inst_ptr = np.concatenate([[0], np.cumsum([len(h) for h in hosts])]).astype(np.int32)
    assert inst_ptr[-1] <= 256
    pl = SimpleNamespace(E=E, R=R, N=2, rank_node=np.array([0, 0, 1, 1], np.int32),
                         poll_weight=rng.integers(1, 9, size=R).astype(np.uint32), inst_ptr=inst_ptr,
                         inst_rank=np.concatenate(hosts).astype(np.int32))
    logits = np.round(rng.standard_normal((T, E)) * 2).astype(np.float32) / 2
    wl2 = SimpleNamespace(logits=logits, x=rng.standard_normal((T, 8)).astype(np.float32))
    ref = oracle.route_permute(logits, pl, k, 1)
    g = run_fused(wl2, pl, k, 1)
    check_route_permute(g, ref, wl2, k)


@pytest.mark.parametrize("E,k,T", [(128, 8, 1500), (200, 5, 700), (256, 64, 300), (8, 8, 100), (3, 1, 129),
                                   (64, 20, 300), (40, 40, 200), (100, 50, 150), (128, 64, 90)])
def test_route_wide_and_degenerate_expert_counts(E, k, T):
    """More than one expert per lane (E > 64), k = E, k = 1, ties everywhere; small k takes the
    arg-max rounds of the top-k kernel, the last four cases (large k for their E) its
    rank-by-broadcast path."""
    rng = np.random.default_rng(E + k)
    R, N = 6, 3
    hosts = [sorted(rng.choice(R, size=rng.integers(1, 4), replace=False).tolist()) for _ in range(E)]
    inst_ptr = np.concatenate([[0], np.cumsum([len(h) for h in hosts])]).astype(np.int32)
    pl = SimpleNamespace(E=E, R=R, N=N, rank_node=np.array([0, 0, 1, 1, 2, 2], np.int32),
                         poll_weight=rng.integers(1, 9, size=R).astype(np.uint32), inst_ptr=inst_ptr,
                         inst_rank=np.concatenate(hosts).astype(np.int32))
    logits = np.round(rng.standard_normal((T, E)) * 2).astype(np.float32) / 2      # heavy ties
    logits[0, :] = 0.0
    logits[1, ::2] = -0.0
    logits[2, ::3] = -np.inf          # masked experts: never ahead of a finite logit, weight exactly 0
    logits[3, 1:] = -np.inf           # one finite logit: the other choices in expert order, weight 0
    wl = SimpleNamespace(logits=logits, x=rng.standard_normal((T, 8)).astype(np.float32))
    ref = oracle.route_permute(logits, pl, k, 2)
    _, g = run_route_permute(wl, pl, k, 2)
    check_route_permute(g, ref, wl, k)


@pytest.mark.parametrize("E,k,T,renorm", [(64, 6, 8193, 1), (96, 8, 9001, 0), (128, 8, 8500, 1), (256, 5, 8200, 0),
                                          (32, 2, 16500, 1), (64, 1, 17000, 0), (36, 3, 8300, 1), (200, 7, 8400, 1),
                                          (64, 8, 20001, 0), (256, 8, 16385, 1), (32, 4, 33000, 0)])
def test_route_large_batches_few_lanes_per_token(E, k, T, renorm):
    """Batches above 8192 tokens with k <= 8 and E >= 32 a multiple of 4 take the top-k kernel that gives
    each token four lanes: expert counts that leave lanes partly or wholly without experts, every
    list length (k up to 2, 4, 6, 8), both softmax normalisations, ragged last chunks of 32 and of 64
    tokens, ties everywhere (logits on a grid of halves, a row of zeros, a row mixing -0.0 and +0.0)."""
    rng = np.random.default_rng(1000 * E + k)
    R, N = 6, 3
    hosts = [sorted(rng.choice(R, size=rng.integers(1, 4), replace=False).tolist()) for _ in range(E)]
    inst_ptr = np.concatenate([[0], np.cumsum([len(h) for h in hosts])]).astype(np.int32)
    pl = SimpleNamespace(E=E, R=R, N=N, rank_node=np.array([0, 0, 1, 1, 2, 2], np.int32),
                         poll_weight=rng.integers(1, 9, size=R).astype(np.uint32), inst_ptr=inst_ptr,
                         inst_rank=np.concatenate(hosts).astype(np.int32))
    logits = np.round(rng.standard_normal((T, E)) * 2).astype(np.float32) / 2
    logits[T // 2:] += (rng.standard_normal((T - T // 2, E)) * 1e-3).astype(np.float32)   # second half: few ties
    logits[0, :] = 0.0
    logits[1, ::2] = -0.0
    logits[2, :] = -7.5
    logits[3, ::3] = -np.inf          # masked experts: never ahead of a finite logit, weight exactly 0
    logits[4, 5:] = -np.inf           # fewer finite logits than k <= 8 may ask for: the rest in expert order, weight 0
    logits[T - 1, 1:] = -np.inf
    wl = SimpleNamespace(logits=logits, x=rng.standard_normal((T, 8)).astype(np.float32))
    ref = oracle.route_permute(logits, pl, k, 4, renorm=renorm)
    _, g = run_route_permute(wl, pl, k, 4, renorm=renorm)
    check_route_permute(g, ref, wl, k)


def test_empty_call_and_argument_errors():
    cfg = CONFIGS["tiny"]
    wl = make_workload(cfg)
    pl = wl.placement
    table = grace.GraceTable.from_placement(pl)
    empty = torch.empty((0, cfg.E), dtype=torch.float32, device="cuda")
    rout = torch.full((cfg.E,), 7, dtype=torch.int32, device="cuda")
    rin = torch.arange(cfg.E, dtype=torch.int32, device="cuda")
    te, tw, ti, cnt = grace.grace_route(table, 0, empty, cfg.k, 1, rin, rout)
    pos, src, ioff, roff, noff, xp = grace.grace_permute(table, ti, torch.empty((0, cfg.d), device="cuda"))
    torch.cuda.synchronize()
    assert host(cnt).tolist() == [0] * cfg.E
    ref = oracle.route_permute(np.zeros((0, cfg.E), np.float32), pl, cfg.k, 0, rr_in=np.arange(cfg.E, dtype=np.uint32))
    np.testing.assert_array_equal(host(rout).view(np.uint32), ref.rr_out)
    assert host(ioff).tolist() == [0] * (pl.I + 1) and host(roff).tolist() == [0] * (pl.R + 1)
    assert host(noff).tolist() == [0] * (pl.N + 1)
    logits = dev(wl.logits)
    for bad in (dict(k=0), dict(k=cfg.E + 1), dict(local_rank=pl.R), dict(local_rank=-1)):
        a = {**dict(k=cfg.k, local_rank=0), **bad}
        with pytest.raises(grace.GraceError):
            grace.grace_route(table, a["local_rank"], logits, a["k"])
    with pytest.raises(grace.GraceError):      # the counter may not be updated in place
        grace.grace_route(table, 0, logits, cfg.k, 1, rin, rin)
    with pytest.raises(grace.GraceError):      # E of the logits differs from the table's
        grace.grace_route(table, 0, torch.zeros((4, cfg.E + 1), device="cuda"), 2)
    with pytest.raises(grace.GraceError):      # 12-byte rows
        grace.grace_permute(table, torch.zeros((4, cfg.k), dtype=torch.int32, device="cuda"),
                            torch.zeros((4, 3), device="cuda"))
    table.destroy()
    with pytest.raises(ValueError):
        grace.grace_route(table, 0, logits, cfg.k)


# ------------------------------------------------------------------- combine --
@pytest.mark.parametrize("name,T,shared", [("tiny", None, False), ("tiny", 77, True), ("olmoe", 512, False),
                                           ("qwen", 300, True)])
def test_combine_matches_oracle_and_identity_experts(name, T, shared):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=T)
    T = wl.logits.shape[0]
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, 0)
    _, g = run_route_permute(wl, wl.placement, cfg.k, 0)
    # identity experts: y = xp, sum_j w_j = 1  ->  out = x
    out = grace.grace_combine(g.xp, g.pos, g.tw)
    x64 = oracle.widen(wl.x)
    assert rel_err(oracle.widen(host(out)), x64) <= (1e-6 if cfg.dtype == "f32" else 2.0 ** -8)
    # arbitrary y, optional shared term, against the oracle on the same stored values
    rng = np.random.default_rng(1)
    y = rng.standard_normal((T * cfg.k, cfg.d)).astype(np.float32)
    ys = rng.standard_normal((T, cfg.d)).astype(np.float32)
    if cfg.dtype == "bf16":
        from workloads import f32_to_bf16_bits
        y, ys = f32_to_bf16_bits(y), f32_to_bf16_bits(ys)
    out = grace.grace_combine(dev(y), g.pos, g.tw, dev(ys) if shared else None)
    want = oracle.combine(oracle.widen(y), ref.perm.perm_pos, ref.topk_weight, oracle.widen(ys) if shared else None)
    tol = 1e-6 if cfg.dtype == "f32" else 2.0 ** -8     # one bf16 rounding of an fp32 sum
    assert rel_err(oracle.widen(host(out)), want) <= tol


# ----------------------------------------------------------------------- FFN --
def _weights64(wl):
    cache = {}

    def weights_of(e):
        if e not in cache:
            cache[e] = tuple(oracle.widen(w) for w in wl.expert_weights(e))
        return cache[e]
    return weights_of


def _stack_dev(wl, experts):
    return tuple(dev(w) for w in wl.stacked_weights(list(experts)))


SMALL = {
    "tiny": CONFIGS["tiny"],
    "bf16_small": LayerConfig("bf16_small", T=700, E=16, k=4, d=256, f=384, dtype="bf16", zipf_s=1.2, nodes=2,
                              gpus_per_node=2, n_hot=2, replica_mode="all", n_shared=2, seed=11),
    "bf16_ragged": LayerConfig("bf16_ragged", T=333, E=8, k=2, d=136, f=200, dtype="bf16", zipf_s=0.8, nodes=2,
                               gpus_per_node=3, n_hot=2, replica_mode="per_node", n_shared=1, seed=12),
    "f32_ragged": LayerConfig("f32_ragged", T=150, E=6, k=3, d=100, f=76, dtype="f32", zipf_s=1.0, nodes=1,
                              gpus_per_node=3, n_hot=1, replica_mode="eq3", n_shared=3, seed=13),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_whole_layer_every_rank_element_by_element(name):
    """grace_expert_ffn looped over all virtual ranks rebuilds the whole layer;
    every intermediate is compared with the oracle element by element."""
    cfg = SMALL[name]
    wl = make_workload(cfg)
    pl = wl.placement
    tol = TOL[cfg.dtype]
    ref = oracle.route_permute(wl.logits, pl, cfg.k, 1)
    table, g = run_route_permute(wl, pl, cfg.k, 1)
    check_route_permute(g, ref, wl, cfg.k)
    x64 = oracle.widen(wl.x)
    w64 = _weights64(wl)
    y = torch.zeros((cfg.T * cfg.k, cfg.d), dtype=g.xp.dtype, device="cuda")
    for r in range(pl.R):
        experts = table.local_experts(r)
        np.testing.assert_array_equal(experts, ref.order.g_expert[ref.order.rank_ptr[r]:ref.order.rank_ptr[r + 1]])
        wg, wu, wd = _stack_dev(wl, experts)
        before = y.clone()
        grace.grace_expert_ffn(table, r, g.xp, g.ioff, cfg.T, cfg.k, wg, wu, wd, y=y)
        torch.cuda.synchronize()
        lo, hi = int(ref.perm.rank_off[r]), int(ref.perm.rank_off[r + 1])
        mask = np.ones(cfg.T * cfg.k, bool)
        mask[lo:hi] = False
        np.testing.assert_array_equal(host(y)[mask], host(before)[mask])      # other ranks' rows untouched
        want = oracle.expert_ffn(ref, x64, cfg.k, [r], w64)
        assert rel_err(oracle.widen(host(y))[lo:hi], want[lo:hi]) <= tol, f"rank {r}"
    y_ref = oracle.expert_ffn(ref, x64, cfg.k, range(pl.R), w64)
    ys = ys_ref = None
    sh = wl.shared_weights()
    if sh is not None:
        ys = grace.grace_shared_ffn(g.x, *[dev(w) for w in sh])
        ys_ref = oracle.shared_ffn(x64, tuple(oracle.widen(w) for w in sh))
        assert rel_err(oracle.widen(host(ys)), ys_ref) <= tol
    out = grace.grace_combine(y, g.pos, g.tw, ys)
    out_ref = oracle.combine(y_ref, ref.perm.perm_pos, ref.topk_weight, ys_ref)
    assert rel_err(oracle.widen(host(out)), out_ref) <= tol


def test_many_tiles_per_workgroup_element_by_element():
    """More output tiles than compute units, ragged segments: every persistent workgroup walks
    several tiles (tile switches, partial tiles, idle wavefronts); one rank's share, every element."""
    cfg = LayerConfig("bf16_many_tiles", T=7000, E=24, k=4, d=192, f=1024, dtype="bf16", zipf_s=1.0, nodes=1,
                      gpus_per_node=2, n_hot=3, replica_mode="all", seed=21)
    wl = make_workload(cfg)
    pl = wl.placement
    lr = 0
    ref = oracle.route_permute(wl.logits, pl, cfg.k, lr)
    table, g = run_route_permute(wl, pl, cfg.k, lr)
    check_route_permute(g, ref, wl, cfg.k)
    lo, hi = int(ref.perm.rank_off[lr]), int(ref.perm.rank_off[lr + 1])
    seg = np.diff(ref.perm.inst_off[ref.order.rank_ptr[lr]:ref.order.rank_ptr[lr + 1] + 1])
    assert sum(-(-int(m) // 256) for m in seg) * (cfg.f // 128) > 2 * 256      # > 2 tiles per workgroup
    wg, wu, wd = _stack_dev(wl, table.local_experts(lr))
    y = grace.grace_expert_ffn(table, lr, g.xp, g.ioff, cfg.T, cfg.k, wg, wu, wd)
    torch.cuda.synchronize()
    want = oracle.expert_ffn(ref, oracle.widen(wl.x), cfg.k, [lr], _weights64(wl), threads=8)
    assert rel_err(oracle.widen(host(y))[lo:hi], want[lo:hi]) <= TOL["bf16"]
    assert not host(y)[:lo].any() and not host(y)[hi:].any()      # rows of the other rank untouched


def test_few_row_tiles_many_column_tiles_element_by_element():
    """Two m-tiles with 36 (up) and 33 (down) n-tiles: dealing whole m-tiles to the XCDs would take
    two rounds of tiles, so the GEMM cuts the (m-tile, n-tile) pairs flat into eight ranges with the
    m index running fastest."""
    cfg = LayerConfig("bf16_wide", T=300, E=2, k=1, d=8448, f=4608, dtype="bf16", zipf_s=0.5, nodes=1,
                      gpus_per_node=1, n_hot=1, replica_mode="all", seed=23)
    wl = make_workload(cfg)
    pl = wl.placement
    ref = oracle.route_permute(wl.logits, pl, cfg.k, 0)
    table, g = run_route_permute(wl, pl, cfg.k, 0)
    check_route_permute(g, ref, wl, cfg.k)
    seg = np.diff(ref.perm.inst_off)
    m_tiles = sum(-(-int(m) // 256) for m in seg)
    assert m_tiles == 2 and cfg.f // 128 > 32 and cfg.d // 256 > 32
    wg, wu, wd = _stack_dev(wl, table.local_experts(0))
    y = grace.grace_expert_ffn(table, 0, g.xp, g.ioff, cfg.T, cfg.k, wg, wu, wd)
    torch.cuda.synchronize()
    want = oracle.expert_ffn(ref, oracle.widen(wl.x), cfg.k, [0], _weights64(wl), threads=8)
    assert rel_err(oracle.widen(host(y)), want) <= TOL["bf16"]


def test_few_tiles_long_k_element_by_element():
    """Two m-tiles, 32 (up) and 16 (down) n-tiles, 64 K steps each: fewer tiles than compute units and
    a long K (the shape of mixtral's projections at a small batch), expert and shared FFN."""
    cfg = LayerConfig("bf16_long_k", T=300, E=2, k=1, d=4096, f=4096, dtype="bf16", zipf_s=0.5, nodes=1,
                      gpus_per_node=1, n_hot=1, replica_mode="all", n_shared=1, seed=24)
    wl = make_workload(cfg)
    pl = wl.placement
    ref = oracle.route_permute(wl.logits, pl, cfg.k, 0)
    table, g = run_route_permute(wl, pl, cfg.k, 0)
    check_route_permute(g, ref, wl, cfg.k)
    seg = np.diff(ref.perm.inst_off)
    m_tiles = sum(-(-int(m) // 256) for m in seg)
    assert m_tiles * (cfg.f // 128) < 256 and cfg.d // 64 >= 64 and cfg.f // 64 >= 64
    wg, wu, wd = _stack_dev(wl, table.local_experts(0))
    y = grace.grace_expert_ffn(table, 0, g.xp, g.ioff, cfg.T, cfg.k, wg, wu, wd)
    torch.cuda.synchronize()
    x64 = oracle.widen(wl.x)
    want = oracle.expert_ffn(ref, x64, cfg.k, [0], _weights64(wl), threads=8)
    assert rel_err(oracle.widen(host(y)), want) <= TOL["bf16"]
    # the shared expert's FFN on the same shape: one segment of 300 rows, K segments in the down projection
    sh = wl.shared_weights()
    ys = grace.grace_shared_ffn(g.x, *[dev(w) for w in sh])
    torch.cuda.synchronize()
    ys_ref = oracle.shared_ffn(x64, tuple(oracle.widen(w) for w in sh))
    assert rel_err(oracle.widen(host(ys)), ys_ref) <= TOL["bf16"]


def test_more_than_64_local_slots_element_by_element():
    """A rank hosting more than 64 expert instances (four row segments per lane in the GEMM's
    segment table), many of them empty or a few rows long."""
    cfg = LayerConfig("bf16_many_slots", T=1500, E=180, k=4, d=128, f=192, dtype="bf16", zipf_s=1.0, nodes=1,
                      gpus_per_node=2, n_hot=4, replica_mode="all", seed=22)
    wl = make_workload(cfg)
    pl = wl.placement
    lr = 1
    ref = oracle.route_permute(wl.logits, pl, cfg.k, lr)
    table, g = run_route_permute(wl, pl, cfg.k, lr)
    check_route_permute(g, ref, wl, cfg.k)
    experts = table.local_experts(lr)
    assert len(experts) > 64
    lo, hi = int(ref.perm.rank_off[lr]), int(ref.perm.rank_off[lr + 1])
    wg, wu, wd = _stack_dev(wl, experts)
    y = grace.grace_expert_ffn(table, lr, g.xp, g.ioff, cfg.T, cfg.k, wg, wu, wd)
    torch.cuda.synchronize()
    want = oracle.expert_ffn(ref, oracle.widen(wl.x), cfg.k, [lr], _weights64(wl), threads=8)
    assert rel_err(oracle.widen(host(y))[lo:hi], want[lo:hi]) <= TOL["bf16"]


def _chosen_tile_height(seg_rows, n_tiles_n, grid):
    """The down projection's rule for its m-tile height (fragments of 16 rows per wavefront): the height
    with the smallest rounds x (HF + 2), ties to the higher tile."""
    best = None
    for hf in (8, 7, 6, 5):
        tiles = sum(-(-int(m) // (32 * hf)) for m in seg_rows) * n_tiles_n
        cost = -(-tiles // grid) * (hf + 2)
        if best is None or cost < best[0]:
            best = (cost, hf)
    return best[1]


@pytest.mark.parametrize("want_hf,seg_rows", [
    (8, [26000, 3000, 777, 1, 0, 900]),        # 256-row tiles fill one round of 256 workgroups (d = 512: 2 n-tiles)
    (7, [22000, 3000, 777, 1, 0, 900]),        # 224-row tiles still fit one round: cheaper than 256-row tiles
    (6, [18000, 3000, 777, 1, 0, 900]),        # 192-row tiles
    (5, [12000, 3000, 777, 1, 0, 900]),        # 160-row tiles
])
def test_expert_down_projection_every_tile_height(want_hf, seg_rows):
    """The expert down projection picks its m-tile height (256, 224, 192 or 160 rows) from the row
    segments it finds on the device; one case per height, ragged segments (an empty one, one of a single
    row), every element of the FFN against the oracle."""
    d, f, k = 512, 128, 1
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    grid = max(8, n_cu // 8 * 8)
    assert _chosen_tile_height(seg_rows, d // 256, grid) == want_hf or grid != 256
    E = len(seg_rows)
    rows = int(sum(seg_rows))
    rng = np.random.default_rng(100 + want_hf)
    table = grace.GraceTable(E, 1, 1, [0], [1], list(range(E + 1)), [0] * E)      # every expert once, on the one rank
    xp = torch.from_numpy(rng.standard_normal((rows, d)).astype(np.float32)).cuda().to(torch.bfloat16)
    wg = torch.from_numpy((0.05 * rng.standard_normal((E, f, d))).astype(np.float32)).cuda().to(torch.bfloat16)
    wu = torch.from_numpy((0.05 * rng.standard_normal((E, f, d))).astype(np.float32)).cuda().to(torch.bfloat16)
    wd = torch.from_numpy((0.05 * rng.standard_normal((E, d, f))).astype(np.float32)).cuda().to(torch.bfloat16)
    off = np.concatenate([[0], np.cumsum(seg_rows)]).astype(np.int32)
    y = grace.grace_expert_ffn(table, 0, xp, torch.from_numpy(off).cuda(), rows, k, wg, wu, wd)
    torch.cuda.synchronize()
    x64, got = oracle.widen(host(xp)), oracle.widen(host(y))
    for e in range(E):
        lo, hi = int(off[e]), int(off[e + 1])
        if hi == lo:
            continue
        want = oracle.ffn_rows(x64[lo:hi], oracle.widen(host(wg[e])), oracle.widen(host(wu[e])), oracle.widen(host(wd[e])),
                               threads=8)
        assert rel_err(got[lo:hi], want) <= TOL["bf16"], (want_hf, e)


@pytest.mark.parametrize("T,d,f,n_shared,k,dtype", [
    (3000, 512, 384, 2, 6, "bf16"),     # 1 KB rows, 12 row tiles x 6 column tiles: every workgroup has K steps to copy in
    (300, 4096, 128, 1, 3, "bf16"),     # 8 KB rows, 2 tiles for 256 workgroups: nearly all rows moved after the tile loop
    (5000, 1024, 1024, 1, 1, "bf16"),   # k = 1
    (700, 2048, 256, 3, 64, "bf16"),    # k = 64: the largest top-k
    (333, 136, 200, 1, 2, "bf16"),      # 272-byte rows: the scatter runs as a launch of its own
    (150, 128, 76, 3, 3, "f32"),        # fp32: likewise
])
def test_shared_up_with_row_scatter_equals_the_two_calls(T, d, f, n_shared, k, dtype):
    """grace_shared_ffn_up_scatter (the shared gate+up projection carrying the row scatter) against
    grace_shared_ffn_up + grace_permute_rows, bit for bit, and the rows against the oracle's gather;
    positions outside the buffer (-1: expert outside the table) are skipped."""
    rng = np.random.default_rng(T + d)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.from_numpy(rng.standard_normal((T, d)).astype(np.float32)).cuda().to(tdt)
    wg = torch.from_numpy((0.05 * rng.standard_normal((n_shared, f, d))).astype(np.float32)).cuda().to(tdt)
    wu = torch.from_numpy((0.05 * rng.standard_normal((n_shared, f, d))).astype(np.float32)).cuda().to(tdt)
    perm = rng.permutation(T * k).astype(np.int32)              # any bijection is a valid dispatch order here
    pos_h = perm.copy()
    dropped = rng.choice(T * k, size=max(1, T * k // 50), replace=False)
    pos_h[dropped] = -1
    pos = torch.from_numpy(pos_h).cuda()
    nbytes = grace.grace_workspace_bytes(T, 1, 1, 1, d, f, n_shared, grace.GRACE_F32 if dtype == "f32" else grace.GRACE_BF16)
    ws_a = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    ws_b = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    xp_a = torch.full((T * k, d), 7.0, dtype=tdt, device="cuda")
    xp_b = torch.full((T * k, d), 7.0, dtype=tdt, device="cuda")
    grace.grace_shared_ffn_up_scatter(x, wg, wu, ws_a, pos, k, xp_a)
    grace.grace_shared_ffn_up(x, wg, wu, ws_b)
    grace.grace_permute_rows(x, pos, k, xp_b)
    torch.cuda.synchronize()
    assert torch.equal(ws_a, ws_b)                                   # the hidden activation, bit for bit
    # the two launches of the shared FFN as separate calls against the single call
    wd = torch.from_numpy((0.05 * rng.standard_normal((n_shared, d, f))).astype(np.float32)).cuda().to(tdt)
    ys_two = grace.grace_shared_ffn_down(wd, ws_b, T)
    ys_one = grace.grace_shared_ffn(x, wg, wu, wd)
    torch.cuda.synchronize()
    assert torch.equal(ys_two.view(torch.uint8), ys_one.view(torch.uint8))
    assert torch.equal(xp_a.view(torch.uint8), xp_b.view(torch.uint8))
    # rows against the definition: xp[p] = x[a // k] where perm_pos[a] = p; dropped positions keep their old contents
    got, xh = host(xp_a), host(x)
    keep = pos_h >= 0
    np.testing.assert_array_equal(got[pos_h[keep]], xh[np.nonzero(keep)[0] // k])
    untouched = np.setdiff1d(np.arange(T * k), pos_h[keep])
    assert len(untouched) == len(dropped)
    np.testing.assert_array_equal(got[untouched], host(torch.full((len(untouched), d), 7.0, dtype=tdt)))


def test_layer_object_rank_share_matches_oracle():
    cfg = SMALL["bf16_small"]
    wl = make_workload(cfg)
    pl = wl.placement
    table = grace.GraceTable.from_placement(pl)
    lr = 2
    wg, wu, wd = _stack_dev(wl, table.local_experts(lr))
    sh = tuple(dev(w) for w in wl.shared_weights())
    layer = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, torch.bfloat16, wg, wu, wd, shared=sh)
    logits, x = dev(wl.logits), dev(wl.x)
    for _ in range(2):       # buffers are reused between calls
        out = layer.forward(logits, x)
    torch.cuda.synchronize()
    ref = oracle.route_permute(wl.logits, pl, cfg.k, lr)
    x64 = oracle.widen(wl.x)
    y_ref = oracle.expert_ffn(ref, x64, cfg.k, [lr], _weights64(wl))
    ys_ref = oracle.shared_ffn(x64, tuple(oracle.widen(w) for w in wl.shared_weights()))
    out_ref = oracle.combine(y_ref, ref.perm.perm_pos, ref.topk_weight, ys_ref)
    assert rel_err(oracle.widen(host(out)), out_ref) <= TOL["bf16"]


@pytest.mark.parametrize("name", ["tiny", "bf16_ragged", "f32_ragged"])
def test_layer_rank_share_after_routing_changes(name):
    """A layer object stepped with changing gate logits (fp32 kernel and the generic bf16 kernel; the
    persistent kernel is covered by the graph replay test): after every step `y` is the oracle's rank
    share for that step's inputs, rows of other ranks zero although earlier steps wrote there."""
    cfg = SMALL[name]
    wl = make_workload(cfg)
    pl = wl.placement
    table = grace.GraceTable.from_placement(pl)
    lr = 1
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    wg, wu, wd = _stack_dev(wl, table.local_experts(lr))
    sh = wl.shared_weights()
    shd = None if sh is None else tuple(dev(w) for w in sh)
    layer = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, tdt, wg, wu, wd, shared=shd)
    x = dev(wl.x)
    x64, w64 = oracle.widen(wl.x), _weights64(wl)
    ys_ref = None if sh is None else oracle.shared_ffn(x64, tuple(oracle.widen(w) for w in sh))
    rng = np.random.default_rng(17)
    ranges = set()
    for rep in range(5):
        lg = wl.logits if rep == 0 else (rng.standard_normal(wl.logits.shape) + 3.0 * rng.standard_normal(cfg.E)).astype(np.float32)
        out = layer.forward(dev(lg), x)
        torch.cuda.synchronize()
        ref = oracle.route_permute(lg, pl, cfg.k, lr)
        lo, hi = int(ref.perm.rank_off[lr]), int(ref.perm.rank_off[lr + 1])
        ranges.add((lo, hi))
        assert not bool(layer.y[:lo].any()) and not bool(layer.y[hi:].any()), f"step {rep}: stale rows outside [{lo},{hi})"
        y_ref = oracle.expert_ffn(ref, x64, cfg.k, [lr], w64)
        assert rel_err(oracle.widen(host(layer.y))[lo:hi], y_ref[lo:hi]) <= TOL[cfg.dtype], f"step {rep}"
        out_ref = oracle.combine(y_ref, ref.perm.perm_pos, ref.topk_weight, ys_ref)
        assert rel_err_rows(oracle.widen(host(out)), out_ref) <= TOL[cfg.dtype], f"step {rep}"
    assert len(ranges) >= 3


@pytest.mark.parametrize("name", ["olmoe_decode64", "olmoe_decode512"])
def test_decode_shaped_rank_share_element_by_element(name):
    """Decode-sized batches (every instance far below a tile): whole rank share, every element."""
    cfg = CONFIGS[name]
    wl = make_workload(cfg)
    pl = wl.placement
    lr = cfg.local_rank
    table = grace.GraceTable.from_placement(pl)
    wg, wu, wd = _stack_dev(wl, table.local_experts(lr))
    layer = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, torch.bfloat16, wg, wu, wd)
    out = layer.forward(dev(wl.logits), dev(wl.x))
    torch.cuda.synchronize()
    ref = oracle.route_permute(wl.logits, pl, cfg.k, lr)
    np.testing.assert_array_equal(host(layer.route_out[2]), ref.topk_inst)
    np.testing.assert_array_equal(host(layer.perm_out[0]), ref.perm.perm_pos)
    np.testing.assert_array_equal(host(layer.perm_out[2]), ref.perm.inst_off)
    x64 = oracle.widen(wl.x)
    y_ref = oracle.expert_ffn(ref, x64, cfg.k, [lr], _weights64(wl), threads=8)
    assert rel_err(oracle.widen(host(layer.y)), y_ref) <= TOL["bf16"]
    out_ref = oracle.combine(y_ref, ref.perm.perm_pos, ref.topk_weight)
    assert rel_err(oracle.widen(host(out)), out_ref) <= TOL["bf16"]


def test_graph_replays_match_eager_and_oracle():
    """A captured step replayed several times, with eager work and synchronisations in
    between and inputs changed in place, gives the eager result every time; and after every
    change of the inputs (the rank's row range moves with the routing) the output is the
    oracle's rank share for those inputs: rows of other ranks are zero again, whatever an
    earlier step left there."""
    cfg = SMALL["bf16_small"]
    wl = make_workload(cfg)
    pl = wl.placement
    table = grace.GraceTable.from_placement(pl)
    lr = 1
    wg, wu, wd = _stack_dev(wl, table.local_experts(lr))
    sh = tuple(dev(w) for w in wl.shared_weights())
    sh64 = tuple(oracle.widen(w) for w in wl.shared_weights())
    w64 = _weights64(wl)
    layer = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, torch.bfloat16, wg, wu, wd, shared=sh)
    eager = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, torch.bfloat16, wg, wu, wd, shared=sh)
    logits, x = dev(wl.logits), dev(wl.x)
    graph = layer.capture(logits, x)
    rng = np.random.default_rng(3)
    ranges = set()
    for rep in range(5):
        if rep:
            # a different hot set every time, so the rows of rank `lr` start and end elsewhere
            bias = 3.0 * rng.standard_normal(cfg.E)
            logits.copy_(torch.from_numpy((rng.standard_normal(wl.logits.shape) + bias).astype(np.float32)).cuda())
            x.copy_(torch.from_numpy(rng.standard_normal(wl.x.shape).astype(np.float32)).cuda().to(torch.bfloat16))
        graph.replay()
        torch.cuda.synchronize()
        want = eager.forward(logits.clone(), x.clone())
        torch.cuda.synchronize()
        assert torch.equal(layer.out, want), f"replay {rep}"
        for a, b in zip(layer.route_out + layer.perm_out, eager.route_out + eager.perm_out):
            assert torch.equal(a, b)
        # against the oracle for the inputs of this replay
        ref = oracle.route_permute(host(logits), pl, cfg.k, lr)
        lo, hi = int(ref.perm.rank_off[lr]), int(ref.perm.rank_off[lr + 1])
        ranges.add((lo, hi))
        np.testing.assert_array_equal(host(layer.perm_out[0]), ref.perm.perm_pos)
        for L in (layer, eager):
            assert not bool(L.y[:lo].any()) and not bool(L.y[hi:].any()), f"replay {rep}: stale rows outside [{lo},{hi})"
        x64 = oracle.widen(host(x))
        y_ref = oracle.expert_ffn(ref, x64, cfg.k, [lr], w64)
        out_ref = oracle.combine(y_ref, ref.perm.perm_pos, ref.topk_weight, oracle.shared_ffn(x64, sh64))
        assert rel_err(oracle.widen(host(layer.out)), out_ref) <= TOL["bf16"], f"replay {rep}"
    assert len(ranges) >= 3      # the range did move


# ------------------------------------------- full-size configs, every element --
@pytest.mark.parametrize("name", ["olmoe", "qwen", "dsv2lite", "mixtral", "qwen3moe"])
def test_full_size_rank_share_every_element(name):
    """BASELINE sizes in the launch configuration bench.py times (GraceMoELayer.forward, twice, so
    that the second step runs on reused buffers): integers bit-exact over the whole call, the
    dispatch buffer bit for bit, and EVERY local FFN row, every shared-expert row and every
    output row against the oracle (16 host threads; the whole rank share is a few seconds to a
    few tens of seconds of oracle time per config)."""
    cfg = CONFIGS[name]
    wl = make_workload(cfg)
    pl = wl.placement
    lr = cfg.local_rank
    table = grace.GraceTable.from_placement(pl)
    experts = table.local_experts(lr)
    wg, wu, wd = _stack_dev(wl, experts)
    sh = wl.shared_weights()
    shd = None if sh is None else tuple(dev(w) for w in sh)
    layer = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, torch.bfloat16, wg, wu, wd, shared=shd)
    logits, x = dev(wl.logits), dev(wl.x)
    for _ in range(2):
        out = layer.forward(logits, x)
    torch.cuda.synchronize()
    threads = min(oracle.max_threads(), 16)
    ref = oracle.route_permute(wl.logits, pl, cfg.k, lr)
    te, tw, ti, cnt = layer.route_out
    pos, src, ioff, roff, noff = layer.perm_out
    np.testing.assert_array_equal(host(te), ref.topk_expert)
    np.testing.assert_array_equal(host(ti), ref.topk_inst)
    np.testing.assert_array_equal(host(cnt), ref.expert_count)
    np.testing.assert_allclose(host(tw), ref.topk_weight, rtol=1e-6, atol=0)
    np.testing.assert_array_equal(host(pos), ref.perm.perm_pos)
    np.testing.assert_array_equal(host(src), ref.perm.perm_src)
    np.testing.assert_array_equal(host(ioff), ref.perm.inst_off)
    np.testing.assert_array_equal(host(roff), ref.perm.rank_off)
    np.testing.assert_array_equal(host(noff), ref.perm.node_off)
    # dispatch buffer, bit for bit, every row
    np.testing.assert_array_equal(host(layer.xp), oracle.gather_rows(wl.x, ref.perm.perm_src, cfg.k))
    # every FFN row of the local share; rows of other ranks are zero
    lo, hi = int(ref.perm.rank_off[lr]), int(ref.perm.rank_off[lr + 1])
    x64 = oracle.widen(wl.x)
    y_ref = oracle.expert_ffn(ref, x64, cfg.k, [lr], _weights64(wl), threads=threads)
    assert rel_err(oracle.widen(host(layer.y[lo:hi])), y_ref[lo:hi]) <= TOL["bf16"]
    if lo > 0:
        assert not bool(layer.y[:lo].any())
    if hi < cfg.T * cfg.k:
        assert not bool(layer.y[hi:].any())
    # every shared-expert row
    ys_ref = None
    if sh is not None:
        ys_ref = oracle.shared_ffn(x64, tuple(oracle.widen(w) for w in sh), threads=threads)
        assert rel_err(oracle.widen(host(layer.y_shared)), ys_ref) <= TOL["bf16"]
    # every output row.  In a rank share a row is the gate-weighted sum over the token's local experts
    # only, so rows differ widely in scale (and a token without a local expert or shared experts has an
    # all-zero row, which must come out as exact zeros): the metric's floor is the rms of the row.
    out_ref = oracle.combine(y_ref, ref.perm.perm_pos, ref.topk_weight, ys_ref)
    got = oracle.widen(host(out))
    assert rel_err_rows(got, out_ref) <= TOL["bf16"]
    # the combine kernel by itself, sharply: from the path's own y, y_shared and gate weights the
    # output is the fp32-accumulated sum rounded once to bf16
    y_own = oracle.widen(host(layer.y))
    own = oracle.combine(y_own, ref.perm.perm_pos, host(tw), None if sh is None else oracle.widen(host(layer.y_shared)))
    slack = 1e-6 * float(np.abs(y_own).max())       # fp32 accumulation of k terms that may cancel
    assert np.all(np.abs(got - own) <= 2.0 ** -8 * np.abs(own) + slack)


def test_routing_report_runs_and_is_consistent(capsys, monkeypatch):
    """routing_report.py (replication and policy ablation on one GPU): totals add up, de-duplication never
    adds traffic, and locality-first routing sends no more rows across nodes than round-robin over all
    instances."""
    import json
    import routing_report
    monkeypatch.setattr(sys, "argv", ["routing_report.py", "--workload", "tiny", "--planner"])
    assert routing_report.main() == 0
    lines = [json.loads(l) for l in capsys.readouterr().out.strip().splitlines()]
    assert [l["setup"] for l in lines] == ["no replicas", "replicas, weighted round-robin", "replicas, locality first",
                                           "planner table (Equations 3, 4), weighted round-robin",
                                           "planner table (Equations 3, 4), locality first"]
    # the planner's table is consumed by the path: replicas exist and flatten the load against no replicas
    assert lines[3]["n_replica"] >= 1 and lines[3]["instances"] > lines[0]["instances"]
    assert lines[3]["rows_per_rank"]["std"] < lines[0]["rows_per_rank"]["std"]
    assert lines[4]["cross_node_tokens"]["one_row_per_assignment"] <= lines[3]["cross_node_tokens"]["one_row_per_assignment"]
    cfg = CONFIGS["tiny"]
    for l in lines:
        assert l["rows_per_rank"]["mean"] * l["ranks"] == cfg.T * cfg.k * l["ranks"]
        assert l["cross_node_tokens"]["dedup"] <= l["cross_node_tokens"]["one_row_per_assignment"]
    assert lines[2]["cross_node_tokens"]["one_row_per_assignment"] <= lines[1]["cross_node_tokens"]["one_row_per_assignment"]
