"""Pins of the CPU oracle against things other than itself: values worked by
hand from the paper's algorithms (tests/golden), closed forms, library
routines (stable argsort, matmul, softmax), brute force on tiny inputs and the
invariants the method guarantees.  None of these tests needs a GPU."""
import itertools
import json
import os
from types import SimpleNamespace

import numpy as np
import pytest
import scipy.special

import oracle
from workloads import CONFIGS, LayerConfig, make_workload

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def gold(name):
    with open(os.path.join(GOLD, name)) as fh:
        return json.load(fh)


def table_from(g):
    return SimpleNamespace(E=g["E"], R=g["R"], N=g["N"], rank_node=np.array(g["rank_node"], np.int32),
                           poll_weight=np.array(g["poll_weight"], np.uint32),
                           inst_ptr=np.array(g["inst_ptr"], np.int32),
                           inst_rank=np.array(g["inst_rank"], np.int32))


# ----------------------------------------------------------------- O1 top-k --
def test_topk_closed_form_golden():
    g = gold("gating_closed_form.json")
    logits = np.log(np.array([g["logits_exp"]], dtype=np.float64)).astype(np.float32)
    te, tw = oracle.topk(logits, g["k"], renorm=0)
    assert te.tolist() == [g["topk_expert"]]
    np.testing.assert_allclose(tw[0], g["weight_no_renorm"], rtol=2e-7)
    te, tw = oracle.topk(logits, g["k"], renorm=1)
    assert te.tolist() == [g["topk_expert"]]
    np.testing.assert_allclose(tw[0], g["weight_renorm"], rtol=2e-7)


@pytest.mark.parametrize("E,k", [(8, 2), (64, 8), (60, 4), (5, 5), (7, 1)])
def test_topk_matches_stable_argsort_and_library_softmax(E, k):
    rng = np.random.default_rng(E * 100 + k)
    logits = rng.standard_normal((300, E)).astype(np.float32)
    logits[:50] = np.round(logits[:50] * 2) / 2        # many exact ties
    logits[50, :] = 0.25                                # all equal
    logits[51, :] = np.where(np.arange(E) % 2 == 0, 0.0, -0.0)   # -0.0 == +0.0 is a tie
    te, tw = oracle.topk(logits, k, renorm=0)
    ref_idx = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :k]
    np.testing.assert_array_equal(te, ref_idx)
    p = scipy.special.softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(tw, np.take_along_axis(p, ref_idx, 1), rtol=3e-7)
    te2, tw2 = oracle.topk(logits, k, renorm=1)
    np.testing.assert_array_equal(te2, ref_idx)
    sel = np.take_along_axis(logits.astype(np.float64), ref_idx, 1)
    np.testing.assert_allclose(tw2, scipy.special.softmax(sel, axis=1), rtol=3e-7)
    np.testing.assert_allclose(tw2.astype(np.float64).sum(1), 1.0, atol=5e-7)


def test_topk_brute_force_subsets():
    """The chosen set maximises the sum of logits over all k-subsets, and among
    maximal subsets is the lexicographically smallest index set (tie rule)."""
    rng = np.random.default_rng(3)
    logits = np.round(rng.standard_normal((40, 6)) * 1.5).astype(np.float32)
    te, _ = oracle.topk(logits, 3, renorm=1)
    for t in range(logits.shape[0]):
        best = max(itertools.combinations(range(6), 3),
                   key=lambda s: (float(sum(np.float64(logits[t, i]) for i in s)), [-i for i in s]))
        assert sorted(te[t].tolist()) == list(best)
        vals = logits[t, te[t]]
        assert all(vals[j] >= vals[j + 1] for j in range(2))          # descending
        assert len(set(te[t].tolist())) == 3                            # distinct


def test_topk_special_cases():
    rng = np.random.default_rng(4)
    logits = rng.standard_normal((20, 9)).astype(np.float32)
    te, tw = oracle.topk(logits, 1, renorm=1)
    np.testing.assert_array_equal(te[:, 0], np.argmax(logits, axis=1))
    np.testing.assert_array_equal(tw, np.ones_like(tw))
    te, tw = oracle.topk(logits, 9, renorm=0)            # k = E: the full softmax, sums to one
    np.testing.assert_allclose(tw.astype(np.float64).sum(1), 1.0, atol=1e-6)
    assert sorted(te[0].tolist()) == list(range(9))
    with pytest.raises(ValueError):
        oracle.topk(logits, 10)


# ------------------------------------------------ O2-O5 hand-worked example --
def test_pick_and_permute_worked_example():
    g = gold("replica_pick_worked_example.json")
    pl = table_from(g)
    order = oracle.instance_order(pl)
    assert order.g_expert.tolist() == g["dispatch_order_expert"]
    assert order.g_rank.tolist() == g["dispatch_order_rank"]
    te = np.array(g["topk_expert"], np.int32)
    c = g["case_rr0"]
    ti, cnt, rout = oracle.pick(te, pl, g["local_rank"])
    assert ti.reshape(-1).tolist() == c["topk_inst"]
    assert cnt.tolist() == c["expert_count"]
    assert rout.tolist() == c["rr_out"]
    pm = oracle.permute(ti, pl)
    assert pm.perm_src.tolist() == c["perm_src"]
    assert pm.perm_pos.tolist() == c["perm_pos"]
    assert pm.inst_off.tolist() == c["inst_off"]
    assert pm.rank_off.tolist() == c["rank_off"]
    assert pm.node_off.tolist() == c["node_off"]
    c = g["case_rr_carry"]
    ti, cnt, rout = oracle.pick(te, pl, g["local_rank"], rr_in=np.array(c["rr_in"], np.uint32))
    assert ti.reshape(-1).tolist() == c["topk_inst"]
    assert cnt.tolist() == c["expert_count"]
    assert rout.tolist() == c["rr_out"]
    c = g["case_wrr_policy"]
    for lr in (c["local_rank"], 0, 5):                  # without locality the source rank does not matter
        ti, cnt, rout = oracle.pick(te, pl, lr, policy=1)
        assert ti.reshape(-1).tolist() == c["topk_inst"]
        assert cnt.tolist() == c["expert_count"]
        assert rout.tolist() == c["rr_out"]
    ti_tar, _, _ = oracle.pick(te, pl, c["local_rank"], policy=0)
    assert order.g_rank[ti_tar.reshape(-1)[5]] == c["local_rank"]      # Algorithm 4 keeps expert 0 on rank 3
    assert ti_tar.reshape(-1).tolist() != c["topk_inst"]


# ----------------------------------------------------- send lists (Section 5) --
def test_send_lists_worked_examples():
    g = gold("replica_pick_worked_example.json")
    pl = table_from(g)
    c = g["send_lists_rr0"]
    sl = oracle.send_lists(np.array(g["case_rr0"]["topk_inst"], np.int32).reshape(6, 2), pl, 0)
    assert sl.rank_send_ptr.tolist() == c["rank_send_ptr"] and sl.rank_send_tok.tolist() == c["rank_send_tok"]
    assert sl.node_send_ptr.tolist() == c["node_send_ptr"] and sl.node_send_tok.tolist() == c["node_send_tok"]
    c = g["send_lists_dup"]
    sl = oracle.send_lists(np.array(c["topk_inst"], np.int32), pl, 0)
    assert sl.rank_send_ptr.tolist() == c["rank_send_ptr"] and sl.rank_send_tok.tolist() == c["rank_send_tok"]
    assert sl.node_send_ptr.tolist() == c["node_send_ptr"] and sl.node_send_tok.tolist() == c["node_send_tok"]
    assert sl.expand.tolist() == c["expand"]
    assert sl.traffic.tolist() == c["traffic"]


@pytest.mark.parametrize("case", ["case_from_larger_node", "case_from_smaller_node"])
def test_send_lists_nodes_of_unequal_size(case):
    """Stage-1 peer in a node of another size: index inside the own node, modulo that node's size."""
    g = gold("send_lists_unequal_nodes.json")
    pl = table_from(g)
    order = oracle.instance_order(pl)
    assert order.g_rank.tolist() == [0, 1, 2, 3, 4] and order.g_expert.tolist() == [0, 1, 0, 1, 2]
    c = g[case]
    sl = oracle.send_lists(np.array(c["topk_inst"], np.int32), pl, c["local_rank"])
    assert sl.rank_send_ptr.tolist() == c["rank_send_ptr"] and sl.rank_send_tok.tolist() == c["rank_send_tok"]
    assert sl.node_send_ptr.tolist() == c["node_send_ptr"] and sl.node_send_tok.tolist() == c["node_send_tok"]
    assert sl.expand.tolist() == c["expand"]
    assert sl.traffic.tolist() == c["traffic"]


@pytest.mark.parametrize("name,local_rank", [("olmoe", 0), ("dsv2lite", 13), ("qwen", 5)])
def test_send_lists_against_library_unique(name, local_rank):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=min(cfg.T, 1500))
    pl = wl.placement
    res = oracle.route_permute(wl.logits, pl, cfg.k, local_rank)
    sl = oracle.send_lists(res.topk_inst, pl, local_rank, res.order)
    T = res.topk_inst.shape[0]
    ranks = res.order.g_rank[res.topk_inst]                  # [T, k]
    nodes = pl.rank_node[ranks]
    for r in range(pl.R):
        want = np.unique(np.nonzero((ranks == r).any(1))[0])
        np.testing.assert_array_equal(sl.rank_send_tok[sl.rank_send_ptr[r]:sl.rank_send_ptr[r + 1]], want)
    for n in range(pl.N):
        want = np.unique(np.nonzero((nodes == n).any(1))[0])
        np.testing.assert_array_equal(sl.node_send_tok[sl.node_send_ptr[n]:sl.node_send_ptr[n + 1]], want)
    # the expansion map leads every assignment back to its own token
    flat_rank = ranks.reshape(-1)
    tok = sl.rank_send_tok[sl.rank_send_ptr[flat_rank] + sl.expand]
    np.testing.assert_array_equal(tok, np.repeat(np.arange(T), cfg.k))
    # de-duplication never sends more than one row per assignment, and at least one per k assignments
    my_node = pl.rank_node[local_rank]
    assert sl.traffic[0] <= sl.traffic[1] <= cfg.k * max(sl.traffic[0], 1) or sl.traffic[1] == 0
    assert sl.traffic[1] == int((nodes != my_node).sum())
    assert sl.traffic[3] == int(((nodes == my_node) & (ranks != local_rank)).sum())


# --------------------------------------------------------- O3 invariants --
def _cands(pl, e, local_rank):
    ranks = pl.inst_rank[pl.inst_ptr[e]:pl.inst_ptr[e + 1]].tolist()
    if local_rank in ranks:
        return [local_rank]
    same = [r for r in ranks if pl.rank_node[r] == pl.rank_node[local_rank]]
    return same if same else ranks


def _cands_policy(pl, e, local_rank, policy):
    if policy == 1:
        return pl.inst_rank[pl.inst_ptr[e]:pl.inst_ptr[e + 1]].tolist()
    return _cands(pl, e, local_rank)


@pytest.mark.parametrize("name", ["tiny", "olmoe", "qwen", "dsv2lite", "mixtral"])
@pytest.mark.parametrize("local_rank,policy", [(0, 0), (3, 0), (1, 1)])
def test_pick_invariants_and_wrr_shares(name, local_rank, policy):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=min(cfg.T, 2048))
    pl = wl.placement
    res = oracle.route_permute(wl.logits, pl, cfg.k, local_rank, policy=policy)
    order = res.order
    ti = res.topk_inst.reshape(-1)
    te = res.topk_expert.reshape(-1)
    # every token gets exactly k distinct experts; every chosen instance hosts its expert
    assert res.topk_expert.shape == (wl.logits.shape[0], cfg.k)
    assert all(len(set(r)) == cfg.k for r in res.topk_expert.tolist())
    np.testing.assert_array_equal(order.g_expert[ti], te)
    np.testing.assert_array_equal(np.bincount(te, minlength=cfg.E), res.expert_count)
    chosen_rank = order.g_rank[ti]
    my_node = pl.rank_node[local_rank]
    for e in range(cfg.E):
        m = te == e
        n = int(m.sum())
        cands = _cands_policy(pl, e, local_rank, policy)
        ranks_e = pl.inst_rank[pl.inst_ptr[e]:pl.inst_ptr[e + 1]].tolist()
        if policy == 1:
            pass
        elif local_rank in ranks_e:                      # tier 1: never leaves the GPU
            assert (chosen_rank[m] == local_rank).all()
        elif any(pl.rank_node[r] == my_node for r in ranks_e):   # tier 2: never leaves the node
            assert (pl.rank_node[chosen_rank[m]] == my_node).all()
        # closed form of block weighted round-robin: over n requests candidate s gets
        # floor(n/W)*w_s + clamp(n mod W - cum_before_s, 0, w_s)
        w = [int(pl.poll_weight[r]) for r in cands]
        W = sum(w)
        cum = 0
        for r, ws in zip(cands, w):
            expect = (n // W) * ws + min(max(n % W - cum, 0), ws)
            assert int((chosen_rank[m] == r).sum()) == expect, (e, r)
            cum += ws
        assert int(res.rr_out[e]) == n % W


def test_pick_equal_weights_is_plain_round_robin_and_single_instance():
    # 1 node x 4 GPUs seen from a rank that hosts nothing: expert 0 on ranks 1,2,3 (equal weights)
    pl = SimpleNamespace(E=2, R=4, N=1, rank_node=np.zeros(4, np.int32), poll_weight=np.full(4, 5, np.uint32),
                         inst_ptr=np.array([0, 3, 4], np.int32), inst_rank=np.array([1, 2, 3, 2], np.int32))
    te = np.zeros((30, 1), np.int32)
    te[::3] = 1
    order = oracle.instance_order(pl)
    ti, cnt, _ = oracle.pick(te, pl, 0)
    r = order.g_rank[ti.reshape(-1)]
    e0 = te.reshape(-1) == 0
    c = np.arange(e0.sum())
    np.testing.assert_array_equal(r[e0], 1 + (c // 5) % 3)      # blocks of 5 = the common weight
    assert (r[~e0] == 2).all()
    pl.poll_weight = np.ones(4, np.uint32)
    ti, _, _ = oracle.pick(te, pl, 0)
    np.testing.assert_array_equal(order.g_rank[ti.reshape(-1)][e0], 1 + c % 3)   # weight 1: c mod m
    # R = 1, no replicas: the pick is the identity expert -> instance map
    pl1 = SimpleNamespace(E=3, R=1, N=1, rank_node=np.zeros(1, np.int32), poll_weight=np.ones(1, np.uint32),
                          inst_ptr=np.arange(4, dtype=np.int32), inst_rank=np.zeros(3, np.int32))
    te = np.array([[2, 0], [1, 2]], np.int32)
    ti, _, _ = oracle.pick(te, pl1, 0)
    np.testing.assert_array_equal(ti, te)
    with pytest.raises(ValueError):
        oracle.pick(te, pl1, 1)


# ------------------------------------------------------ O5 permutation --
@pytest.mark.parametrize("name", ["tiny", "olmoe", "dsv2lite"])
def test_permutation_is_stable_argsort_and_offsets_are_cumsums(name):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, T=min(cfg.T, 1024))
    pl = wl.placement
    res = oracle.route_permute(wl.logits, pl, cfg.k, 0)
    pm, order = res.perm, res.order
    ti = res.topk_inst.reshape(-1)
    n = ti.shape[0]
    np.testing.assert_array_equal(pm.perm_src, np.argsort(ti, kind="stable"))
    np.testing.assert_array_equal(pm.perm_pos[pm.perm_src], np.arange(n))          # bijection
    np.testing.assert_array_equal(np.sort(pm.perm_pos), np.arange(n))
    cnt = np.bincount(ti, minlength=pl.I)
    np.testing.assert_array_equal(pm.inst_off, np.concatenate([[0], np.cumsum(cnt)]))
    assert pm.inst_off[-1] == pm.rank_off[-1] == pm.node_off[-1] == n
    np.testing.assert_array_equal(pm.rank_off, pm.inst_off[order.rank_ptr])
    first_rank_of_node = np.searchsorted(pl.rank_node, np.arange(pl.N + 1))
    np.testing.assert_array_equal(pm.node_off, pm.rank_off[first_rank_of_node])
    keys = ti[pm.perm_src]
    assert (np.diff(keys) >= 0).all()
    same = np.diff(keys) == 0
    assert (np.diff(pm.perm_src)[same] > 0).all()                                   # stable
    # dispatch order really is (node, rank, expert)
    trip = list(zip(pl.rank_node[order.g_rank].tolist(), order.g_rank.tolist(), order.g_expert.tolist()))
    assert trip == sorted(trip)
    xp = oracle.gather_rows(wl.x, pm.perm_src, cfg.k)
    np.testing.assert_array_equal(xp, wl.x[pm.perm_src // cfg.k])


def test_permute_rejects_bad_instance_id():
    pl = table_from(gold("replica_pick_worked_example.json"))
    with pytest.raises(ValueError):
        oracle.permute(np.array([[0, 9]], np.int32), pl)


# -------------------------------------------------------------- O6 FFN --
def test_ffn_closed_form_golden():
    g = gold("swiglu_closed_form.json")
    y = oracle.ffn_rows(np.array(g["x"]), np.array(g["w_gate"]), np.array(g["w_up"]), np.array(g["w_down"]))
    np.testing.assert_allclose(y, g["y"], rtol=1e-13)


def test_ffn_matches_library_matmul_and_special_cases():
    rng = np.random.default_rng(11)
    n, d, f = 37, 24, 40
    x = rng.standard_normal((n, d))
    wg, wu, wd = rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))
    y = oracle.ffn_rows(x, wg, wu, wd, threads=3)
    g = x @ wg.T
    ref = (g * scipy.special.expit(g) * (x @ wu.T)) @ wd.T
    np.testing.assert_allclose(y, ref, rtol=1e-11, atol=1e-11)
    # non-symmetric shapes catch a transposed operand; a zero down projection gives zeros
    assert np.all(oracle.ffn_rows(x, wg, wu, np.zeros((d, f))) == 0.0)
    # accumulate: two experts of width f == one expert of width 2f (concatenated gate/up, stacked down)
    wg2, wu2, wd2 = rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))
    acc = oracle.ffn_rows(x, wg, wu, wd)
    oracle.ffn_rows(x, wg2, wu2, wd2, out=acc, accumulate=True)
    wide = oracle.ffn_rows(x, np.vstack([wg, wg2]), np.vstack([wu, wu2]), np.hstack([wd, wd2]))
    np.testing.assert_allclose(acc, wide, rtol=1e-11, atol=1e-11)
    ys = oracle.shared_ffn(x, (np.stack([wg, wg2]), np.stack([wu, wu2]), np.stack([wd, wd2])))
    np.testing.assert_allclose(ys, wide, rtol=1e-11, atol=1e-11)


# ---------------------------------------------------------- O7 combine --
def test_combine_identity_experts_returns_inputs_and_one_hot_gathers():
    cfg = CONFIGS["tiny"]
    wl = make_workload(cfg)
    res = oracle.route_permute(wl.logits, wl.placement, cfg.k, 0, renorm=1)
    x64 = oracle.widen(wl.x)
    xp = x64[res.perm.perm_src // cfg.k]                 # identity experts: y = xp
    out = oracle.combine(xp, res.perm.perm_pos, res.topk_weight)
    np.testing.assert_allclose(out, x64, rtol=0, atol=2e-6)      # sum_j w_j = 1 up to fp32 rounding of w
    # one-hot weights: a pure gather of the j=1 row; use distinguishable rows
    y = np.arange(cfg.T * cfg.k * 3, dtype=np.float64).reshape(cfg.T * cfg.k, 3)
    w = np.zeros((cfg.T, cfg.k), np.float32)
    w[:, 1] = 1.0
    out = oracle.combine(y, res.perm.perm_pos, w)
    np.testing.assert_array_equal(out, y[res.perm.perm_pos.reshape(cfg.T, cfg.k)[:, 1]])
    ys = np.ones((cfg.T, 3))
    out2 = oracle.combine(y, res.perm.perm_pos, w, y_shared=ys)
    np.testing.assert_array_equal(out2, out + 1.0)
    # general weights against a library contraction
    w = np.random.default_rng(0).random((cfg.T, cfg.k)).astype(np.float32)
    ref = np.einsum("tj,tjc->tc", w.astype(np.float64), y[res.perm.perm_pos.reshape(cfg.T, cfg.k)])
    np.testing.assert_allclose(oracle.combine(y, res.perm.perm_pos, w), ref, rtol=1e-13)


# ------------------------------------------ P1 lossless: whole layer, any table --
def _dense_moe(wl, k, renorm, weights_of, shared):
    """Plain top-k MoE layer with no placement table at all (library routines)."""
    logits = wl.logits.astype(np.float64)
    x = oracle.widen(wl.x)
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    p = scipy.special.softmax(logits, axis=1)
    w = np.take_along_axis(p, idx, 1)
    if renorm:
        w = w / w.sum(1, keepdims=True)
    w = w.astype(np.float32).astype(np.float64)
    out = np.zeros_like(x)
    for e in range(wl.cfg.E):
        wg, wu, wd = weights_of(e)
        g = x @ wg.T
        ye = (g * scipy.special.expit(g) * (x @ wu.T)) @ wd.T
        for j in range(k):
            m = idx[:, j] == e
            out[m] += w[m, j][:, None] * ye[m]
    if shared is not None:
        for s in range(shared[0].shape[0]):
            g = x @ shared[0][s].T
            out += (g * scipy.special.expit(g) * (x @ shared[1][s].T)) @ shared[2][s].T
    return out


@pytest.mark.parametrize("base,n_shared", [("tiny", 0), ("tiny", 2)])
def test_layer_is_lossless_for_any_valid_table(base, n_shared):
    """Grouping, replication and routing move work, never change the result
    (abstract; Section 4): the layer output over all ranks equals the plain
    top-k MoE definition, for the config's table and for a trivial one."""
    c0 = CONFIGS[base]
    cfg = LayerConfig(**{**c0.__dict__, "n_shared": n_shared, "T": 96})
    wl = make_workload(cfg)
    x64 = oracle.widen(wl.x)
    cache = {}

    def weights_of(e):
        if e not in cache:
            cache[e] = tuple(oracle.widen(w) for w in wl.expert_weights(e))
        return cache[e]

    sh = wl.shared_weights()
    sh64 = None if sh is None else tuple(oracle.widen(w) for w in sh)
    ref = _dense_moe(wl, cfg.k, 1, weights_of, sh64)
    trivial = SimpleNamespace(E=cfg.E, R=1, N=1, rank_node=np.zeros(1, np.int32),
                              poll_weight=np.ones(1, np.uint32),
                              inst_ptr=np.arange(cfg.E + 1, dtype=np.int32),
                              inst_rank=np.zeros(cfg.E, np.int32))
    outs = []
    for pl, lr in ((wl.placement, 0), (wl.placement, 3), (trivial, 0)):
        res = oracle.route_permute(wl.logits, pl, cfg.k, lr)
        y = oracle.expert_ffn(res, x64, cfg.k, range(pl.R), weights_of)
        ys = oracle.shared_ffn(x64, sh64) if sh64 is not None else None
        outs.append(oracle.combine(y, res.perm.perm_pos, res.topk_weight, ys))
        np.testing.assert_allclose(outs[-1], ref, rtol=1e-10, atol=1e-12)
    # rank-share mode: the shares of all ranks add up to the routed part of the layer
    res = oracle.route_permute(wl.logits, wl.placement, cfg.k, 0)
    total = np.zeros_like(ref)
    for r in range(wl.placement.R):
        y = oracle.expert_ffn(res, x64, cfg.k, [r], weights_of)
        total += oracle.combine(y, res.perm.perm_pos, res.topk_weight)
    routed_ref = _dense_moe(wl, cfg.k, 1, weights_of, None)
    np.testing.assert_allclose(total, routed_ref, rtol=1e-10, atol=1e-12)
