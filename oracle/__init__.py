"""CPU oracle for the GRACE-MoE layer hot path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``grace_oracle.c`` (plain C loops, fp64).  Only the
tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package; the product path never does.  Parity pins live in
``tests/test_oracle_*.py``.

A placement table is passed as any object with the attributes
``E, R, N, rank_node, poll_weight, inst_ptr, inst_rank`` (the CSR form of the
paper's expert placement + replica table and polling weights, Sections 4.1-4.3).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "grace_oracle.c")
_SO = os.path.join(_HERE, "libgrace_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP only parallelises independent rows)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-fno-fast-math", "-ffp-contract=off", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        for name in ("oracle_topk", "oracle_instance_order", "oracle_pick", "oracle_permute",
                     "oracle_gather_rows", "oracle_ffn_rows", "oracle_combine", "oracle_send_lists", "oracle_max_threads"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def max_threads() -> int:
    return int(lib().oracle_max_threads())


# -- storage widening ---------------------------------------------------------
def widen(a: np.ndarray) -> np.ndarray:
    """fp32 array or bf16 bit pattern (uint16) -> float64 values."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# -- O1 ------------------------------------------------------------------------
def topk(logits: np.ndarray, k: int, renorm: int = 1):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    te = np.empty((T, k), dtype=np.int32)
    tw = np.empty((T, k), dtype=np.float32)
    _check(lib().oracle_topk(_p(logits), C.c_int32(T), C.c_int32(E), C.c_int32(k), C.c_int32(renorm),
                             _p(te), _p(tw)), "topk")
    return te, tw


# -- O4 ------------------------------------------------------------------------
@dataclass
class InstanceOrder:
    csr_to_g: np.ndarray   # [I] CSR index -> dispatch-order id
    g_expert: np.ndarray   # [I]
    g_rank: np.ndarray     # [I]
    rank_ptr: np.ndarray   # [R+1]


def instance_order(pl) -> InstanceOrder:
    inst_ptr, inst_rank, rank_node = _i32(pl.inst_ptr), _i32(pl.inst_rank), _i32(pl.rank_node)
    I = int(inst_ptr[-1])
    o = InstanceOrder(np.empty(I, np.int32), np.empty(I, np.int32), np.empty(I, np.int32),
                      np.empty(pl.R + 1, np.int32))
    _check(lib().oracle_instance_order(C.c_int32(pl.E), C.c_int32(pl.R), _p(rank_node), _p(inst_ptr),
                                       _p(inst_rank), _p(o.csr_to_g), _p(o.g_expert), _p(o.g_rank),
                                       _p(o.rank_ptr)), "instance_order")
    return o


# -- O2 + O3 -------------------------------------------------------------------
def pick(topk_expert: np.ndarray, pl, local_rank: int, rr_in: Optional[np.ndarray] = None,
         order: Optional[InstanceOrder] = None, policy: int = 0):
    """-> (topk_inst [T,k] dispatch-order ids, expert_count [E], rr_out [E])."""
    te = _i32(topk_expert)
    T, k = te.shape
    order = order or instance_order(pl)
    rank_node, inst_ptr, inst_rank = _i32(pl.rank_node), _i32(pl.inst_ptr), _i32(pl.inst_rank)
    pw = np.ascontiguousarray(pl.poll_weight, dtype=np.uint32)
    rin = None if rr_in is None else np.ascontiguousarray(rr_in, dtype=np.uint32)
    rout = np.empty(pl.E, dtype=np.uint32)
    ti = np.empty((T, k), dtype=np.int32)
    cnt = np.empty(pl.E, dtype=np.int32)
    _check(lib().oracle_pick(_p(te), C.c_int32(T), C.c_int32(k), C.c_int32(pl.E), C.c_int32(pl.R),
                             _p(rank_node), _p(pw), _p(inst_ptr), _p(inst_rank), _p(order.csr_to_g),
                             C.c_int32(local_rank), C.c_int32(policy), _p(rin), _p(rout), _p(ti), _p(cnt)), "pick")
    return ti, cnt, rout


# -- O5 ------------------------------------------------------------------------
@dataclass
class Permutation:
    perm_pos: np.ndarray   # [T*k] assignment -> buffer position
    perm_src: np.ndarray   # [T*k] buffer position -> assignment
    inst_off: np.ndarray   # [I+1]
    rank_off: np.ndarray   # [R+1]
    node_off: np.ndarray   # [N+1]


def permute(topk_inst: np.ndarray, pl, order: Optional[InstanceOrder] = None) -> Permutation:
    ti = _i32(topk_inst)
    T, k = ti.shape
    order = order or instance_order(pl)
    I = int(pl.inst_ptr[-1])
    rank_node = _i32(pl.rank_node)
    pm = Permutation(np.empty(T * k, np.int32), np.empty(T * k, np.int32), np.empty(I + 1, np.int32),
                     np.empty(pl.R + 1, np.int32), np.empty(pl.N + 1, np.int32))
    _check(lib().oracle_permute(_p(ti), C.c_int32(T), C.c_int32(k), C.c_int32(I), C.c_int32(pl.R),
                                C.c_int32(pl.N), _p(order.g_rank), _p(rank_node), _p(pm.perm_pos),
                                _p(pm.perm_src), _p(pm.inst_off), _p(pm.rank_off), _p(pm.node_off)),
           "permute")
    return pm


def gather_rows(x: np.ndarray, perm_src: np.ndarray, k: int) -> np.ndarray:
    x = np.ascontiguousarray(x)
    src = _i32(perm_src)
    out = np.empty((src.shape[0], x.shape[1]), dtype=x.dtype)
    _check(lib().oracle_gather_rows(_p(x), C.c_int64(x.shape[1] * x.itemsize), _p(src),
                                    C.c_int64(src.shape[0]), C.c_int32(k), _p(out)), "gather_rows")
    return out


# -- send lists -----------------------------------------------------------------
@dataclass
class SendLists:
    rank_send_ptr: np.ndarray   # [R+1]
    rank_send_tok: np.ndarray   # [rank_send_ptr[R]]
    node_send_ptr: np.ndarray   # [N+1]
    node_send_tok: np.ndarray   # [node_send_ptr[N]]
    expand: np.ndarray          # [T*k]
    traffic: np.ndarray         # [4] int64


def send_lists(topk_inst: np.ndarray, pl, local_rank: int, order: Optional[InstanceOrder] = None) -> SendLists:
    ti = _i32(topk_inst)
    T, k = ti.shape
    order = order or instance_order(pl)
    rank_node = _i32(pl.rank_node)
    n = T * k
    out = SendLists(np.empty(pl.R + 1, np.int32), np.empty(max(n, 1), np.int32), np.empty(pl.N + 1, np.int32),
                    np.empty(max(n, 1), np.int32), np.empty(max(n, 1), np.int32), np.empty(4, np.int64))
    _check(lib().oracle_send_lists(_p(ti), C.c_int32(T), C.c_int32(k), C.c_int32(int(pl.inst_ptr[-1])),
                                   C.c_int32(pl.R), C.c_int32(pl.N), _p(order.g_rank), _p(rank_node),
                                   C.c_int32(local_rank), _p(out.rank_send_ptr), _p(out.rank_send_tok),
                                   _p(out.node_send_ptr), _p(out.node_send_tok), _p(out.expand), _p(out.traffic)),
           "send_lists")
    out.rank_send_tok = out.rank_send_tok[:out.rank_send_ptr[-1]]
    out.node_send_tok = out.node_send_tok[:out.node_send_ptr[-1]]
    out.expand = out.expand[:n]
    return out


# -- O6 ------------------------------------------------------------------------
def ffn_rows(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
             out: Optional[np.ndarray] = None, accumulate: bool = False, threads: int = 1) -> np.ndarray:
    """SwiGLU FFN of one expert on dense rows.  All arrays float64;
    w_gate, w_up: [f, d]; w_down: [d, f]; x: [n, d] -> y [n, d]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    wg = np.ascontiguousarray(w_gate, dtype=np.float64)
    wu = np.ascontiguousarray(w_up, dtype=np.float64)
    wd = np.ascontiguousarray(w_down, dtype=np.float64)
    n, d = x.shape
    f = wg.shape[0]
    assert wg.shape == (f, d) and wu.shape == (f, d) and wd.shape == (d, f)
    if out is None:
        assert not accumulate
        out = np.empty((n, d), dtype=np.float64)
    assert out.shape == (n, d) and out.dtype == np.float64 and out.flags.c_contiguous
    _check(lib().oracle_ffn_rows(_p(x), C.c_int64(n), C.c_int32(d), C.c_int32(f), _p(wg), _p(wu), _p(wd),
                                 _p(out), C.c_int32(1 if accumulate else 0), C.c_int32(threads)), "ffn_rows")
    return out


# -- O7 ------------------------------------------------------------------------
def combine(y: np.ndarray, perm_pos: np.ndarray, topk_weight: np.ndarray,
            y_shared: Optional[np.ndarray] = None) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float64)
    tw = np.ascontiguousarray(topk_weight, dtype=np.float32)
    T, k = tw.shape
    d = y.shape[1]
    pos = _i32(perm_pos)
    assert y.shape[0] == T * k and pos.shape[0] == T * k
    ys = None if y_shared is None else np.ascontiguousarray(y_shared, dtype=np.float64)
    out = np.empty((T, d), dtype=np.float64)
    _check(lib().oracle_combine(_p(y), _p(pos), _p(tw), C.c_int32(T), C.c_int32(k), C.c_int32(d),
                                _p(ys), _p(out)), "combine")
    return out


# -- whole layer ----------------------------------------------------------------
@dataclass
class LayerResult:
    topk_expert: np.ndarray
    topk_weight: np.ndarray
    topk_inst: np.ndarray
    expert_count: np.ndarray
    rr_out: np.ndarray
    perm: Permutation
    order: InstanceOrder
    y: Optional[np.ndarray] = None          # [T*k, d] float64, rows of other ranks zero in rank-share mode
    y_shared: Optional[np.ndarray] = None   # [T, d] float64
    out: Optional[np.ndarray] = None        # [T, d] float64


def route_permute(logits, pl, k: int, local_rank: int, renorm: int = 1, rr_in=None, policy: int = 0) -> LayerResult:
    te, tw = topk(logits, k, renorm)
    order = instance_order(pl)
    ti, cnt, rout = pick(te, pl, local_rank, rr_in, order, policy)
    pm = permute(ti, pl, order)
    return LayerResult(te, tw, ti, cnt, rout, pm, order)


def expert_ffn(res: LayerResult, x64: np.ndarray, k: int, ranks: Sequence[int], weights_of, threads: int = 1,
               rows: Optional[np.ndarray] = None) -> np.ndarray:
    """y [T*k, d] float64: rows of the instances hosted by `ranks` computed with
    their expert's weights, everything else zero.  weights_of(e) returns float64
    (w_gate, w_up, w_down).  `rows` (buffer positions) restricts the work to a
    sample; other rows stay zero."""
    n = res.perm.perm_src.shape[0]
    d = x64.shape[1]
    y = np.zeros((n, d), dtype=np.float64)
    want = None if rows is None else np.zeros(n, dtype=bool)
    if want is not None:
        want[np.asarray(rows, dtype=np.int64)] = True
    for r in ranks:
        for g in range(int(res.order.rank_ptr[r]), int(res.order.rank_ptr[r + 1])):
            lo, hi = int(res.perm.inst_off[g]), int(res.perm.inst_off[g + 1])
            ps = np.arange(lo, hi)
            if want is not None:
                ps = ps[want[lo:hi]]
            if ps.size == 0:
                continue
            wg, wu, wd = weights_of(int(res.order.g_expert[g]))
            xin = x64[res.perm.perm_src[ps] // k]
            y[ps] = ffn_rows(xin, wg, wu, wd, threads=threads)
    return y


def shared_ffn(x64: np.ndarray, shared64, threads: int = 1, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Sum of the always-on shared experts on every token (or the given rows)."""
    T, d = x64.shape
    ys = np.zeros((T, d), dtype=np.float64)
    if shared64 is None:
        return ys
    wg, wu, wd = shared64
    sel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    acc = np.zeros((sel.shape[0], d), dtype=np.float64)
    xin = np.ascontiguousarray(x64[sel])
    for s in range(wg.shape[0]):
        ffn_rows(xin, wg[s], wu[s], wd[s], out=acc, accumulate=True, threads=threads)
    ys[sel] = acc
    return ys
