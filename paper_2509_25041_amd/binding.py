"""ctypes binding of the C ABI declared in include/grace_moe.h."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

from . import build as _build

GRACE_F32, GRACE_BF16 = 0, 1
GRACE_POLICY_TAR, GRACE_POLICY_WRR = 0, 1
SHARE_STATE_INTS = 8      # GRACE_SHARE_STATE_INTS
_STATUS = {0: "GRACE_OK", -1: "GRACE_EINVAL", -2: "GRACE_ESHAPE", -3: "GRACE_ETABLE", -4: "GRACE_ENOMEM",
           -5: "GRACE_EHIP"}

EXPORTS = ("grace_table_validate", "grace_table_create", "grace_table_destroy", "grace_table_info",
           "grace_table_instances", "grace_table_local_experts", "grace_table_set_fold_limits", "grace_workspace_bytes",
           "grace_route",
           "grace_permute", "grace_permute_rows", "grace_route_permute", "grace_route_permute_static", "grace_send_lists", "grace_expert_ffn", "grace_expert_ffn_up",
           "grace_expert_ffn_down", "grace_expert_ffn_up_share", "grace_expert_ffn_down_share",
           "grace_shared_ffn", "grace_shared_ffn_up", "grace_shared_ffn_down", "grace_shared_ffn_up_scatter", "grace_combine", "grace_mfma_sustained",
           "grace_last_error")

_lib: Optional[C.CDLL] = None


class GraceError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{_STATUS.get(status, status)}: {text}")
        self.status = status


def library_path() -> str:
    return _build.LIB


def load_library() -> C.CDLL:
    """Load the in-tree shared library.  It is built first when it is absent or older than any of
    its sources, so a forgotten rebuild cannot put yesterday's kernels under today's tests; where the
    sources are newer and no compiler is available the call fails instead of loading the old code."""
    global _lib
    if _lib is not None:
        return _lib
    if _build.is_stale():
        _build.build()
    lib = C.CDLL(_build.LIB)
    vp, i32, u64 = C.c_void_p, C.c_int32, C.c_size_t
    lib.grace_last_error.restype = C.c_char_p
    lib.grace_last_error.argtypes = []
    lib.grace_table_validate.argtypes = [i32, i32, i32, vp, vp, vp, vp]
    lib.grace_table_create.argtypes = [C.POINTER(vp), i32, i32, i32, vp, vp, vp, vp, vp]
    lib.grace_table_destroy.argtypes = [vp]
    lib.grace_table_info.argtypes = [vp] + [C.POINTER(i32)] * 5
    lib.grace_table_instances.argtypes = [vp, vp, vp, vp]
    lib.grace_table_local_experts.argtypes = [vp, i32, vp, C.POINTER(i32)]
    lib.grace_table_set_fold_limits.argtypes = [vp, i32, i32]
    lib.grace_workspace_bytes.restype = u64
    lib.grace_workspace_bytes.argtypes = [i32] * 7 + [C.c_int]
    lib.grace_route.argtypes = [vp, i32, C.c_int, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.grace_permute.argtypes = [vp, vp, i32, i32, vp, i32, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.grace_permute_rows.argtypes = [vp, vp, i32, i32, i32, C.c_int, vp, vp]
    lib.grace_route_permute.argtypes = [vp, i32, C.c_int, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                        vp, i32, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.grace_route_permute_static.argtypes = [vp, i32, C.c_int, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                               vp, i32, C.c_int, vp, vp, vp, vp, vp, vp, vp]
    lib.grace_send_lists.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.grace_expert_ffn.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp, vp, vp]
    lib.grace_expert_ffn_up.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp]
    lib.grace_expert_ffn_down.argtypes = [vp, i32, vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp]
    lib.grace_expert_ffn_up_share.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp, vp]
    lib.grace_expert_ffn_down_share.argtypes = [vp, i32, vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp, vp]
    lib.grace_shared_ffn.argtypes = [vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp, vp, vp]
    lib.grace_shared_ffn_up.argtypes = [vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp]
    lib.grace_shared_ffn_up_scatter.argtypes = [vp, i32, i32, i32, i32, C.c_int, vp, vp, vp, vp, i32, vp, vp]
    lib.grace_shared_ffn_down.argtypes = [i32, i32, i32, i32, C.c_int, vp, vp, vp, vp]
    lib.grace_combine.argtypes = [vp, vp, vp, i32, i32, i32, C.c_int, vp, vp, vp]
    lib.grace_mfma_sustained.argtypes = [i32, i32, C.POINTER(C.c_double), vp]
    for name in EXPORTS:
        if name not in ("grace_last_error", "grace_workspace_bytes"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def grace_last_error() -> str:
    return load_library().grace_last_error().decode()


def _check(status: int) -> None:
    if status != 0:
        raise GraceError(status, grace_last_error())


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dp(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device tensors must be contiguous and live on the GPU")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GRACE_F32
    if t.dtype == torch.bfloat16:
        return GRACE_BF16
    raise ValueError(f"unsupported dtype {t.dtype}")


def grace_table_validate(E, R, N, rank_node, poll_weight, inst_ptr, inst_rank) -> None:
    """Host-only validation of a placement table; raises GraceError."""
    a = (_host(rank_node, np.int32), _host(poll_weight, np.uint32), _host(inst_ptr, np.int32),
         _host(inst_rank, np.int32))
    _check(load_library().grace_table_validate(E, R, N, *[_hp(x) for x in a]))


def grace_workspace_bytes(T, E, k, I, d=0, f=0, n_shared=0, dt=GRACE_BF16) -> int:
    return int(load_library().grace_workspace_bytes(T, E, k, I, d, f, n_shared, dt))


class GraceTable:
    """Owns a grace_table (device copy on the current GPU)."""

    def __init__(self, E, R, N, rank_node, poll_weight, inst_ptr, inst_rank):
        lib = load_library()
        a = (_host(rank_node, np.int32), _host(poll_weight, np.uint32), _host(inst_ptr, np.int32),
             _host(inst_rank, np.int32))
        h = C.c_void_p()
        _check(lib.grace_table_create(C.byref(h), E, R, N, *[_hp(x) for x in a], _stream()))
        self._h = h
        v = [C.c_int32() for _ in range(5)]
        _check(lib.grace_table_info(h, *[C.byref(x) for x in v]))
        self.E, self.R, self.N, self.I, self.max_local_slots = (int(x.value) for x in v)

    @classmethod
    def from_placement(cls, pl) -> "GraceTable":
        return cls(pl.E, pl.R, pl.N, pl.rank_node, pl.poll_weight, pl.inst_ptr, pl.inst_rank)

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("table was destroyed")
        return self._h

    def instances(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """(inst_expert [I], inst_rank [I], rank_ptr [R+1]) in dispatch order."""
        ie, ir, rp = np.empty(self.I, np.int32), np.empty(self.I, np.int32), np.empty(self.R + 1, np.int32)
        _check(load_library().grace_table_instances(self.handle, _hp(ie), _hp(ir), _hp(rp)))
        return ie, ir, rp

    def local_experts(self, rank: int) -> np.ndarray:
        buf = np.empty(max(self.max_local_slots, 1), np.int32)
        n = C.c_int32()
        _check(load_library().grace_table_local_experts(self.handle, rank, _hp(buf), C.byref(n)))
        return buf[:n.value].copy()

    def set_fold_limits(self, one_level_max: int = -1, two_level_max: int = -1) -> None:
        """Switch points of the index kernels' prefix-count algorithms for calls with this table
        (negative: defaults); see grace_moe.h."""
        _check(load_library().grace_table_set_fold_limits(self.handle, one_level_max, two_level_max))

    def destroy(self) -> None:
        if getattr(self, "_h", None) is not None:
            h, self._h = self._h, None
            _check(load_library().grace_table_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _ws(ws: Optional[torch.Tensor], nbytes: int, device) -> torch.Tensor:
    if ws is None:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    elif ws.numel() * ws.element_size() < nbytes:
        raise ValueError(f"workspace too small: need {nbytes} bytes")
    return ws


def grace_route(table: GraceTable, local_rank: int, logits: torch.Tensor, k: int, renorm: int = 1,
                rr_in: Optional[torch.Tensor] = None, rr_out: Optional[torch.Tensor] = None,
                ws: Optional[torch.Tensor] = None, out=None, policy: int = GRACE_POLICY_TAR):
    """-> (topk_expert [T,k] i32, topk_weight [T,k] f32, topk_inst [T,k] i32, expert_count [E] i32)."""
    T, E = logits.shape
    dev = logits.device
    if logits.dtype != torch.float32:
        raise ValueError("logits must be float32")
    if out is None:
        out = (torch.empty((T, k), dtype=torch.int32, device=dev), torch.empty((T, k), dtype=torch.float32, device=dev),
               torch.empty((T, k), dtype=torch.int32, device=dev), torch.empty((E,), dtype=torch.int32, device=dev))
    te, tw, ti, cnt = out
    ws = _ws(ws, grace_workspace_bytes(T, E, max(k, 1), table.I), dev)
    _check(load_library().grace_route(table.handle, local_rank, policy, _dp(logits), T, E, k, renorm, _dp(rr_in), _dp(rr_out),
                                      _dp(te), _dp(tw), _dp(ti), _dp(cnt), _dp(ws), _stream()))
    return te, tw, ti, cnt


def grace_permute(table: GraceTable, topk_inst: torch.Tensor, x: Optional[torch.Tensor], ws: Optional[torch.Tensor] = None,
                  out=None, xp: Optional[torch.Tensor] = None):
    """-> (perm_pos, perm_src, inst_off, rank_off, node_off, xp)."""
    T, k = topk_inst.shape
    dev = topk_inst.device
    if out is None:
        i32 = dict(dtype=torch.int32, device=dev)
        out = (torch.empty(T * k, **i32), torch.empty(T * k, **i32), torch.empty(table.I + 1, **i32),
               torch.empty(table.R + 1, **i32), torch.empty(table.N + 1, **i32))
    pos, src, ioff, roff, noff = out
    d, dt = 0, GRACE_BF16
    if x is not None:
        d, dt = x.shape[1], _dtype_code(x)
        if xp is None:
            xp = torch.empty((T * k, d), dtype=x.dtype, device=dev)
    ws = _ws(ws, grace_workspace_bytes(T, table.E, k, table.I), dev)
    _check(load_library().grace_permute(table.handle, _dp(topk_inst), T, k, _dp(x), d, dt, _dp(pos), _dp(src), _dp(ioff),
                                        _dp(roff), _dp(noff), _dp(xp) if x is not None else None, _dp(ws), _stream()))
    return pos, src, ioff, roff, noff, xp


def grace_route_permute(table: GraceTable, local_rank: int, logits: torch.Tensor, k: int, x: Optional[torch.Tensor],
                        renorm: int = 1, rr_in: Optional[torch.Tensor] = None, rr_out: Optional[torch.Tensor] = None,
                        ws: Optional[torch.Tensor] = None, policy: int = GRACE_POLICY_TAR):
    """grace_route and grace_permute as one call with fewer launches (see grace_moe.h).
    -> ((topk_expert, topk_weight, topk_inst, expert_count), (perm_pos, perm_src, inst_off, rank_off, node_off, xp))."""
    T, E = logits.shape
    dev = logits.device
    if logits.dtype != torch.float32:
        raise ValueError("logits must be float32")
    i32 = dict(dtype=torch.int32, device=dev)
    te, tw = torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device=dev)
    ti, cnt = torch.empty((T, k), **i32), torch.empty((E,), **i32)
    pos, src = torch.empty(T * k, **i32), torch.empty(T * k, **i32)
    ioff, roff, noff = torch.empty(table.I + 1, **i32), torch.empty(table.R + 1, **i32), torch.empty(table.N + 1, **i32)
    d, dt, xp = 0, GRACE_BF16, None
    if x is not None:
        d, dt = x.shape[1], _dtype_code(x)
        xp = torch.empty((T * k, d), dtype=x.dtype, device=dev)
    ws = _ws(ws, grace_workspace_bytes(T, E, max(k, 1), table.I), dev)
    _check(load_library().grace_route_permute(table.handle, local_rank, policy, _dp(logits), T, E, k, renorm, _dp(rr_in),
                                              _dp(rr_out), _dp(te), _dp(tw), _dp(ti), _dp(cnt), _dp(x), d, dt, _dp(pos),
                                              _dp(src), _dp(ioff), _dp(roff), _dp(noff),
                                              _dp(xp) if x is not None else None, _dp(ws), _stream()))
    return (te, tw, ti, cnt), (pos, src, ioff, roff, noff, xp)


def grace_route_permute_static(table: GraceTable, local_rank: int, logits: torch.Tensor, k: int, x: Optional[torch.Tensor],
                               renorm: int = 1, rr_in: Optional[torch.Tensor] = None, rr_out: Optional[torch.Tensor] = None,
                               policy: int = GRACE_POLICY_TAR, out=None):
    """grace_route_permute on the library's static scratch instead of a workspace (see grace_moe.h).
    `out` = ((topk_expert, topk_weight, topk_inst, expert_count), (perm_pos, perm_src, inst_off, rank_off,
    node_off, xp)) reuses the caller's output tensors; the C call itself allocates nothing."""
    T, E = logits.shape
    dev = logits.device
    if logits.dtype != torch.float32:
        raise ValueError("logits must be float32")
    d, dt = (0, GRACE_BF16) if x is None else (x.shape[1], _dtype_code(x))
    if out is None:
        i32 = dict(dtype=torch.int32, device=dev)
        out = ((torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device=dev), torch.empty((T, k), **i32),
                torch.empty((E,), **i32)),
               (torch.empty(T * k, **i32), torch.empty(T * k, **i32), torch.empty(table.I + 1, **i32),
                torch.empty(table.R + 1, **i32), torch.empty(table.N + 1, **i32),
                None if x is None else torch.empty((T * k, d), dtype=x.dtype, device=dev)))
    (te, tw, ti, cnt), (pos, src, ioff, roff, noff, xp) = out
    _check(load_library().grace_route_permute_static(table.handle, local_rank, policy, _dp(logits), T, E, k, renorm, _dp(rr_in),
                                                     _dp(rr_out), _dp(te), _dp(tw), _dp(ti), _dp(cnt), _dp(x), d, dt, _dp(pos),
                                                     _dp(src), _dp(ioff), _dp(roff), _dp(noff),
                                                     _dp(xp) if x is not None else None, _stream()))
    return out


def grace_send_lists(table: GraceTable, local_rank: int, topk_inst: torch.Tensor, ws: Optional[torch.Tensor] = None):
    """-> (rank_send_ptr [R+1], rank_send_tok [T*k], node_send_ptr [N+1], node_send_tok [T*k], expand [T*k],
    traffic [4] int64); see grace_moe.h."""
    T, k = topk_inst.shape
    dev = topk_inst.device
    i32 = dict(dtype=torch.int32, device=dev)
    rp, rt = torch.empty(table.R + 1, **i32), torch.full((T * k,), -1, **i32)
    np_, nt = torch.empty(table.N + 1, **i32), torch.full((T * k,), -1, **i32)
    ex = torch.empty(T * k, **i32)
    tr = torch.empty(4, dtype=torch.int64, device=dev)
    ws = _ws(ws, grace_workspace_bytes(T, table.E, k, table.I), dev)
    _check(load_library().grace_send_lists(table.handle, local_rank, _dp(topk_inst), T, k, _dp(rp), _dp(rt), _dp(np_),
                                           _dp(nt), _dp(ex), _dp(tr), _dp(ws), _stream()))
    return rp, rt, np_, nt, ex, tr


def grace_expert_ffn(table: GraceTable, rank: int, xp: torch.Tensor, inst_off: torch.Tensor, T: int, k: int,
                     w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor, y: Optional[torch.Tensor] = None,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y [T*k, d]; only the rows of `rank` are written (a fresh y starts as zeros)."""
    d = xp.shape[1]
    dt = _dtype_code(xp)
    S = w_gate.shape[0]
    f = w_gate.shape[1] if S > 0 else (w_down.shape[2] if w_down.dim() == 3 else 8)
    if S > 0 and (tuple(w_gate.shape) != (S, f, d) or tuple(w_up.shape) != (S, f, d) or tuple(w_down.shape) != (S, d, f)):
        raise ValueError("weights must be w_gate/w_up [S,f,d] and w_down [S,d,f]")
    for w in (w_gate, w_up, w_down):
        if w.dtype != xp.dtype:
            raise ValueError("weights and activations must share one dtype")
    if y is None:
        y = torch.zeros((T * k, d), dtype=xp.dtype, device=xp.device)
    ws = _ws(ws, grace_workspace_bytes(T, table.E, k, table.I, d, f, 0, dt), xp.device)
    _check(load_library().grace_expert_ffn(table.handle, rank, _dp(xp), _dp(inst_off), T, k, d, f, dt,
                                           _dp(w_gate) if S else None, _dp(w_up) if S else None,
                                           _dp(w_down) if S else None, _dp(y), _dp(ws), _stream()))
    return y


def grace_expert_ffn_up(table: GraceTable, rank: int, xp: torch.Tensor, inst_off: torch.Tensor, T: int, k: int,
                        w_gate: torch.Tensor, w_up: torch.Tensor, ws: torch.Tensor) -> None:
    S, f, d = w_gate.shape
    _check(load_library().grace_expert_ffn_up(table.handle, rank, _dp(xp), _dp(inst_off), T, k, d, f, _dtype_code(xp),
                                              _dp(w_gate) if S else None, _dp(w_up) if S else None, _dp(ws), _stream()))


def grace_expert_ffn_down(table: GraceTable, rank: int, inst_off: torch.Tensor, T: int, k: int, w_down: torch.Tensor,
                          y: torch.Tensor, ws: torch.Tensor) -> None:
    S, d, f = w_down.shape
    _check(load_library().grace_expert_ffn_down(table.handle, rank, _dp(inst_off), T, k, d, f, _dtype_code(y),
                                                _dp(w_down) if S else None, _dp(y), _dp(ws), _stream()))


def grace_expert_ffn_up_share(table: GraceTable, rank: int, xp: torch.Tensor, inst_off: torch.Tensor, T: int, k: int,
                              w_gate: torch.Tensor, w_up: torch.Tensor, state: torch.Tensor, ws: torch.Tensor) -> None:
    """grace_expert_ffn_up that also records the rank's row range of this step in `state` (first half of
    the pair with grace_expert_ffn_down_share); see grace_moe.h."""
    if state.dtype != torch.int32 or state.numel() < SHARE_STATE_INTS:
        raise ValueError(f"state must hold {SHARE_STATE_INTS} int32")
    S, f, d = w_gate.shape
    _check(load_library().grace_expert_ffn_up_share(table.handle, rank, _dp(xp), _dp(inst_off), T, k, d, f, _dtype_code(xp),
                                                    _dp(w_gate) if S else None, _dp(w_up) if S else None, _dp(state),
                                                    _dp(ws), _stream()))


def grace_expert_ffn_down_share(table: GraceTable, rank: int, inst_off: torch.Tensor, T: int, k: int, w_down: torch.Tensor,
                                y: torch.Tensor, state: torch.Tensor, ws: torch.Tensor) -> None:
    """grace_expert_ffn_down that also zeroes the rows the previous step (same `state`: SHARE_STATE_INTS
    int32 on the device, zero before the first step, kept by grace_expert_ffn_up_share) wrote outside the
    rank's current row range; see grace_moe.h."""
    if state.dtype != torch.int32 or state.numel() < SHARE_STATE_INTS:
        raise ValueError(f"state must hold {SHARE_STATE_INTS} int32")
    S, d, f = w_down.shape
    _check(load_library().grace_expert_ffn_down_share(table.handle, rank, _dp(inst_off), T, k, d, f, _dtype_code(y),
                                                      _dp(w_down) if S else None, _dp(y), _dp(state), _dp(ws), _stream()))


def grace_shared_ffn(x: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor,
                     y_shared: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    T, d = x.shape
    n_shared, f, _ = w_gate.shape
    dt = _dtype_code(x)
    if tuple(w_up.shape) != (n_shared, f, d) or tuple(w_down.shape) != (n_shared, d, f):
        raise ValueError("weights must be w_gate/w_up [n,f,d] and w_down [n,d,f]")
    if y_shared is None:
        y_shared = torch.empty((T, d), dtype=x.dtype, device=x.device)
    ws = _ws(ws, grace_workspace_bytes(T, 1, 1, 1, d, f, n_shared, dt), x.device)
    _check(load_library().grace_shared_ffn(_dp(x), T, d, f, n_shared, dt, _dp(w_gate), _dp(w_up), _dp(w_down),
                                           _dp(y_shared), _dp(ws), _stream()))
    return y_shared


def grace_shared_ffn_up(x: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor, ws: torch.Tensor) -> None:
    """First launch of grace_shared_ffn: the hidden activation of all T rows into ws; see grace_moe.h."""
    T, d = x.shape
    n_shared, f, _ = w_gate.shape
    if tuple(w_up.shape) != (n_shared, f, d):
        raise ValueError("weights must be w_gate/w_up [n,f,d]")
    _check(load_library().grace_shared_ffn_up(_dp(x), T, d, f, n_shared, _dtype_code(x), _dp(w_gate), _dp(w_up), _dp(ws),
                                              _stream()))


def grace_shared_ffn_down(w_down: torch.Tensor, ws: torch.Tensor, T: int,
                          y_shared: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Second launch of grace_shared_ffn: reads the hidden activation grace_shared_ffn_up left in ws; see grace_moe.h."""
    n_shared, d, f = w_down.shape
    if y_shared is None:
        y_shared = torch.empty((T, d), dtype=w_down.dtype, device=w_down.device)
    _check(load_library().grace_shared_ffn_down(T, d, f, n_shared, _dtype_code(w_down), _dp(w_down), _dp(y_shared), _dp(ws),
                                                _stream()))
    return y_shared


def grace_permute_rows(x: torch.Tensor, perm_pos: torch.Tensor, k: int, xp: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The row movement of grace_permute alone: xp[perm_pos[t*k+j]] = x[t]; see grace_moe.h."""
    T, d = x.shape
    if xp is None:
        xp = torch.empty((T * k, d), dtype=x.dtype, device=x.device)
    _check(load_library().grace_permute_rows(_dp(x), _dp(perm_pos), T, k, d, _dtype_code(x), _dp(xp), _stream()))
    return xp


def grace_shared_ffn_up_scatter(x: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor, ws: torch.Tensor,
                                perm_pos: torch.Tensor, k: int, xp: torch.Tensor) -> None:
    """grace_shared_ffn_up (hidden activation into ws) and grace_permute_rows (rows into xp) as one call; see
    grace_moe.h."""
    T, d = x.shape
    n_shared, f, _ = w_gate.shape
    _check(load_library().grace_shared_ffn_up_scatter(_dp(x), T, d, f, n_shared, _dtype_code(x), _dp(w_gate), _dp(w_up),
                                                      _dp(ws), _dp(perm_pos), k, _dp(xp), _stream()))


def grace_combine(y: torch.Tensor, perm_pos: torch.Tensor, topk_weight: torch.Tensor,
                  y_shared: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    T, k = topk_weight.shape
    d = y.shape[1]
    if out is None:
        out = torch.empty((T, d), dtype=y.dtype, device=y.device)
    _check(load_library().grace_combine(_dp(y), _dp(perm_pos), _dp(topk_weight), T, k, d, _dtype_code(y), _dp(y_shared),
                                        _dp(out), _stream()))
    return out


def grace_mfma_sustained(random_operands: bool = True, lds_fed: bool = True) -> float:
    """Sustained bf16 MFMA TFLOP/s of the current device (see grace_moe.h)."""
    out = C.c_double()
    _check(load_library().grace_mfma_sustained(int(random_operands), int(lds_fed), C.byref(out), _stream()))
    return float(out.value)
