"""One rank's share of a GRACE-MoE layer as a sequence of library calls with
preallocated buffers (no allocation, no host synchronisation per step)."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Tuple

import torch

from .binding import SHARE_STATE_INTS, GraceTable, _check, _dtype_code, grace_workspace_bytes, load_library

STAGES = ("route", "permute", "route_permute", "ffn_up", "ffn_down", "shared_up", "shared_down", "combine")


class GraceMoELayer:
    """route -> permute -> grouped expert FFN (local share) [-> shared FFN] -> combine.

    Weights are stacked in the slot order of `local_rank`
    (GraceTable.local_experts): w_gate, w_up [S,f,d]; w_down [S,d,f].
    Rows of other ranks are zero in `y` on every step (their results would arrive
    over the reverse all-to-all in a multi-GPU deployment): the rank's row range
    moves with the routing, so each step clears what an earlier step wrote outside
    the current range (grace_expert_ffn_up_share / _down_share do it inside the
    two projections' launches: no extra launch, no memset, the step stays capturable
    in a HIP graph).

    All buffers are allocated once; a step is four to six C calls whose argument lists
    are marshalled once per (logits, x, rr_in, rr_out, stream) and reused, so the
    host cost of a step is a few microseconds per call.
    """

    def __init__(self, table: GraceTable, local_rank: int, T: int, k: int, d: int, f: int, dtype: torch.dtype,
                 w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor, shared=None, renorm: int = 1,
                 device="cuda", policy: int = 0):
        self.table, self.local_rank, self.T, self.k, self.d, self.f = table, local_rank, T, k, d, f
        self.renorm = renorm
        self.policy = policy
        self.w = (w_gate, w_up, w_down)
        self.shared = shared
        self.n_shared = 0 if shared is None else shared[0].shape[0]
        S = w_gate.shape[0]
        if S and (tuple(w_gate.shape) != (S, f, d) or tuple(w_up.shape) != (S, f, d) or tuple(w_down.shape) != (S, d, f)):
            raise ValueError("weights must be w_gate/w_up [S,f,d] and w_down [S,d,f]")
        if shared is not None and (tuple(shared[0].shape) != (self.n_shared, f, d) or
                                   tuple(shared[1].shape) != (self.n_shared, f, d) or
                                   tuple(shared[2].shape) != (self.n_shared, d, f)):
            raise ValueError("shared weights must be [n,f,d], [n,f,d], [n,d,f]")
        for w in self.w + (tuple(shared) if shared is not None else ()):
            if w.dtype != dtype or not w.is_cuda or not w.is_contiguous():
                raise ValueError("weights must be contiguous device tensors of the layer dtype")
        i32 = dict(dtype=torch.int32, device=device)
        n = T * k
        self.route_out = (torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device=device),
                          torch.empty((T, k), **i32), torch.empty((table.E,), **i32))
        self.perm_out = (torch.empty(n, **i32), torch.empty(n, **i32), torch.empty(table.I + 1, **i32),
                         torch.empty(table.R + 1, **i32), torch.empty(table.N + 1, **i32))
        self.xp = torch.empty((n, d), dtype=dtype, device=device)
        self.y = torch.zeros((n, d), dtype=dtype, device=device)
        self.y_state = torch.zeros(SHARE_STATE_INTS, **i32)   # row range of y written by the previous step (grace_expert_ffn_up_share / _down_share)
        self.y_shared = torch.empty((T, d), dtype=dtype, device=device) if self.n_shared else None
        self.out = torch.empty((T, d), dtype=dtype, device=device)
        self.dt = _dtype_code(self.xp)
        self.ws = torch.empty(grace_workspace_bytes(T, table.E, k, table.I, d, f, self.n_shared, self.dt),
                              dtype=torch.uint8, device=device)
        # routing and permutation as one call (fewer launches than grace_route + grace_permute);
        # False: the two separate calls
        self.single_call_dispatch = True
        # with shared experts: the dispatch call builds only the index arrays and the row scatter rides
        # on the shared experts' gate+up projection (grace_shared_ffn_up_scatter), which then runs
        # ahead of the expert FFN; False: the scatter is part of the dispatch call
        self.fuse_scatter = self.n_shared > 0
        self.ws_shared = None
        self._key = None
        self._calls: List[Tuple[str, object, tuple]] = []

    def _marshal(self, logits, x, rr_in, rr_out, stream):
        lib = load_library()
        if logits.dtype != torch.float32 or tuple(logits.shape) != (self.T, self.table.E):
            raise ValueError("logits must be float32 [T, E]")
        if x.dtype != self.xp.dtype or tuple(x.shape) != (self.T, self.d):
            raise ValueError("x must be [T, d] of the layer dtype")
        for t in (logits, x, rr_in, rr_out):
            if t is not None and (not t.is_cuda or not t.is_contiguous()):
                raise ValueError("device tensors must be contiguous and live on the GPU")
        p = lambda t: None if t is None else C.c_void_p(t.data_ptr())
        st = C.c_void_p(stream)
        h, lr, T, k, d, f, dt = self.table.handle, self.local_rank, self.T, self.k, self.d, self.f, self.dt
        te, tw, ti, cnt = self.route_out
        pos, src, ioff, roff, noff = self.perm_out
        wg, wu, wd = self.w
        S = wg.shape[0]
        ws = p(self.ws)
        fuse = self.fuse_scatter and self.shared is not None
        xr, xpr = (None, None) if fuse else (p(x), p(self.xp))     # rows moved by the dispatch call, or not
        if self.single_call_dispatch:
            calls = [("route_permute", lib.grace_route_permute,
                      (h, lr, self.policy, p(logits), T, self.table.E, k, self.renorm, p(rr_in), p(rr_out), p(te), p(tw),
                       p(ti), p(cnt), xr, d, dt, p(pos), p(src), p(ioff), p(roff), p(noff), xpr, ws, st))]
        else:
            calls = [
                ("route", lib.grace_route, (h, lr, self.policy, p(logits), T, self.table.E, k, self.renorm, p(rr_in),
                                            p(rr_out), p(te), p(tw), p(ti), p(cnt), ws, st)),
                ("permute", lib.grace_permute, (h, p(ti), T, k, xr, d, dt, p(pos), p(src), p(ioff), p(roff), p(noff),
                                                xpr, ws, st)),
            ]
        if fuse:
            # the shared gate+up projection first: its hidden activation needs a workspace of its own,
            # because the expert FFN's hidden activation is written before the shared down projection runs
            sg, su, sd = self.shared
            if self.ws_shared is None:
                self.ws_shared = torch.empty(grace_workspace_bytes(T, 1, 1, 1, d, f, self.n_shared, dt), dtype=torch.uint8,
                                             device=self.xp.device)
            calls.append(("shared_up", lib.grace_shared_ffn_up_scatter, (p(x), T, d, f, self.n_shared, dt, p(sg), p(su),
                                                                        p(self.ws_shared), p(pos), k, p(self.xp), st)))
        calls += [
            ("ffn_up", lib.grace_expert_ffn_up_share, (h, lr, p(self.xp), p(ioff), T, k, d, f, dt, p(wg) if S else None,
                                                       p(wu) if S else None, p(self.y_state), ws, st)),
            ("ffn_down", lib.grace_expert_ffn_down_share, (h, lr, p(ioff), T, k, d, f, dt, p(wd) if S else None,
                                                           p(self.y), p(self.y_state), ws, st)),
        ]
        if self.shared is not None:
            sg, su, sd = self.shared
            if not fuse:
                calls.append(("shared_up", lib.grace_shared_ffn_up, (p(x), T, d, f, self.n_shared, dt, p(sg), p(su), ws, st)))
            calls.append(("shared_down", lib.grace_shared_ffn_down, (T, d, f, self.n_shared, dt, p(sd), p(self.y_shared),
                                                                     p(self.ws_shared) if fuse else ws, st)))
        calls.append(("combine", lib.grace_combine, (p(self.y), p(pos), p(tw), T, k, d, dt, p(self.y_shared),
                                                     p(self.out), st)))
        return calls

    def forward(self, logits: torch.Tensor, x: torch.Tensor, rr_in: Optional[torch.Tensor] = None,
                rr_out: Optional[torch.Tensor] = None,
                events: Optional[List[Tuple[str, torch.cuda.Event, torch.cuda.Event]]] = None,
                event_pool: Optional[List[torch.cuda.Event]] = None,
                timed_stages: Optional[Tuple[str, ...]] = None) -> torch.Tensor:
        """One layer step on torch's current stream.  With `events` (a list to
        append to), a pair of HIP events is recorded around every library call,
        or only around the calls named in `timed_stages`; `event_pool` supplies
        pre-created timing events (popped two per timed call)."""
        stream = torch.cuda.current_stream().cuda_stream
        key = (logits.data_ptr(), x.data_ptr(), None if rr_in is None else rr_in.data_ptr(),
               None if rr_out is None else rr_out.data_ptr(), stream)
        if key != self._key:
            self._calls = self._marshal(logits, x, rr_in, rr_out, stream)
            self._key = key
            self._keep = (logits, x, rr_in, rr_out)
        if events is None:
            for _, fn, args in self._calls:
                rc = fn(*args)
                if rc != 0:
                    _check(rc)
        else:
            for name, fn, args in self._calls:
                if timed_stages is not None and name not in timed_stages:
                    rc = fn(*args)
                    if rc != 0:
                        _check(rc)
                    continue
                if event_pool:
                    a, b = event_pool.pop(), event_pool.pop()
                else:
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                rc = fn(*args)
                b.record()
                if rc != 0:
                    _check(rc)
                events.append((name, a, b))
        return self.out

    def capture(self, logits: torch.Tensor, x: torch.Tensor, rr_in: Optional[torch.Tensor] = None,
                rr_out: Optional[torch.Tensor] = None) -> "torch.cuda.CUDAGraph":
        """Record one step into a HIP graph (the library enqueues only kernels: no
        memset nodes, no allocation, no synchronisation).  Replays read `logits`,
        `x`, `rr_in` in place and leave the result in `self.out`.  Call `forward`
        once before capturing so that one-time kernel attributes are set."""
        self.forward(logits, x, rr_in, rr_out)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.forward(logits, x, rr_in, rr_out)
        self._key = None  # the capture stream is gone; re-marshal on the next eager call
        return graph
