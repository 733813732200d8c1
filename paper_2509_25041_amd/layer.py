"""One rank's share of a GRACE-MoE layer as a sequence of library calls with
preallocated buffers (no allocation, no host synchronisation per step)."""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import torch

from .binding import (GraceTable, _dtype_code, grace_combine, grace_expert_ffn_down, grace_expert_ffn_up,
                      grace_permute, grace_route, grace_shared_ffn, grace_workspace_bytes)

STAGES = ("route", "permute", "ffn_up", "ffn_down", "shared_ffn", "combine")


class GraceMoELayer:
    """route -> permute -> grouped expert FFN (local share) [-> shared FFN] -> combine.

    Weights are stacked in the slot order of `local_rank`
    (GraceTable.local_experts): w_gate, w_up [S,f,d]; w_down [S,d,f].
    Rows of other ranks stay zero in `y` (their results would arrive over the
    reverse all-to-all in a multi-GPU deployment).
    """

    def __init__(self, table: GraceTable, local_rank: int, T: int, k: int, d: int, f: int, dtype: torch.dtype,
                 w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor, shared=None, renorm: int = 1,
                 device="cuda"):
        self.table, self.local_rank, self.T, self.k, self.d, self.f = table, local_rank, T, k, d, f
        self.renorm = renorm
        self.w = (w_gate, w_up, w_down)
        self.shared = shared
        n_shared = 0 if shared is None else shared[0].shape[0]
        i32 = dict(dtype=torch.int32, device=device)
        n = T * k
        self.route_out = (torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device=device),
                          torch.empty((T, k), **i32), torch.empty((table.E,), **i32))
        self.perm_out = (torch.empty(n, **i32), torch.empty(n, **i32), torch.empty(table.I + 1, **i32),
                         torch.empty(table.R + 1, **i32), torch.empty(table.N + 1, **i32))
        self.xp = torch.empty((n, d), dtype=dtype, device=device)
        self.y = torch.zeros((n, d), dtype=dtype, device=device)
        self.y_shared = torch.empty((T, d), dtype=dtype, device=device) if n_shared else None
        self.out = torch.empty((T, d), dtype=dtype, device=device)
        dt = _dtype_code(self.xp)
        self.ws = torch.empty(grace_workspace_bytes(T, table.E, k, table.I, d, f, n_shared, dt), dtype=torch.uint8,
                              device=device)

    def forward(self, logits: torch.Tensor, x: torch.Tensor, rr_in: Optional[torch.Tensor] = None,
                rr_out: Optional[torch.Tensor] = None,
                events: Optional[List[Tuple[str, torch.cuda.Event, torch.cuda.Event]]] = None) -> torch.Tensor:
        """One layer step.  With `events` (a list to append to), a pair of HIP
        events is recorded around every library call on the current stream."""
        def timed(name, fn):
            if events is None:
                return fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            r = fn()
            b.record()
            events.append((name, a, b))
            return r

        te, tw, ti, cnt = timed("route", lambda: grace_route(self.table, self.local_rank, logits, self.k, self.renorm,
                                                             rr_in, rr_out, ws=self.ws, out=self.route_out))
        pos, src, ioff, roff, noff, xp = timed("permute", lambda: grace_permute(self.table, ti, x, ws=self.ws,
                                                                                out=self.perm_out, xp=self.xp))
        timed("ffn_up", lambda: grace_expert_ffn_up(self.table, self.local_rank, xp, ioff, self.T, self.k, self.w[0],
                                                    self.w[1], self.ws))
        timed("ffn_down", lambda: grace_expert_ffn_down(self.table, self.local_rank, ioff, self.T, self.k, self.w[2],
                                                        self.y, self.ws))
        if self.shared is not None:
            timed("shared_ffn", lambda: grace_shared_ffn(x, *self.shared, y_shared=self.y_shared, ws=self.ws))
        return timed("combine", lambda: grace_combine(self.y, pos, tw, self.y_shared, out=self.out))
