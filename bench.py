#!/usr/bin/env python3
"""Benchmark of the GRACE-MoE layer hot path on one MI355X.

A step is one pass of the whole path (route -> permute -> grouped expert FFN of
the local share -> [shared FFN] -> combine) over one seeded synthetic batch
already resident in HBM.  Prints one JSON line (see the design doc for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def cpu_baseline(wl, cfg, budget_s: float = 15.0):
    """The oracle as it stands, timed on this host for the same rank share.
    Integer steps, row gather and combine run on the full batch; the FFN runs on
    an evenly spaced sample of the local rows and is scaled to all of them."""
    import numpy as np
    import oracle

    threads = min(oracle.max_threads(), 16)
    lr = cfg.local_rank
    t0 = time.perf_counter()
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, lr)
    xp = oracle.gather_rows(wl.x, ref.perm.perm_src, cfg.k)
    t_meta = time.perf_counter() - t0
    lo, hi = int(ref.perm.rank_off[lr]), int(ref.perm.rank_off[lr + 1])
    m_loc = hi - lo
    x64 = oracle.widen(wl.x)
    cache = {}

    def weights_of(e):
        if e not in cache:
            cache[e] = tuple(oracle.widen(w) for w in wl.expert_weights(e))
        return cache[e]

    for g in range(int(ref.order.rank_ptr[lr]), int(ref.order.rank_ptr[lr + 1])):
        weights_of(int(ref.order.g_expert[g]))           # widening is set-up, not timed
    # calibrate on a few rows, then size the sample for the budget
    n_cal = min(m_loc, 4 * threads)
    rows = np.unique(np.linspace(lo, hi - 1, n_cal).astype(np.int64)) if m_loc else np.zeros(0, np.int64)
    t0 = time.perf_counter()
    oracle.expert_ffn(ref, x64, cfg.k, [lr], weights_of, threads=threads, rows=rows)
    t_cal = time.perf_counter() - t0
    per_row = t_cal / max(len(rows), 1)
    n_s = int(min(m_loc, max(n_cal, budget_s / max(per_row, 1e-9))))
    rows = np.unique(np.linspace(lo, hi - 1, n_s).astype(np.int64)) if m_loc else rows
    t0 = time.perf_counter()
    y = oracle.expert_ffn(ref, x64, cfg.k, [lr], weights_of, threads=threads, rows=rows)
    t_ffn_sample = time.perf_counter() - t0
    t_ffn = t_ffn_sample * (m_loc / max(len(rows), 1))
    t_shared = 0.0
    ys = None
    sh = wl.shared_weights()
    if sh is not None:
        sh64 = tuple(oracle.widen(w) for w in sh)
        toks = np.unique(np.linspace(0, cfg.T - 1, max(threads, int(budget_s / 3 / max(per_row * sh[0].shape[0], 1e-9))))
                         .astype(np.int64))
        toks = toks[:cfg.T]
        t0 = time.perf_counter()
        ys = oracle.shared_ffn(x64, sh64, threads=threads, rows=toks)
        t_shared = (time.perf_counter() - t0) * (cfg.T / len(toks))
    t0 = time.perf_counter()
    oracle.combine(y, ref.perm.perm_pos, ref.topk_weight, ys)
    t_comb = time.perf_counter() - t0
    total = t_meta + t_ffn + t_shared + t_comb
    return {
        "value": cfg.T / total, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": (f"route+permute+row gather+combine on all T={cfg.T} tokens ({t_meta + t_comb:.2f} s); expert FFN on "
                   f"{len(rows)} of {m_loc} local rows ({t_ffn_sample:.2f} s, scaled x{m_loc / max(len(rows), 1):.1f})"
                   + (f"; shared FFN sampled, scaled to {t_shared:.1f} s" if sh is not None else "")),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="olmoe", help="olmoe (BASELINE configs[1], default) | qwen | dsv2lite | mixtral | tiny | olmoe_decode64 | olmoe_decode512")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate", type=int, default=1,
                    help="also time the step cycling over this many independent sets of weights, inputs and buffers "
                         "(cold Infinity Cache; for working sets below its 256 MB)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy kernel (known traffic, for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2509_25041_amd as grace
    from workloads import CONFIGS, make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = CONFIGS[args.workload]
    wl = make_workload(cfg)
    pl = wl.placement
    lr = cfg.local_rank

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    table = grace.GraceTable.from_placement(pl)
    experts = table.local_experts(lr)
    wg, wu, wd = (dev(w) for w in wl.stacked_weights(list(experts)))
    sh = wl.shared_weights()
    shd = None if sh is None else tuple(dev(w) for w in sh)
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    layer = grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, tdt, wg, wu, wd, shared=shd)
    logits, x = dev(wl.logits), dev(wl.x)

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        layer.forward(logits, x)
    torch.cuda.synchronize()
    roff = layer.perm_out[3].cpu().numpy()
    m_loc = int(roff[lr + 1] - roff[lr])
    ioff = layer.perm_out[2].cpu().numpy()
    _, _, rank_ptr = table.instances()
    seg = np.diff(ioff[rank_ptr[lr]:rank_ptr[lr + 1] + 1])

    # timed region: exactly `steps` steps; a pair of HIP events around the call that launches the
    # dominant kernel, on the stream the kernels run on (every event is a marker packet between
    # two kernels, so the other calls are timed in a second, untimed pass below)
    events = []
    pool = [torch.cuda.Event(enable_timing=True) for _ in range(14 * args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layer.forward(logits, x, events=events, event_pool=pool, timed_stages=("ffn_up",))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    up_ms = float(np.mean([a.elapsed_time(b) for _, a, b in events]))

    # every call's time: the same steps again with events around all of them
    events = []
    for _ in range(args.steps):
        layer.forward(logits, x, events=events, event_pool=pool)
    torch.cuda.synchronize()
    per_stage = {}
    for name, a, b in events:
        per_stage.setdefault(name, []).append(a.elapsed_time(b))
    stage_ms = {k: float(np.mean(v)) for k, v in per_stage.items()}
    stage_ms["ffn_up_all_calls_timed"] = stage_ms["ffn_up"]
    stage_ms["ffn_up"] = up_ms

    # the same step as one HIP graph launch (extra information; `value` stays the eager loop)
    graph = layer.capture(logits, x)
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # the same step cycling over several independent copies of everything it touches, so that no
    # step finds its weights or buffers in the Infinity Cache
    rotated_ms = None
    if args.rotate > 1:
        sets = [(layer, logits, x)]
        for _ in range(args.rotate - 1):
            shc = None if shd is None else tuple(w.clone() for w in shd)
            sets.append((grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, tdt, wg.clone(), wu.clone(), wd.clone(),
                                             shared=shc), logits.clone(), x.clone()))
        for i in range(2 * len(sets)):
            L, lg, xx = sets[i % len(sets)]
            L.forward(lg, xx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            L, lg, xx = sets[i % len(sets)]
            L.forward(lg, xx)
        torch.cuda.synchronize()
        rotated_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    d, f, k, T = cfg.d, cfg.f, cfg.k, cfg.T
    el = 4 if cfg.dtype == "f32" else 2
    flops_up = 4.0 * d * f * m_loc           # gate + up projections: the dominant kernel
    flops_down = 2.0 * d * f * m_loc
    up_tflops = flops_up / (stage_ms["ffn_up"] * 1e-3) / 1e12
    bytes_permute = T * d * el + T * k * d * el + 12 * T * k
    bytes_combine = T * k * d * el + T * d * el * (2 if sh is not None else 1) + 8 * T * k
    bytes_route = T * (4 * cfg.E + 12 * k)

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = json.load(fh).get("ffn_up_hbm_bytes_per_launch")

    result = {
        "metric": "MoE-layer tokens/s on 1 GPU (route+permute+grouped FFN+combine)",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={T} d={d} E={cfg.E} f={f} top-{k}, {cfg.nodes}x{cfg.gpus_per_node} virtual "
                               f"ranks, local rank {lr}, Zipf s={cfg.zipf_s}", "local_rows": m_loc,
                   "local_slots": int(len(experts)), "rows_per_slot_min_max": [int(seg.min()), int(seg.max())] if len(seg) else [0, 0],
                   "n_shared": cfg.n_shared},
        "roofline": {"kernel": "gemm_bf16_persist_kernel<true> (grouped gate+up projection with fused SwiGLU)" if cfg.dtype == "bf16"
                     else "gemm_f32_kernel<true>",
                     "bound": "mfma", "achieved": up_tflops, "peak": PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else 157.3,
                     "unit": "TFLOP/s", "frac": up_tflops / (PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else 157.3),
                     "traffic": traffic, "avg_launch_ms": stage_ms["ffn_up"]},
        "stages_ms": stage_ms,
        "graph_replay_ms_per_step": graph_ms,
        "rotated_ms_per_step": rotated_ms,
        "rotate_sets": args.rotate,
        "stages_achieved": {
            "ffn_down_TFLOPs": flops_down / (stage_ms["ffn_down"] * 1e-3) / 1e12,
            "combine_GBs": bytes_combine / (stage_ms["combine"] * 1e-3) / 1e9,
            "hbm_peak_GBs": PEAK_HBM_GBS,
        },
    }
    if "route_permute" in stage_ms:      # decode-sized batch: routing and permutation are one call
        result["stages_achieved"]["route_permute_GBs"] = (bytes_route + bytes_permute) / (stage_ms["route_permute"] * 1e-3) / 1e9
    else:
        result["stages_achieved"]["route_GBs"] = bytes_route / (stage_ms["route"] * 1e-3) / 1e9
        result["stages_achieved"]["permute_GBs"] = bytes_permute / (stage_ms["permute"] * 1e-3) / 1e9
    # the HBM-bound calls together: algorithmic bytes of routing, permutation and combine over their summed time
    t_hbm = stage_ms["combine"] + (stage_ms["route_permute"] if "route_permute" in stage_ms
                                   else stage_ms["route"] + stage_ms["permute"])
    result["stages_achieved"]["route_permute_combine_GBs"] = (bytes_route + bytes_permute + bytes_combine) / (t_hbm * 1e-3) / 1e9
    if sh is not None:
        result["stages_achieved"]["shared_ffn_TFLOPs"] = 6.0 * d * f * cfg.n_shared * T / (stage_ms["shared_ffn"] * 1e-3) / 1e12
    if cfg.dtype == "bf16":
        # what the MFMA units sustain on this device (no global traffic), for context next to the nominal peak
        result["mfma_sustained_TFLOPs"] = {
            "constant_operands_registers": grace.grace_mfma_sustained(False, False),
            "random_operands_registers": grace.grace_mfma_sustained(True, False),
            "random_operands_lds_fed": grace.grace_mfma_sustained(True, True),
        }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, cfg)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
