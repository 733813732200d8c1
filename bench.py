#!/usr/bin/env python3
"""Benchmark of the GRACE-MoE layer hot path on one MI355X.

A step is one pass of the whole path (route -> permute -> grouped expert FFN of
the local share -> [shared FFN] -> combine) over one seeded synthetic batch
already resident in HBM.  Prints one JSON line: the headline workload (the
largest single-GPU configuration, DeepSeek-V2-Lite-shaped) with the roofline of
its dominant kernel, the other configurations under `per_config`, and the CPU
oracle timed on the host cores as `cpu_baseline`.
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
PEAK_F32_TFLOPS = 157.3     # fp32 vector
PEAK_HBM_GBS = 8000.0
HEADLINE = "dsv2lite"
OTHERS = ("olmoe", "mixtral", "qwen", "qwen3moe", "olmoe_decode64", "olmoe_decode512", "tiny")
ROTATE_BELOW_BYTES = 256 << 20   # Infinity Cache: smaller working sets are also timed over rotating buffer sets

KERNEL_OF_STAGE = {
    "ffn_up": "gemm_bf16_persist_kernel<true, *, EXPERTS> (grouped gate+up projection, fused SwiGLU)",
    "ffn_down": "gemm_bf16_persist_kernel<false, *, EXPERTS> (grouped down projection)",
    "shared_up": "gemm_bf16_persist_kernel<true, 1, SHARED> (shared experts' gate+up projection, fused SwiGLU; carries the row scatter)",
    "shared_down": "gemm_bf16_persist_kernel<false, 1, SHARED> (shared experts' down projection)",
    "combine": "combine_kernel (weighted gather to token order)",
    "route_permute": "topk + pick + positions + scatter_rows_kernel (one call; the row scatter moves the bytes)",
}


def host_info():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "cpu_model": model}


def cpu_baseline(wl, cfg, budget_s: float = 12.0, single_budget_s: float = 6.0):
    """The oracle as it stands, timed on this host for the same rank share, once on all the
    threads OpenMP gives it and once on a single thread.  Integer steps, row gather and combine
    run on the full batch (they are single-threaded loops in the oracle); the FFNs run on evenly
    spaced samples of the rows, sized to the time budgets, and are scaled to all rows."""
    import numpy as np
    import oracle

    threads = oracle.max_threads()
    lr = cfg.local_rank
    t0 = time.perf_counter()
    ref = oracle.route_permute(wl.logits, wl.placement, cfg.k, lr)
    oracle.gather_rows(wl.x, ref.perm.perm_src, cfg.k)
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
    sh = wl.shared_weights()
    sh64 = None if sh is None else tuple(oracle.widen(w) for w in sh)
    n_sh = 0 if sh is None else sh[0].shape[0]

    def spaced(a, b, n):
        return np.unique(np.linspace(a, b - 1, max(1, n)).astype(np.int64)) if b > a else np.zeros(0, np.int64)

    def ffn_leg(nthreads, budget):
        """-> (seconds for all local rows, seconds for all shared rows, text)"""
        cal = spaced(lo, hi, 4 * nthreads)
        t0 = time.perf_counter()
        oracle.expert_ffn(ref, x64, cfg.k, [lr], weights_of, threads=nthreads, rows=cal)
        per_row = (time.perf_counter() - t0) / max(len(cal), 1)
        share = budget * (m_loc / max(m_loc + n_sh * cfg.T, 1))
        rows = spaced(lo, hi, int(min(m_loc, max(len(cal), share / max(per_row, 1e-9)))))
        t0 = time.perf_counter()
        y = oracle.expert_ffn(ref, x64, cfg.k, [lr], weights_of, threads=nthreads, rows=rows)
        t_s = time.perf_counter() - t0
        t_ffn = t_s * (m_loc / max(len(rows), 1))
        text = f"expert FFN on {len(rows)} of {m_loc} local rows ({t_s:.2f} s, scaled x{m_loc / max(len(rows), 1):.1f})"
        t_shared, ys = 0.0, None
        if sh64 is not None:
            toks = spaced(0, cfg.T, int(min(cfg.T, max(nthreads, (budget - share) / max(per_row * n_sh, 1e-9)))))
            t0 = time.perf_counter()
            ys = oracle.shared_ffn(x64, sh64, threads=nthreads, rows=toks)
            t_s = time.perf_counter() - t0
            t_shared = t_s * (cfg.T / len(toks))
            text += f"; shared FFN on {len(toks)} of {cfg.T} tokens ({t_s:.2f} s, scaled x{cfg.T / len(toks):.1f})"
        return t_ffn, t_shared, text, y, ys

    t_ffn, t_shared, text, y, ys = ffn_leg(threads, budget_s)
    t0 = time.perf_counter()
    oracle.combine(y, ref.perm.perm_pos, ref.topk_weight, ys)
    t_comb = time.perf_counter() - t0
    total = t_meta + t_ffn + t_shared + t_comb
    t_ffn1, t_shared1, text1, _, _ = ffn_leg(1, single_budget_s)
    total1 = t_meta + t_ffn1 + t_shared1 + t_comb
    out = {
        "value": cfg.T / total, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": (f"{cfg.name}: route+permute+row gather+combine on all T={cfg.T} tokens ({t_meta + t_comb:.2f} s); " + text),
        "single_thread": {"value": cfg.T / total1, "unit": "tokens/s", "cores": 1, "sample": text1},
    }
    out.update(host_info())
    return out


def run_workload(name: str, steps: int, warmup: int, rotate: int = 0, mfma_probe: bool = False):
    """Times `steps` steps of one workload; returns (result dict, workload, config)."""
    import numpy as np
    import torch

    import paper_2509_25041_amd as grace
    from workloads import CONFIGS, make_workload

    cfg = CONFIGS[name]
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

    for _ in range(warmup):
        layer.forward(logits, x)
    torch.cuda.synchronize()
    roff = layer.perm_out[3].cpu().numpy()
    m_loc = int(roff[lr + 1] - roff[lr])
    ioff = layer.perm_out[2].cpu().numpy()
    _, _, rank_ptr = table.instances()
    seg = np.diff(ioff[rank_ptr[lr]:rank_ptr[lr + 1] + 1])

    d, f, k, T = cfg.d, cfg.f, cfg.k, cfg.T
    el = 4 if cfg.dtype == "f32" else 2
    peak_mm = PEAK_F32_TFLOPS if cfg.dtype == "f32" else PEAK_BF16_TFLOPS
    bytes_route = T * (4 * cfg.E + 12 * k)
    bytes_permute = T * d * el + T * k * d * el + 12 * T * k
    bytes_combine = T * k * d * el + T * d * el * (2 if sh is not None else 1) + 8 * T * k
    # with shared experts the row scatter rides on the shared gate+up projection's launch: the dispatch call
    # then builds only the index arrays
    fused_scatter = bool(getattr(layer, "fuse_scatter", False)) and sh is not None
    bytes_dispatch = bytes_route + (12 * T * k if fused_scatter else bytes_permute)
    # algorithmic work per launch of the kernel behind each call: (bound, amount, unit scale, peak)
    work = {
        "ffn_up": ("mfma", 4.0 * d * f * m_loc), "ffn_down": ("mfma", 2.0 * d * f * m_loc),
        "shared_up": ("mfma", 4.0 * d * f * cfg.n_shared * T), "shared_down": ("mfma", 2.0 * d * f * cfg.n_shared * T),
        "combine": ("hbm", float(bytes_combine)), "route_permute": ("hbm", float(bytes_dispatch)),
    }

    def achieved(stage, ms):
        bound, amount = work[stage]
        if bound == "mfma":
            return amount / (ms * 1e-3) / 1e12, peak_mm, "TFLOP/s"
        return amount / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"

    pool = [torch.cuda.Event(enable_timing=True) for _ in range(20 * (steps + 8))]

    def all_events_pass(n):
        events = []
        for _ in range(n):
            layer.forward(logits, x, events=events, event_pool=pool)
        torch.cuda.synchronize()
        per = {}
        for nm, a, b in events:
            per.setdefault(nm, []).append(a.elapsed_time(b))
        return {s: float(np.mean(v)) for s, v in per.items()}

    # which call holds the dominant kernel: a short pass with events around every call
    pre = all_events_pass(8)
    dominant = max((s for s in pre if s in work), key=lambda s: pre[s])

    # timed region: exactly `steps` steps; one pair of HIP events per step, around the call that
    # launches the dominant kernel, on the stream the kernels run on (every event is a marker
    # packet between two kernels, so the other calls are timed in a second pass below)
    events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        layer.forward(logits, x, events=events, event_pool=pool, timed_stages=(dominant,))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    dom_ms = float(np.mean([a.elapsed_time(b) for _, a, b in events]))

    stage_ms = all_events_pass(steps)
    stage_ms[dominant + "_all_calls_timed"] = stage_ms[dominant]
    stage_ms[dominant] = dom_ms

    # the same step as one HIP graph launch (extra information; `value` stays the eager loop)
    graph = layer.capture(logits, x)
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3 / steps
    del graph

    # working set of a step; below the Infinity Cache size the step is also timed cycling over
    # independent copies of everything it touches, so that no step finds its data in that cache
    ws_bytes = sum(t.numel() * t.element_size() for t in (wg, wu, wd, layer.xp, layer.y, layer.out, x, logits))
    ws_bytes += m_loc * f * el + (sum(w.numel() * w.element_size() for w in shd) if shd else 0)
    n_sets = rotate if rotate > 1 else (4 if ws_bytes < ROTATE_BELOW_BYTES else 0)
    rotated_ms = None
    if n_sets > 1:
        sets = [(layer, logits, x)]
        for _ in range(n_sets - 1):
            shc = None if shd is None else tuple(w.clone() for w in shd)
            sets.append((grace.GraceMoELayer(table, lr, cfg.T, cfg.k, cfg.d, cfg.f, tdt, wg.clone(), wu.clone(), wd.clone(),
                                             shared=shc), logits.clone(), x.clone()))
        for i in range(2 * len(sets)):
            L, lg, xx = sets[i % len(sets)]
            L.forward(lg, xx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            L, lg, xx = sets[i % len(sets)]
            L.forward(lg, xx)
        torch.cuda.synchronize()
        rotated_ms = (time.perf_counter() - t0) * 1e3 / steps
        del sets

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{name}.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = json.load(fh).get("per_stage_hbm_bytes_per_launch", {}).get(dominant)

    # the shared gate+up projection carries the row scatter: also time the projection by itself (outside the
    # timed region), so that the line shows what the scatter costs it
    carried = None
    if fused_scatter and dominant == "shared_up":
        import ctypes as C
        lib = grace.load_library()
        sg, su, _ = shd
        pp = lambda t: C.c_void_p(t.data_ptr())
        args = (pp(x), T, d, f, cfg.n_shared, layer.dt, pp(sg), pp(su), pp(layer.ws_shared),
                C.c_void_p(torch.cuda.current_stream().cuda_stream))
        evs = []
        for i in range(steps + 3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = lib.grace_shared_ffn_up(*args)
            e1.record()
            assert rc == 0
            if i >= 3:
                evs.append((e0, e1))
        torch.cuda.synchronize()
        alone_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))
        sc_bytes = float(T * d * el + T * k * d * el)
        carried = {"what": "row scatter of the dispatch permutation (grace_permute_rows), moved by the same launch",
                   "bytes": sc_bytes, "projection_alone_ms": alone_ms,
                   "projection_alone_frac": work[dominant][1] / (alone_ms * 1e-3) / 1e12 / peak_mm,
                   "cost_of_carrying_ms": dom_ms - alone_ms}
    ach, peak, unit = achieved(dominant, dom_ms)
    stages_achieved = {}
    for s in stage_ms:
        if s in work:
            a, p, u = achieved(s, stage_ms[s])
            stages_achieved[s] = {"achieved": a, "unit": u, "frac": a / p}
    if not fused_scatter:
        t_hbm = stage_ms.get("combine", 0.0) + stage_ms.get("route_permute", 0.0)
        stages_achieved["route_permute_combine"] = {
            "achieved": (bytes_route + bytes_permute + bytes_combine) / (t_hbm * 1e-3) / 1e9, "unit": "GB/s",
            "frac": (bytes_route + bytes_permute + bytes_combine) / (t_hbm * 1e-3) / 1e9 / PEAK_HBM_GBS}
    result = {
        "ms_per_step": ms_per_step,
        "tokens_per_s": T / (ms_per_step * 1e-3),
        "dtype": "bf16" if cfg.dtype == "bf16" else cfg.dtype,
        "config": {"workload": f"{cfg.name}: T={T} d={d} E={cfg.E} f={f} top-{k}, {cfg.nodes}x{cfg.gpus_per_node} virtual "
                               f"ranks, local rank {lr}, Zipf s={cfg.zipf_s}, {cfg.n_shared} shared experts",
                   "local_rows": m_loc, "local_slots": int(len(experts)),
                   "rows_per_slot_min_max": [int(seg.min()), int(seg.max())] if len(seg) else [0, 0],
                   "n_shared": cfg.n_shared, "working_set_MB": ws_bytes / 1e6,
                   "row_scatter": "carried by the shared gate+up projection's launch" if fused_scatter else "in the dispatch call"},
        "roofline": {"kernel": KERNEL_OF_STAGE[dominant] if cfg.dtype == "bf16" else f"{dominant} (fp32 FMA path)",
                     "stage": dominant, "bound": work[dominant][0], "achieved": ach, "peak": peak, "unit": unit,
                     "frac": ach / peak, "traffic": traffic, "avg_launch_ms": dom_ms,
                     "algorithmic_per_launch": work[dominant][1], "carries": carried},
        "stages_ms": stage_ms,
        "stages_achieved": stages_achieved,
        "graph_replay_ms_per_step": graph_ms,
        "rotated_ms_per_step": rotated_ms,
        "rotate_sets": n_sets,
    }
    if mfma_probe and cfg.dtype == "bf16":
        # what the MFMA units sustain on this device (no global traffic), for context next to the nominal peak
        result["mfma_sustained_TFLOPs"] = {
            "constant_operands_registers": grace.grace_mfma_sustained(False, False),
            "random_operands_registers": grace.grace_mfma_sustained(True, False),
            "random_operands_lds_fed": grace.grace_mfma_sustained(True, True),
        }
    del layer, wg, wu, wd, shd, logits, x, pool, events
    torch.cuda.empty_cache()
    return result, wl, cfg


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE,
                    help=f"{HEADLINE} (largest single-GPU configuration, default) | " + " | ".join(OTHERS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="time only --workload, not the other configurations")
    ap.add_argument("--per-config-steps", type=int, default=50)
    ap.add_argument("--rotate", type=int, default=0,
                    help="time the step also cycling over this many independent sets of weights, inputs and buffers "
                         "(default: 4 sets when the working set is below the 256 MB Infinity Cache)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy kernel (known traffic, for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head, wl, cfg = run_workload(args.workload, args.steps, args.warmup, args.rotate, mfma_probe=True)
    result = {
        "metric": "MoE-layer tokens/s on 1 GPU (route+permute+grouped FFN+combine)",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
    }
    for key in ("config", "roofline", "stages_ms", "stages_achieved", "graph_replay_ms_per_step", "rotated_ms_per_step",
                "rotate_sets", "mfma_sustained_TFLOPs"):
        if key in head:
            result[key] = head[key]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, cfg)
    del wl
    if not args.no_per_config:
        per = {}
        for name in OTHERS:
            if name == args.workload:
                continue
            r, _, _ = run_workload(name, args.per_config_steps, min(args.warmup, 10))
            per[name] = {"ms_per_step": r["ms_per_step"], "tokens_per_s": r["tokens_per_s"], "dtype": r["dtype"],
                         "steps": args.per_config_steps, "workload": r["config"]["workload"],
                         "local_rows": r["config"]["local_rows"],
                         "dominant": {q: r["roofline"][q] for q in ("kernel", "stage", "bound", "achieved", "unit", "frac",
                                                                   "avg_launch_ms")},
                         "stages_ms": r["stages_ms"], "stages_achieved": r["stages_achieved"],
                         "graph_replay_ms_per_step": r["graph_replay_ms_per_step"],
                         "rotated_ms_per_step": r["rotated_ms_per_step"], "rotate_sets": r["rotate_sets"]}
        result["per_config"] = per
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
