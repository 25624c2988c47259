"""Benchmark of the batched constrained-compression dynamic program (Alg. 1) on one MI355X.

One "step" = one whole solve of the workload's K candidates: table fill (Eq. 2-3), final
argmin over t and walk back, inputs already resident in device memory.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload rn50_k1024]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Plain (non-packed) vector ALU peak of the chip: 256 compute units x 4 SIMDs x 16 lanes, one
# 32-bit lane-operation per lane per clock at 2.4 GHz.  (The published 157.3 TFLOP/s fp32 vector
# figure is this number x 2 for fused multiply-add x 2 for packed fp32; neither applies to an
# add / compare / select chain.)
ALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9
# One update of Alg. 1's inner loop: an fp32 add and an fp32 min when D itself is recorded;
# an fp32 add, a compare and two selects (value, level) when the level is tracked per cell.
LANE_OPS_PER_UPDATE = {"d": 2, "level": 4}
# LDS: one 4-byte read of the shifted previous row per update; 128 bytes per clock per compute
# unit for 32-bit reads (64 lanes in two clocks).
LDS_PEAK_BYTES = 256 * 128 * 2.4e9
LDS_BYTES_PER_UPDATE = 4
# HBM bytes per launch of the fill kernel, from FETCH_SIZE / WRITE_SIZE counter runs scaled by a
# plain copy of known size (profiles/dp_fill_rn50_k1024_*.md).  None where not measured.
MEASURED_TRAFFIC_BYTES = {("rn50_k1024", "d"): 957e6, ("rn50_k1024", "level"): 246e6}


def executed_updates_per_candidate(tau: np.ndarray, B: int, merge_equal_times: bool) -> int:
    """Inner-loop trips of Alg. 1 on the table the device actually fills: times reduced by each
    layer's minimum (budget B - M) and rows cut at the largest reachable reduced time.  Level s
    of layer l then visits t' = shift .. top_l.  With the D record, levels of a layer that take
    the same time are served by one update (the smallest of their errors), so only the distinct
    times of a layer count."""
    t = tau.astype(np.int64)
    mn = t.min(axis=1)
    bp = B - int(mn.sum())
    if bp < 0:
        return 0
    delta = t - mn[:, None]
    span = np.where(delta <= bp, delta, 0).max(axis=1)
    top = np.minimum(np.cumsum(span), bp)
    if not merge_equal_times:
        return int(np.clip(top[:, None] + 1 - delta, 0, None).sum())
    return int(sum(np.clip(top[l] + 1 - np.unique(delta[l]), 0, None).sum()
                   for l in range(t.shape[0])))


def executed_updates_level_record(tau: np.ndarray, err: np.ndarray, B: int) -> int:
    """The same count for the level record, summed over the candidates: every level is visited
    except those that cannot win (an earlier level of the layer takes the same time with an error
    no larger), which depends on the candidate's errors."""
    t = tau.astype(np.int64)
    mn = t.min(axis=1)
    bp = B - int(mn.sum())
    if bp < 0:
        return 0
    delta = t - mn[:, None]
    span = np.where(delta <= bp, delta, 0).max(axis=1)
    top = np.minimum(np.cumsum(span), bp)
    total = 0
    for l in range(t.shape[0]):
        for d in np.unique(delta[l]):
            if d > top[l]:
                continue
            idx = np.flatnonzero(delta[l] == d)               # ascending level index
            e = err[:, l, idx]
            visit = np.ones(e.shape, dtype=bool)
            if idx.size > 1:
                visit[:, 1:] = e[:, 1:] < np.minimum.accumulate(e, axis=1)[:, :-1]
            total += int(visit.sum()) * int(top[l] + 1 - d)
    return total


def host_cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the chip needs some tens of milliseconds of load to settle its clocks: with 3 warm-up and
    # 20 timed steps of 0.6 ms the step reads 8 % longer than in steady state
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="rn50_k1024")
    ap.add_argument("--record", choices=["d", "level"], default="d",
                    help="what the fill records per cell: fp32 D (fast) or the one-byte level")
    ap.add_argument("--candidates", type=int, default=None,
                    help="solve only the first N candidates of the workload (experiments)")
    ap.add_argument("--from-incumbent", type=int, default=0, metavar="D",
                    help="time spdy_dp_solve_from_incumbent instead: every candidate is candidate 0 "
                         "with D random layers resampled (one round of the search of Sec. 3.3), "
                         "sorted by its first resampled layer")
    ap.add_argument("--checkpoints", type=int, default=None, metavar="STRIDE",
                    help="time spdy_dp_solve_checkpointed instead (0: stride about sqrt(L)): a "
                         "record of about 2 sqrt(L) rows per candidate, two fills")
    ap.add_argument("--overlap", action="store_true",
                    help="pipeline consecutive steps over two streams and two workspaces: the "
                         "walk back of step i runs beside the fill of step i + 1")
    ap.add_argument("--one-call", action="store_true",
                    help="time spdy_dp_solve_batched as one call instead of its two stages "
                         "(no fill-stage events, so no roofline objects)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size reference for "
                         "FETCH_SIZE / WRITE_SIZE counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (candidates would shard across GPUs with no "
              "communication inside a solve); --gpus must be 1", file=sys.stderr)
        return 2

    import torch

    import paper_2201_13096_amd as dp
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dp.binding.lib()

    cfg = workloads.CONFIGS[args.workload]
    tau, err, B = workloads.generate(cfg, K=args.candidates)
    K, L, S = err.shape
    dev = torch.device("cuda:0")
    first_layer = None
    if args.from_incumbent > 0:
        if args.record != "d":
            print("bench.py: --from-incumbent needs the D record", file=sys.stderr)
            return 2
        rng = np.random.Generator(np.random.PCG64(1))
        d = min(args.from_incumbent, L)
        mutated = np.repeat(err[:1], K, axis=0)
        first_layer = np.empty(K, dtype=np.int32)
        for k in range(K):
            layers = rng.choice(L, size=d, replace=False)
            mutated[k, layers] = err[k, layers]
            first_layer[k] = layers.min()
        by_first = np.argsort(first_layer, kind="stable")
        incumbent = np.ascontiguousarray(err[:1])
        err = np.ascontiguousarray(mutated[by_first])
        first_layer = np.ascontiguousarray(first_layer[by_first])
    tau_d = torch.from_numpy(tau).to(dev)
    err_d = torch.from_numpy(err).to(dev)
    if args.checkpoints is not None:
        if args.record != "d" or args.from_incumbent > 0 or args.overlap:
            print("bench.py: --checkpoints goes with the D record only, and with neither "
                  "--from-incumbent nor --overlap", file=sys.stderr)
            return 2
        ws = torch.empty(dp.spdy_dp_workspace_bytes_checkpointed(K, L, S, B, args.checkpoints),
                         dtype=torch.uint8, device=dev)
    else:
        ws = dp.alloc_workspace(K, L, S, B, dev, compact=(args.record == "level"))
    profile = torch.empty((K, L), dtype=torch.int16, device=dev)
    cost = torch.empty((K,), dtype=torch.float32, device=dev)

    if first_layer is not None:
        first_d = torch.from_numpy(first_layer).to(dev)
        inc_ws = dp.alloc_workspace(1, L, S, B, dev)
        dp.spdy_dp_solve_batched(tau_d, torch.from_numpy(incumbent).to(dev), B, workspace=inc_ws)

    if args.overlap:
        if first_layer is not None:
            print("bench.py: --overlap and --from-incumbent exclude each other", file=sys.stderr)
            return 2
        fill_stream, walk_stream = torch.cuda.Stream(), torch.cuda.Stream()
        slots = [(ws, profile, cost),
                 (dp.alloc_workspace(K, L, S, B, dev, compact=(args.record == "level")),
                  torch.empty_like(profile), torch.empty_like(cost))]
        walked = [None, None]                 # event: the walk back that last used the slot
        turn = [0]

    def step(ev_a=None, ev_b=None):
        if args.checkpoints is not None:      # one call, several fills: no single fill stage
            if ev_a is not None:
                ev_a.record()
            dp.spdy_dp_solve_checkpointed(tau_d, err_d, B, args.checkpoints, profile, cost, ws)
            if ev_b is not None:
                ev_b.record()
            return
        if args.overlap:
            i = turn[0] % 2
            turn[0] += 1
            ws_i, profile_i, cost_i = slots[i]
            if walked[i] is not None:
                fill_stream.wait_event(walked[i])
            if ev_a is not None:
                ev_a.record(fill_stream)
            dp.spdy_dp_fill(tau_d, err_d, B, cost_i, ws_i, stream=fill_stream)
            filled = ev_b if ev_b is not None else torch.cuda.Event()
            filled.record(fill_stream)
            walk_stream.wait_event(filled)
            dp.spdy_dp_backtrace(tau_d, err_d, B, profile_i, cost_i, ws_i, stream=walk_stream)
            walked[i] = torch.cuda.Event()
            walked[i].record(walk_stream)
            return
        if first_layer is not None:           # one fused call: no event between its stages
            if ev_a is not None:
                ev_a.record()
            dp.spdy_dp_solve_from_incumbent(tau_d, err_d, first_d, B, inc_ws, profile, cost, ws)
            if ev_b is not None:
                ev_b.record()
            return
        if args.one_call:
            if ev_a is not None:
                ev_a.record()
            dp.spdy_dp_solve_batched(tau_d, err_d, B, profile, cost, ws)
            if ev_b is not None:
                ev_b.record()
            return
        # the two stages of spdy_dp_solve_batched, with events around the fill stage
        if ev_a is not None:
            ev_a.record()
        dp.spdy_dp_fill(tau_d, err_d, B, cost, ws)
        if ev_b is not None:
            ev_b.record()
        dp.spdy_dp_backtrace(tau_d, err_d, B, profile, cost, ws)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # HIP events around the fill stage of every fourth timed step (an event pair costs about as
    # much as a kernel launch, which shows on a 0.6 ms step)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           if i % 4 == 0 else (None, None) for i in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in evs:
        step(a, b)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    fill_samples = [a.elapsed_time(b) for a, b in evs if a is not None]
    fill_ms = float(np.mean(fill_samples))

    nominal = K * L * S * B
    if args.record == "d":
        executed = K * executed_updates_per_candidate(tau, B, True)
    elif S <= 64:
        executed = executed_updates_level_record(tau, err, B)
    else:                                         # more than 64 levels: every level is visited
        executed = K * executed_updates_per_candidate(tau, B, False)
    value = nominal / (ms_per_step * 1e-3)
    ops = LANE_OPS_PER_UPDATE[args.record]
    achieved = executed * ops / (fill_ms * 1e-3)
    lds_achieved = executed * LDS_BYTES_PER_UPDATE / (fill_ms * 1e-3)

    p_gpu = profile.cpu().numpy()
    c_gpu = cost.cpu().numpy()

    out = {
        "metric": "DP cell-updates/s (K*L*S*B/s)",
        "value": value,
        "unit": "cell-updates/s",
        "candidates_per_s": K / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name + ("+overlap" if args.overlap else ""),
                   "K": K, "L": L, "S": S, "B": B, "record": args.record,
                   "executed_updates": executed, "nominal_updates": nominal},
        "roofline": {
            "bound": "alu",
            "kernel": "dp_fill",
            "achieved": achieved / 1e12,
            "peak": ALU_PEAK_LANE_OPS / 1e12,
            "unit": "Tlane-op/s",
            "frac": achieved / ALU_PEAK_LANE_OPS,
            "lane_ops_per_update": ops,
            "kernel_ms": fill_ms,
            "kernel_ms_median": float(np.median(fill_samples)),
            "kernel_ms_min": float(np.min(fill_samples)),
            "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, args.record))
            if K == cfg.K else None,
        },
        "roofline_lds": {
            "achieved": lds_achieved / 1e12,
            "peak": LDS_PEAK_BYTES / 1e12,
            "unit": "TB/s",
            "frac": lds_achieved / LDS_PEAK_BYTES,
        },
    }

    if out["roofline"]["traffic"] is not None:    # the record stream, not the bound
        out["roofline"]["hbm_gbps"] = out["roofline"]["traffic"] / (fill_ms * 1e-3) / 1e9

    if not args.no_cpu_baseline:
        import oracle
        threads = min(16, os.cpu_count() or 1)
        # bounded sample: as many candidates of this workload as about 20 s of CPU work allows
        t_one0 = time.perf_counter()
        oracle.solve_ref(tau, err[:1], B)
        t_one = time.perf_counter() - t_one0
        n = int(max(threads, min(K, 20.0 / max(t_one, 1e-6))))
        n = min(K, n)
        t_c0 = time.perf_counter()
        p_ref, c_ref = oracle.solve_ref(tau, err[:n], B, threads=threads)
        t_c = time.perf_counter() - t_c0
        out["cpu_baseline"] = {
            "value": n * L * S * B / t_c,
            "unit": "cell-updates/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"first {n} of {K} candidates of {cfg.name}, {threads} threads; "
                      f"one candidate on one thread took {t_one * 1e3:.1f} ms",
            "single_thread_ms_per_candidate": t_one * 1e3,
            "cpu": host_cpu_model(),
        }
        out["parity"] = bool((p_gpu[:n] == p_ref).all() and
                             (c_gpu[:n].view(np.uint32) == c_ref.view(np.uint32)).all())
    if args.checkpoints is not None:
        del out["roofline"], out["roofline_lds"]
        out["config"]["workload"] = f"{cfg.name}+checkpoints(stride={args.checkpoints})"
        out["config"]["workspace_bytes"] = int(ws.numel())
        out["config"]["workspace_bytes_full_record"] = int(dp.spdy_dp_workspace_bytes(K, L, S, B))
    if args.one_call:
        out.pop("roofline", None)
        out.pop("roofline_lds", None)
        out["config"]["workload"] = cfg.name + "+one_call"
    if first_layer is not None:
        # the roofline objects describe the plain fill; here the event pair spans the whole call
        # and a varying part of the updates is skipped
        out.pop("roofline", None)
        out.pop("roofline_lds", None)
        out["config"]["workload"] = f"{cfg.name}+from_incumbent(d={args.from_incumbent})"
        out["config"]["mean_first_layer"] = float(first_layer.mean())
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
