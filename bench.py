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

# Nominal peaks of the chip (256 compute units, 2.4 GHz).
# LDS: 128 bytes per clock per compute unit for reads of up to 64 bits per lane (a 64-lane 32-bit
# read takes two clocks); aligned 128-bit reads run at twice that on this generation.
# Vector ALU: 128 plain 32-bit lane-instructions per clock per compute unit (4 SIMDs, a 64-lane
# instruction every two clocks each).  The published 157.3 TFLOP/s fp32 vector figure is this
# x 2 for fused multiply-add; an add / min chain gets one operation per instruction.  (The rate
# probe issues 98 - 105 lane-instructions per clock per compute unit on add / min / min3 mixes,
# counted with SQ_INSTS_VALU, so the unit is not a 64-lane one.)
COMPUTE_UNITS = 256
CLOCK_HZ = 2.4e9
LDS_PEAK_B32 = COMPUTE_UNITS * 128 * CLOCK_HZ
LDS_PEAK_B128 = COMPUTE_UNITS * 256 * CLOCK_HZ
ALU_PEAK_LANE_OPS = COMPUTE_UNITS * 128 * CLOCK_HZ
# Algorithmic cost of one executed update of Alg. 1's inner loop.
#   LDS: one 4-byte read of the shifted previous row plus the 4 / S bytes the new row's write
#        costs per update.
#   ALU, D record: an fp32 add and an fp32 min; as built one v_min3_f32 folds two updates, so 1.5
#        issued instructions per update.  Level record: add, compare, select of the level, min.
LANE_OPS_PER_UPDATE = {"d": 2.0, "level": 4.0}
LANE_OPS_AS_BUILT = {"d": 1.5, "level": 4.0}
PROFILES = os.path.join(ROOT, "profiles")
KERNEL_SOURCE = os.path.join(ROOT, "paper_2201_13096_amd", "csrc", "spdy_dp.hip")
PROBE = os.path.join(ROOT, "paper_2201_13096_amd", "peaks_probe")


def kernel_source_id() -> str:
    """Short hash of the HIP source: counter figures taken from a tracked profile only count while
    the kernel they were taken on is the one in the tree."""
    import hashlib
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:12]


def tracked_traffic(workload: str, record: str):
    """HBM bytes per launch of the fill kernel from profiles/dp_fill_hbm_traffic.txt (FETCH_SIZE +
    WRITE_SIZE counter runs scaled by a plain copy of known size), or None when the file has no
    line for this workload and record taken on the present kernel source."""
    path = os.path.join(PROFILES, "dp_fill_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                tok = line.split("#", 1)[0].split()
                if len(tok) >= 5 and tok[0] == workload and tok[1] == record \
                        and tok[2] == kernel_source_id():
                    return float(tok[3]) + float(tok[4])
    except OSError:
        pass
    return None


def measured_peaks():
    """Run the rate probe (a separate executable) as a child process; None if it is not built or
    fails.  Called before this process touches the GPU."""
    import subprocess
    if not os.path.exists(PROBE):
        return None
    try:
        res = subprocess.run([PROBE], capture_output=True, text=True, timeout=120)
        if res.returncode != 0:
            return None
        return json.loads(res.stdout.strip().splitlines()[-1])
    except (OSError, ValueError, subprocess.TimeoutExpired):
        return None


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


def host_threads() -> int:
    """Threads the oracle leg may use: the cores this process is allowed on, at most 16 (the CPU
    share that goes with one GPU on a shared host)."""
    try:
        n = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        n = os.cpu_count() or 1
    return max(1, min(16, n))


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
    ap.add_argument("--no-probe", action="store_true",
                    help="do not run the VALU / LDS rate probe before the benchmark")
    ap.add_argument("--settle-steps", type=int, default=200,
                    help="steps run after the timed ones and timed separately (reported as "
                         "steady_state: the core clock only settles after some tens of "
                         "milliseconds of load)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size reference for "
                         "FETCH_SIZE / WRITE_SIZE counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (candidates would shard across GPUs with no "
              "communication inside a solve); --gpus must be 1", file=sys.stderr)
        return 2

    # the rate probe runs as a child process of its own, before this process touches the GPU
    peaks = None if args.no_probe else measured_peaks()

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
    p_gpu = profile.cpu().numpy()
    c_gpu = cost.cpu().numpy()

    # the same again, after the timed region, once the clocks have settled (reported beside it)
    steady = None
    if args.settle_steps > 0:
        evs2 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                if i % 4 == 0 else (None, None) for i in range(args.settle_steps)]
        for _ in range(args.settle_steps // 2):
            step()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for a, b in evs2:
            step(a, b)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        steady = {"steps": args.settle_steps,
                  "ms_per_step": (t3 - t2) * 1e3 / args.settle_steps,
                  "kernel_ms": float(np.mean([a.elapsed_time(b) for a, b in evs2
                                              if a is not None]))}

    nominal = K * L * S * B
    if args.record == "d":
        executed = K * executed_updates_per_candidate(tau, B, True)
    elif S <= 64:
        executed = executed_updates_level_record(tau, err, B)
    else:                                         # more than 64 levels: every level is visited
        executed = K * executed_updates_per_candidate(tau, B, False)
    value = nominal / (ms_per_step * 1e-3)
    seconds = fill_ms * 1e-3
    lds_bytes = executed * 4.0 * (1.0 + 1.0 / S)
    lane_ops = executed * LANE_OPS_PER_UPDATE[args.record]
    lane_ops_built = executed * LANE_OPS_AS_BUILT[args.record]

    def rate(obj, key):
        return None if peaks is None or obj not in peaks else peaks[obj].get(key)

    # The D-record fill is bound by LDS reads (4 bytes of the shifted row per update, an add and
    # half a v_min3 beside it); the level-record fill by the vector ALU (four instructions per
    # update).  Both objects are always reported; `roofline` is the binding one.  With at most 64
    # levels the D-record sweep reads 128 bits per lane, so its peak is the 128-bit one; the
    # fraction of the 32-bit-read peak (what a lane = bucket layout can reach at best) is beside it.
    wide_reads = args.record == "d" and S <= 64
    lds_peak = LDS_PEAK_B128 if wide_reads else LDS_PEAK_B32
    lds_probe = "lds_read_b128" if wide_reads else "lds_read_b32"
    lds_obj = {
        "bound": "lds",
        "kernel": "dp_fill",
        "achieved": lds_bytes / seconds / 1e12,
        "peak": lds_peak / 1e12,
        "unit": "TB/s",
        "frac": lds_bytes / seconds / lds_peak,
        "bytes_per_update": 4.0 * (1.0 + 1.0 / S),
        "peak_is": ("nominal: 256 CU x 256 B/clk x 2.4 GHz, aligned 128-bit reads" if wide_reads else
                    "nominal: 256 CU x 128 B/clk x 2.4 GHz, reads of up to 64 bits per lane"),
        "peak_measured": rate(lds_probe, "tb_per_s"),
        "frac_of_measured": None if rate(lds_probe, "tb_per_s") is None
        else lds_bytes / seconds / 1e12 / rate(lds_probe, "tb_per_s"),
        "peak_b32_nominal": LDS_PEAK_B32 / 1e12,
        "frac_of_b32_nominal": lds_bytes / seconds / LDS_PEAK_B32,
        "peak_b32_measured": rate("lds_read_b32", "tb_per_s"),
    }
    probe_mix = "valu_add_add_min3" if args.record == "d" else "valu_add_cmp_sel_min"
    valu_obj = {
        "bound": "alu",
        "kernel": "dp_fill",
        "achieved": lane_ops / seconds / 1e12,
        "peak": ALU_PEAK_LANE_OPS / 1e12,
        "unit": "Tlane-op/s",
        "frac": lane_ops / seconds / ALU_PEAK_LANE_OPS,
        "lane_ops_per_update": LANE_OPS_PER_UPDATE[args.record],
        "as_built": {"lane_ops_per_update": LANE_OPS_AS_BUILT[args.record],
                     "achieved": lane_ops_built / seconds / 1e12,
                     "frac": lane_ops_built / seconds / ALU_PEAK_LANE_OPS},
        "peak_is": "nominal: 256 CU x 128 lane-instructions/clk x 2.4 GHz (157.3 TFLOP/s / 2)",
        "peak_measured": rate(probe_mix, "tlane_ops_per_s"),
        "peak_measured_mix": probe_mix,
    }
    roofline = dict(lds_obj if args.record == "d" else valu_obj)
    roofline.update({
        "kernel_ms": fill_ms,
        "kernel_ms_median": float(np.median(fill_samples)),
        "kernel_ms_min": float(np.min(fill_samples)),
        "executed_updates_per_s": executed / seconds,
        # per clock and compute unit, beside what the sweep loop alone reaches in the rate probe
        # (no barriers, stores or table hand-over): the practical ceiling of this instruction mix
        "updates_per_clk_cu": executed / seconds / CLOCK_HZ / COMPUTE_UNITS,
        "bare_sweep_updates_per_clk_cu": rate("sweep_b128" if wide_reads else "sweep_b32",
                                              "updates_per_clk_cu"),
        "traffic": tracked_traffic(cfg.name, args.record) if K == cfg.K else None,
    })
    if roofline["traffic"] is not None:           # the record stream: not the bound
        roofline["hbm_gbps"] = roofline["traffic"] / seconds / 1e9

    out = {
        "metric": "DP cell-updates/s (nominal K*L*S*B per second of whole solve)",
        "value": value,
        "unit": "cell-updates/s",
        "executed_updates_per_s": executed / (ms_per_step * 1e-3),
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
        "roofline": roofline,
        "roofline_lds": lds_obj,
        "roofline_valu": valu_obj,
        "steady_state": steady,
        "measured_peaks": peaks,
    }
    if not args.no_cpu_baseline:
        import oracle
        threads = host_threads()
        # (i) one thread on min(K, 8) candidates; (ii) all threads on a bounded sample: as many
        # candidates of this workload as about 20 s of CPU work allows
        n1 = min(K, 8)
        t_one0 = time.perf_counter()
        oracle.solve_ref(tau, err[:n1], B)
        t_one = (time.perf_counter() - t_one0) / n1
        n = int(min(K, max(threads, 20.0 * threads / max(t_one, 1e-6))))
        t_c0 = time.perf_counter()
        p_ref, c_ref = oracle.solve_ref(tau, err[:n], B, threads=threads)
        t_c = time.perf_counter() - t_c0
        out["cpu_baseline"] = {
            "value": n * L * S * B / t_c,
            "unit": "cell-updates/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"first {n} of {K} candidates of {cfg.name} on {threads} threads "
                      f"({t_c:.2f} s); single thread: first {n1} candidates, "
                      f"{t_one * 1e3:.1f} ms per candidate",
            "candidates_per_s": n / t_c,
            "single_thread": {"candidates": n1, "ms_per_candidate": t_one * 1e3,
                              "value": L * S * B / t_one},
            "cpu": host_cpu_model(),
            "host_logical_cores": os.cpu_count(),
        }
        out["parity"] = bool((p_gpu[:n] == p_ref).all() and
                             (c_gpu[:n].view(np.uint32) == c_ref.view(np.uint32)).all())
    if args.checkpoints is not None:
        for key in ("roofline", "roofline_lds", "roofline_valu"):
            out.pop(key, None)
        out["config"]["workload"] = f"{cfg.name}+checkpoints(stride={args.checkpoints})"
        out["config"]["workspace_bytes"] = int(ws.numel())
        out["config"]["workspace_bytes_full_record"] = int(dp.spdy_dp_workspace_bytes(K, L, S, B))
    if args.one_call:
        for key in ("roofline", "roofline_lds", "roofline_valu"):
            out.pop(key, None)
        out["config"]["workload"] = cfg.name + "+one_call"
    if first_layer is not None:
        # the roofline objects describe the plain fill; here the event pair spans the whole call
        # and a varying part of the updates is skipped
        for key in ("roofline", "roofline_lds", "roofline_valu"):
            out.pop(key, None)
        out["config"]["workload"] = f"{cfg.name}+from_incumbent(d={args.from_incumbent})"
        out["config"]["mean_first_layer"] = float(first_layer.mean())
    if steady is not None and "roofline" in out:
        steady["roofline_frac"] = out["roofline"]["frac"] * fill_ms / steady["kernel_ms"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
