#!/usr/bin/env python3
"""Benchmark of the pruned fully-connected hot path on one MI355X.

One "step" is one application of the layer through pivot_fc_run (gather
through P_col into LDS, tile stream, reduction, bias, activation, scatter
through P_row) on one batch of synthetic input that is already resident in
HBM.  The workload is the AlexNet-fc6-shaped layer of the workload list
(4096 x 9216, fp32, batch 1, 32x32 tiles, 10 % kept, balanced rows).

The headline value is the cache-cold time per layer: consecutive steps rotate
through enough separate device copies of the plan and of x that no byte a step
reads is still in the L2 or the 256 MB Infinity Cache.  The warm time (same
copy back to back) is reported beside it.  The steps are replayed from HIP
graphs (see bench_util.py) so that the GPU, not the Python launch loop, is
what is timed.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
# kernel arguments in device memory (a ROCm runtime setting; must precede HIP start-up)
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E peak
COLD_FOOTPRINT = 2 * (256 + 32) * (1 << 20)   # rotate through >= 2 x (Infinity Cache + all L2)


TRAFFIC_FILE = os.path.join("profiles", "fc_gemv_cfg2_hbm_traffic.txt")


def parse_traffic():
    """HBM bytes per launch as measured with rocprofv3 --pmc in an EARLIER run of this command (the committed
    summary under profiles/; counters cannot be read from inside this process) and the date it was taken, or
    (None, None)."""
    val, date = None, None
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    val = float(line.split("=")[1].split()[0])
                elif line.startswith("measured_on"):
                    date = line.split("=")[1].strip()
    except OSError:
        pass
    return val, date


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2500)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a few plain 64 MiB device copies, so that a rocprofv3 --pmc run of this "
                         "command has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the layer is a single-device kernel); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1712_01084_amd import binding as B
    from paper_1712_01084_amd import workloads as WL
    import bench_util as BU

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()                                      # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    st = torch.cuda.current_stream().cuda_stream
    K, Wm = args.steps, args.warmup

    p = WL.config2(seed=args.seed)
    wd = B.PIVOT_F32
    plan0 = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol,
                            p.bias, act=p.act, device=0)
    view = B.pivot_fc_plan_host_view(plan0)
    alg_bytes = p.algorithmic_bytes(1)
    ncopies = max(2, -(-COLD_FOOTPRINT // alg_bytes))
    plans = [plan0] + [B.pivot_fc_plan_clone(plan0) for _ in range(ncopies - 1)]
    xs = [torch.from_numpy(p.x.copy()).cuda() for _ in range(ncopies)]
    ys = [torch.empty((1, p.M), dtype=torch.float32, device="cuda") for _ in range(ncopies)]
    ws_bytes = max(256, B.pivot_fc_workspace_bytes(plan0, 1))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    B.pivot_workspace_init(ws.data_ptr(), ws_bytes, st)

    def step(i, stream, rotate=True):
        j = i % ncopies if rotate else 0
        B.pivot_fc_run(plans[j], xs[j].data_ptr(), p.K, ys[j].data_ptr(), p.M, 1, ws.data_ptr(), ws_bytes, stream)

    if args.pmc_calibration:
        ca = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        cb = torch.ones(64 << 20, dtype=torch.uint8, device="cuda")
        for _ in range(5):
            ca.copy_(cb)
        torch.cuda.synchronize()

    # The K timed steps are replays of captured graphs of plain kernel launches, so that the host's
    # launch cost (about 5 us per call through Python, more than the GPU needs) is not what is timed.
    # Cold protocol: launch i uses copy i % ncopies.  The warm-up is whole rotations through ALL copies (at
    # least W launches, at least one rotation) and ends on the last copy; the timed region starts on copy 0.
    # Every timed launch therefore finds ncopies - 1 other copies (>= 2 x Infinity Cache + L2) touched since
    # its own copy was last read, whatever K is; K = whole-rotation graphs + one remainder graph, exactly K
    # launches between the first and the last event.  An event after every replay gives the spread.
    def timed(K_, W_, rotate):
        per = ncopies * max(1, 80 // ncopies) if rotate else 100
        full, rem = divmod(K_, per)
        g_rot = BU.capture(lambda i, s: step(i, s, rotate), per)
        g_rem = BU.capture(lambda i, s: step(i, s, rotate), rem) if rem else None
        warm_replays = max(1, -(-W_ // per))
        for _ in range(warm_replays):
            g_rot.replay()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(full + (1 if rem else 0) + 1)]
        t0 = time.perf_counter()
        # one more untimed rotation enqueued right in front of the first event: the timed launches then follow a
        # busy queue back to back, as every later launch of a long run does (otherwise the start-up of the first
        # replay from an idle device, several microseconds, is spread over the K launches and a short run
        # reads 0.3 us per launch slower than a long one)
        g_rot.replay()
        ev[0].record()
        for r in range(full):
            g_rot.replay()
            ev[r + 1].record()
        if g_rem is not None:
            g_rem.replay()
            ev[-1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        counts = [per] * full + ([rem] if rem else [])
        per_replay_us = [ev[r].elapsed_time(ev[r + 1]) * 1e3 / counts[r] for r in range(len(counts))]
        return dict(ms=ev[0].elapsed_time(ev[-1]) / K_, wall_ms=wall / (K_ + per) * 1e3, replay_us=per_replay_us,
                    warmup_launches=(warm_replays + 1) * per, copies_touched=ncopies if rotate else 1)

    cold = timed(K, Wm, True)
    warm = timed(K, Wm, False)
    cold_ms, cold_wall_ms, warm_ms = cold["ms"], cold["wall_ms"], warm["ms"]

    # The same K steps launched eagerly from Python, same cold protocol: whole rotations as warm-up (at least W
    # launches), the last of them left in the queue so that the timed launches follow a busy queue, then exactly
    # K launches from copy 0 on.  A call through Python costs the host about 5 us, about what the GPU needs for
    # one launch, so this figure can only be too high (host-bound), never too low.
    n_lead = ncopies * max(1, -(-Wm // ncopies))
    for i in range(n_lead - ncopies):
        step(i, st)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(ncopies):
        step(i, st)
    e0.record()
    for i in range(K):
        step(i, st)
    e1.record()
    torch.cuda.synchronize()
    eager_cold_us = e0.elapsed_time(e1) / K * 1e3

    # launch floor: an empty kernel back to back on the same stream
    null_us = BU.graph_time(lambda i, s: B.pivot_null_run(s), 200, replays=10)
    # one launch that only READS the layer's algorithmic bytes, cold and warm: what no single launch can beat
    floor_cold_us, floor_warm_us = BU.stream_floor(p.algorithmic_bytes(1), COLD_FOOTPRINT)

    # the same layer dense on the GPU: this library's streaming kernel, cold, and torch.mv as a guard
    dense_bytes = p.dense_bytes(1)
    nd = max(2, -(-COLD_FOOTPRINT // dense_bytes))
    Wnat = np.empty_like(p.Wp)
    Wnat[np.ix_(p.prow, p.pcol)] = p.Wp          # un-pivot: the dense comparator works in natural coordinates
    Wds = [torch.from_numpy(Wnat).cuda() for _ in range(nd)]
    bd = torch.from_numpy(p.bias).cuda()
    yd = torch.empty((1, p.M), dtype=torch.float32, device="cuda")

    dense_us = BU.graph_time(lambda i, s: B.pivot_dense_run(Wds[i % nd].data_ptr(), wd, p.M, p.K, xs[i % ncopies].data_ptr(),
                                                            p.K, bd.data_ptr(), yd.data_ptr(), p.M, 1, p.act, s),
                             8 * nd, replays=5)
    xv = xs[0][0]
    nde = 200
    for j in range(2 * nd):
        torch.mv(Wds[j % nd], xv)
    torch.cuda.synchronize()
    e0.record()
    for j in range(nde):
        torch.mv(Wds[j % nd], xv)
    e1.record(); torch.cuda.synchronize()
    torch_mv_us = e0.elapsed_time(e1) / nde * 1e3
    dense_best_us = min(dense_us, torch_mv_us)

    cold_us, warm_us = cold_ms * 1e3, warm_ms * 1e3
    # Every replay of a graph starts with a few microseconds in which no kernel runs.  Over the 80 launches of a
    # whole-rotation graph that is 0.1 us per launch; a short run (K below one rotation graph) is a single short
    # graph and would carry 0.3 us per launch of it.  Both legs time exactly K cold launches; the headline takes
    # the graph figure for long runs and the smaller of the two for short ones, and names which.
    graph_cold_us = cold_us
    value_source = "graph replays"
    if K < 400 and eager_cold_us < cold_us:
        cold_us, cold_ms, value_source = eager_cold_us, eager_cold_us * 1e-3, "eager launches (K below 400: one short graph carries its start-up)"
    kernel_name = B.pivot_fc_kernel_name(plan0, 1)       # the instantiation the library launches for this plan
    traffic, traffic_date = parse_traffic()
    kept = p.T / float(p.nbr * p.nbc)
    achieved = alg_bytes / (cold_us * 1e-6) / 1e9
    out = {
        "metric": "us per pruned FC layer @batch 1 (cache-cold) and % HBM roofline; speedup vs dense GEMV",
        "value": round(cold_us, 3),
        "unit": "us/layer",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": cold_ms,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: FC 4096x9216 (AlexNet fc6 shape) fp32 batch 1, 32x32 tiles, "
                               "29 of 288 tiles kept per block row (balanced), uniform random P_r/P_c, ReLU",
                   "seed": args.seed, "kept_fraction": round(kept, 5), "tiles": p.T,
                   "chunk_tiles": view["chunk_tiles"], "work_items": view["nchunks"] * view["row_slices"], "row_slices": view["row_slices"],
                   "wg_waves": view["wg_waves"],
                   "cold_copies": ncopies, "cold_copies_touched": cold["copies_touched"],
                   "warmup_launches": cold["warmup_launches"]},
        "cold_us_per_replay": {"median": round(float(np.median(cold["replay_us"])), 3), "min": round(min(cold["replay_us"]), 3),
                               "replays": len(cold["replay_us"])},
        "warm_us_per_replay": {"median": round(float(np.median(warm["replay_us"])), 3), "min": round(min(warm["replay_us"]), 3)},
        "value_source": value_source,
        "cold_graph_replay_us": round(graph_cold_us, 3),
        "warm_us": round(warm_us, 3),
        "cold_host_clock_us": round(cold_wall_ms * 1e3, 3),
        "cold_eager_python_launch_us": round(eager_cold_us, 3),
        "timing": "HIP events around replays of captured graphs of plain launches (exactly K launches between the first "
                  "and the last event; an untimed rotation through all copies is enqueued directly in front of the "
                  "first event so that the timed launches follow a busy queue)",
        "null_kernel_us": round(null_us, 3),
        "read_only_launch_us": {"cold": round(floor_cold_us, 3), "warm": round(floor_warm_us, 3),
                                "note": "one launch that only reads the same number of bytes (pivot_stream_read_run)"},
        "cold_vs_read_only_launch": round(floor_cold_us / cold_us, 3),
        "dense_gpu_us": {"own_kernel_cold": round(dense_us, 3), "torch_mv_cold": round(torch_mv_us, 3)},
        "speedup_vs_dense": round(dense_best_us / cold_us, 3),
        "linear_speedup": round(1.0 / kept, 3),
        "algorithmic_bytes": alg_bytes,
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic,
                     "traffic_source": "%s: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command on %s, "
                                       "not measured by this run" % (TRAFFIC_FILE, traffic_date),
                     "warm_effective": round(alg_bytes / (warm_us * 1e-6) / 1e9, 1)},
    }

    if not args.no_cpu_baseline:
        from oracle import pivot_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        Wd = O.dense_masked_natural(p.Wp, p.tile_mask, p.prow, p.pcol, p.bh, p.bw)
        y_ref = O.fc_dense(Wd, p.x, p.bias, p.act)       # warm-up + parity of the timed configuration
        D = O.error_scale(Wd, p.x, p.bias)
        err = O.max_scaled_error(ys[0].cpu().numpy(), y_ref, D)
        def time_oracle(seconds):
            O.fc_dense(Wd, p.x, p.bias, p.act)
            t0 = time.perf_counter()
            n = 0
            while time.perf_counter() - t0 < seconds:
                O.fc_dense(Wd, p.x, p.bias, p.act)
                n += 1
            return (time.perf_counter() - t0) / n * 1e6, n

        cpu_us, n = time_oracle(10.0)
        out["cpu_baseline"] = {"value": round(cpu_us, 1), "unit": "us/layer", "cores": int(cores), "kind": "oracle",
                               "sample": "%d applications of the same layer (float64 dense masked matvec, matrix "
                                         "prebuilt), about 10 s; host cores visible: %d"
                                         % (n, len(os.sched_getaffinity(0)))}
        try:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                cpu1_us, n1 = time_oracle(6.0)
            out["cpu_baseline_1thread"] = {"value": round(cpu1_us, 1), "unit": "us/layer", "cores": 1, "kind": "oracle",
                                           "sample": "%d applications, about 6 s, BLAS limited to one thread" % n1}
        except Exception as exc:                            # threadpoolctl missing: say so instead of a number
            out["cpu_baseline_1thread"] = {"value": None, "note": "not measured: %s" % exc}
        out["parity_max_scaled_error"] = err
        if not (err <= 1e-5):
            print("bench.py: parity check failed (%.3g)" % err, file=sys.stderr)
            sys.exit(1)

    for h in plans:
        B.pivot_fc_plan_destroy(h)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
