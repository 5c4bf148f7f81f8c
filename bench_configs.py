#!/usr/bin/env python3
"""Times every workload configuration (not only the one bench.py reports) on
one MI355X: cache-cold and warm microseconds per layer application, effective
GB/s against the 8 TB/s HBM roofline, and the same layer dense on the GPU.
Prints one JSON line per case and a markdown table at the end.

Every time is the median (and the minimum) of five measurements, each a HIP-event pair around several
replays of a captured graph of plain launches.

    python bench_configs.py [--configs 1,2,3,4,5] [--seeds 0,1,2]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

import numpy as np
import torch

from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL
import bench_util as BU

HBM = 8000.0
COLD_FOOTPRINT = 2 * (256 + 32) * (1 << 20)
ROWS = []


def wd(p):
    return B.PIVOT_F32 if p.wdtype == WL.F32 else B.PIVOT_F16


def dev_plan(p):
    return B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd(p), p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol,
                           p.bias, act=p.act, device=0)


def workspace(n):
    ws = torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")
    B.pivot_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    return ws


def gt(enqueue, n_launch, replays=4):
    """GPU-side us per launch: replays of a captured graph of n_launch plain launches (bench_util.py)."""
    return BU.graph_time(enqueue, n_launch, replays=replays, repeats=3)


def gts(enqueue, n_launch, replays=4):
    """(median, min) of five such measurements."""
    return BU.graph_time(enqueue, n_launch, replays=replays, repeats=5, stats=True)


def emit(name, us_cold, us_warm, alg_bytes, dense_us=None, extra=None):
    cold_min = warm_min = None
    if isinstance(us_cold, tuple):
        us_cold, cold_min = us_cold
    if isinstance(us_warm, tuple):
        us_warm, warm_min = us_warm
    row = {"case": name, "cold_min_us": None if cold_min is None else round(cold_min, 2),
           "warm_min_us": None if warm_min is None else round(warm_min, 2), "cold_us": None if us_cold is None else round(us_cold, 2), "warm_us": round(us_warm, 2),
           "alg_MB": round(alg_bytes / 1e6, 3),
           "cold_GBs": None if us_cold is None else round(alg_bytes / us_cold / 1e3, 1),
           "cold_frac": None if us_cold is None else round(alg_bytes / us_cold / 1e3 / HBM, 4),
           "warm_GBs": round(alg_bytes / us_warm / 1e3, 1),
           "dense_us": None if dense_us is None else round(dense_us, 2)}
    if dense_us is not None and us_cold is not None:
        row["speedup_vs_dense"] = round(dense_us / us_cold, 2)
    if us_cold is not None:
        fc, fw = BU.stream_floor(alg_bytes)
        row["read_only_cold_us"] = round(fc, 2)
        row["read_only_warm_us"] = round(fw, 2)
        row["cold_vs_read_only"] = round(fc / us_cold, 3)
    if extra:
        row.update(extra)
    ROWS.append(row)
    print(json.dumps(row), flush=True)


def time_fc(p, iters, name, dense=True):
    st = torch.cuda.current_stream().cuda_stream
    batch = p.batch
    plan0 = dev_plan(p)
    v = B.pivot_fc_plan_host_view(plan0)
    alg = p.algorithmic_bytes(batch)
    ncopies = int(max(2, min(600, -(-COLD_FOOTPRINT // alg))))
    plans = [plan0] + [B.pivot_fc_plan_clone(plan0) for _ in range(ncopies - 1)]
    xs = [torch.from_numpy(p.x.copy()).cuda() for _ in range(ncopies)]
    yd = torch.empty((batch, p.M), dtype=torch.float32, device="cuda")
    ws = workspace(B.pivot_fc_workspace_bytes(plan0, batch))

    def go(rot):
        def f(i, s):
            j = i % ncopies if rot else 0
            B.pivot_fc_run(plans[j], xs[j].data_ptr(), p.K, yd.data_ptr(), p.M, batch, ws.data_ptr(), ws.numel(), s)
        return f

    cold = gts(go(True), ncopies * max(1, 64 // ncopies))
    warm = gts(go(False), 100)
    dense_us = None
    if dense:
        Wnat = np.empty_like(p.Wp)
        Wnat[np.ix_(p.prow, p.pcol)] = p.Wp
        nd = int(max(2, -(-COLD_FOOTPRINT // p.dense_bytes(batch))))
        Wds = [torch.from_numpy(Wnat).cuda() for _ in range(nd)]
        bd = torch.from_numpy(p.bias).cuda()

        def god(i, s):
            B.pivot_dense_run(Wds[i % nd].data_ptr(), wd(p), p.M, p.K, xs[i % ncopies].data_ptr(), p.K,
                              bd.data_ptr(), yd.data_ptr(), p.M, batch, p.act, s)

        own = gt(god, 4 * nd)
        # rocBLAS through torch, launched eagerly (its launch cost is below these kernels' run time)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(2 * nd):
            torch.matmul(xs[i % ncopies], Wds[i % nd].t())
        torch.cuda.synchronize()
        e0.record()
        for i in range(8 * nd):
            torch.matmul(xs[i % ncopies], Wds[i % nd].t())
        e1.record()
        torch.cuda.synchronize()
        lib = e0.elapsed_time(e1) * 1e3 / (8 * nd)
        dense_us = min(own, lib)
        del Wds
    emit(name, cold, warm, alg, dense_us,
         {"kept": round(p.T / (p.nbr * p.nbc), 4), "work_items": v["nchunks"] * v["row_slices"],
          "row_slices": v["row_slices"], "chunk_tiles": v["chunk_tiles"], "wg_waves": v["wg_waves"]})
    for h in plans:
        B.pivot_fc_plan_destroy(h)
    torch.cuda.empty_cache()


def time_chain(probs, iters, name, per_layer=False):
    st = torch.cuda.current_stream().cuda_stream
    alg = sum(p.algorithmic_bytes(1) for p in probs)
    ncopies = int(max(2, -(-COLD_FOOTPRINT // alg)))
    sets = []
    for _ in range(ncopies):
        plans = [dev_plan(p) for p in probs] if not sets else [B.pivot_fc_plan_clone(h) for h in sets[0][0]]
        sets.append((plans, B.pivot_mlp_plan(plans, B.PIVOT_MLP_LAUNCH_PER_LAYER if per_layer else 0)))
    xs = [torch.from_numpy(probs[0].x.copy()).cuda() for _ in range(ncopies)]
    M = probs[-1].M
    yd = torch.empty((1, M), dtype=torch.float32, device="cuda")
    ws = workspace(B.pivot_mlp_workspace_bytes(sets[0][1], 1))

    def go(rot):
        def f(i, s):
            j = i % ncopies if rot else 0
            B.pivot_mlp_run(sets[j][1], xs[j].data_ptr(), probs[0].K, yd.data_ptr(), M, 1, ws.data_ptr(), ws.numel(), s)
        return f

    cold = gts(go(True), ncopies * max(1, 24 // ncopies))
    warm = gts(go(False), 40)
    torch.cuda.synchronize()
    for plans, mlp in sets:
        assert B.pivot_mlp_status(mlp, st) == 0
    emit(name, cold, warm, alg, None, {"launches": len(probs) if per_layer else 1})
    for plans, mlp in sets:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)
    torch.cuda.empty_cache()


def time_lstm(lp, name, per_step=False):
    st = torch.cuda.current_stream().cuda_stream
    p = lp.fc
    plan = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd(p), p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol,
                           p.bias, act=p.act, device=0,
                           flags=B.PIVOT_PLAN_LSTM_LAUNCH_PER_STEP if per_step else B.PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS)
    # (ONE_LAUNCH_ALWAYS: the one-step sequences below are to time the one-launch form's first step; left to itself
    # pivot_lstm_run takes the launch-per-step form for sequences of fewer than 4 steps)
    steps, batch = lp.xs.shape[0], lp.xs.shape[1]
    xsd = torch.from_numpy(lp.xs).cuda()
    hd = torch.zeros((batch, lp.H), device="cuda")
    cd = torch.zeros((batch, lp.H), device="cuda")
    ws = workspace(B.pivot_lstm_workspace_bytes(plan, lp.H, lp.I, steps, batch))

    def go(i, s):
        B.pivot_lstm_run(plan, lp.H, lp.I, xsd.data_ptr(), hd.data_ptr(), cd.data_ptr(), None, steps, batch,
                         ws.data_ptr(), ws.numel(), s)

    total, total_min = gts(go, 1, replays=5)
    assert B.pivot_lstm_status(plan, steps, batch, ws.data_ptr(), st) == 0
    # the first step finds the weights in HBM, the other 255 on chip: a one-step sequence timed over rotating
    # copies of the plan (cold) and on one copy (warm); each includes the set-up kernels of a sequence
    alg = p.algorithmic_bytes(batch)
    ncopies = int(max(2, -(-COLD_FOOTPRINT // alg)))
    plans = [plan] + [B.pivot_fc_plan_clone(plan) for _ in range(ncopies - 1)]
    ws1 = workspace(B.pivot_lstm_workspace_bytes(plan, lp.H, lp.I, 1, batch))

    def one(rot):
        def f(i, s):
            B.pivot_lstm_run(plans[i % ncopies if rot else 0], lp.H, lp.I, xsd.data_ptr(), hd.data_ptr(), cd.data_ptr(), None,
                             1, batch, ws1.data_ptr(), ws1.numel(), s)
        return f
    first_cold = gts(one(True), ncopies)
    first_warm = gts(one(False), 50)
    emit(name, None, (total / steps, total_min / steps), alg, None,
         {"steps": steps, "total_us": round(total, 1), "total_min_us": round(total_min, 1),
          "first_step_cold_us": round(first_cold[0], 2), "first_step_cold_min_us": round(first_cold[1], 2),
          "first_step_warm_us": round(first_warm[0], 2),
          "note": "warm_us = per-step time of the whole sequence (matvec + cell, set-up kernels included; the weights stay "
                  "on chip after step 1); first_step_* = a sequence of ONE step, set-up kernels included, over rotating "
                  "copies of the plan (cold) or one copy (warm)"})
    for h in plans:
        B.pivot_fc_plan_destroy(h)
    torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--seeds", default="0,1,2")
    ap.add_argument("--iters", type=int, default=300)
    args = ap.parse_args()
    seeds = [int(v) for v in args.seeds.split(",")]
    which = set(args.configs.split(","))
    assert torch.cuda.is_available(), "needs a GPU"
    B.lib()
    st = torch.cuda.current_stream().cuda_stream

    def null_us():
        return gt(lambda i, s: B.pivot_null_run(s), 200, replays=10)

    print(json.dumps({"case": "null kernel back to back", "us": round(null_us(), 2)}), flush=True)
    for seed in seeds:
        tag = " seed %d" % seed
        if "1" in which:
            time_fc(WL.config1(seed=seed), args.iters, "cfg1 1024x1024 f32 16x16 25% b1" + tag)
        if "2" in which:
            time_fc(WL.config2(seed=seed), args.iters, "cfg2 4096x9216 f32 32x32 10% bal b1" + tag)
        if "3" in which:
            for frac in WL.CONFIG3_FRACS:
                for batch in (1, 4, 16):
                    time_fc(WL.config3(seed=seed, batch=batch, frac=frac), args.iters,
                            "cfg3 4096x4096 f16 64x16 %g%% b%d" % (frac * 100, batch) + tag, dense=(seed == seeds[0]))
        if "4" in which:
            for elim in (False, True):
                for per_layer in (False, True):
                    time_chain(WL.config4(seed=seed, eliminated=elim), args.iters,
                               "cfg4 MLP 25088-4096-4096-1000 f32 %s, %s" % ("eliminated" if elim else "composed",
                                                                           "launch per layer" if per_layer else "one launch") + tag,
                               per_layer=per_layer)
        if "5" in which:
            time_lstm(WL.config5(seed=seed), "cfg5 LSTM gates 8192x3072 f16 16x32 zipf b8, 256 steps, one launch" + tag)
            time_lstm(WL.config5(seed=seed), "cfg5 LSTM gates 8192x3072 f16 16x32 zipf b8, 256 steps, launch per step" + tag,
                      per_step=True)

    print("\n| case | kept | cold us (median) | cold us (min) | cold GB/s | % of 8 TB/s | read-only launch, cold us | warm us (median) | warm us (min) | warm GB/s | first step cold us | dense us (best of own, rocBLAS) | speedup vs dense |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for r in ROWS:
        f = lambda k, fmt="%s": ("-" if r.get(k) is None else fmt % r[k])
        print("| %s | %s | %s | %s | %s | %s | %s | %s | %s | %s | %s | %s | %s |" % (
            r["case"], f("kept"), f("cold_us"), f("cold_min_us"), f("cold_GBs"),
            "-" if r.get("cold_frac") is None else "%.1f" % (100 * r["cold_frac"]), f("read_only_cold_us"),
            f("warm_us"), f("warm_min_us"), f("warm_GBs"), f("first_step_cold_us"), f("dense_us"), f("speedup_vs_dense")))


if __name__ == "__main__":
    main()
