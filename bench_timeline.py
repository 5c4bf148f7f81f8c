#!/usr/bin/env python3
"""In-kernel timeline of the batch-1 layer kernel (fc_gemv_kernel) on one MI355X.

A second build of the library with -DPIVOT_TRACE (same sources; the stamps
compile to nothing in the product build) records the device's constant 100 MHz
clock at eight points per wavefront.  This script launches a layer back to
back (cache-cold: rotating through separate device copies of the plan and of
x; warm: one copy), keeps the stamps of the LAST launch of every burst, and
prints, per phase, the median over wavefronts, the 90th percentile and the
latest wavefront, all relative to the first wavefront's start.

    python bench_timeline.py --build            # on the CPU: builds paper_1712_01084_amd/libpivotfc_trace.so
    python bench_timeline.py [--cases cfg2,cfg4l1,cfg4,cfg1,cfg3d]    # on the GPU (cfg4: the one-launch chain kernel)

Ablations: builds of the same sources with -DPIVOT_ABLATE=bits leave one part
of the vector kernel's work out (no x, no staging, no copy of x, no store, no
epilogue; their results are wrong on purpose) and are timed like the product
(cold and warm us per launch, replayed graphs), which prices each part:

    python bench_timeline.py --build-ablations  # on the CPU (after the product build)
    python bench_timeline.py --ablations        # on the GPU

The stamps cost a few tens of nanoseconds per phase, so a traced launch is
slightly slower than the product kernel; the table shows where the time goes,
the product's time per launch comes from bench.py / bench_configs.py.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")
TRACE_LIB = os.path.join(ROOT, "paper_1712_01084_amd", "libpivotfc_trace.so")

PHASES = ["wave started", "every load issued", "copy of x stored to LDS", "past the barrier behind the copy",
          "x-segments staged", "last weight consumed", "sums of all waves in LDS", "outputs stored"]


def build():
    from paper_1712_01084_amd import build as Bd
    print(Bd.build(out=TRACE_LIB, objdir=os.path.join(Bd.HERE, "_build_trace"), device_flags=Bd.DEVICE + ["-DPIVOT_TRACE"]))


ABLATIONS = [(0, "product"), (1, "no x at all (no copy, no gather index, no staging)"),
             (2, "x copied into LDS but never staged (no barrier behind the copy, no gather)"),
             (4, "no copy of x (barrier and LDS-to-LDS gather kept)"), (8, "outputs computed but not stored"),
             (16, "no reduction, no outputs"), (17, "no x and no reduction: the weight stream alone")]


def ablation_lib(bits):
    from paper_1712_01084_amd import build as Bd
    return Bd.LIB if bits == 0 else os.path.join(Bd.HERE, "libpivotfc_abl%d.so" % bits)


def build_ablations():
    from paper_1712_01084_amd import build as Bd
    for bits, _ in ABLATIONS:
        if bits:
            print(Bd.build(out=ablation_lib(bits), objdir=os.path.join(Bd.HERE, "_build_trace", "abl%d" % bits),
                           device_flags=Bd.DEVICE + ["-DPIVOT_ABLATE=%d" % bits], only=["pivot_gemv_f32.hip"]))


def time_ablations():
    """Each library in a process of its own (one process cannot load two builds of the same symbols)."""
    import json
    import subprocess
    print("# What each part of the batch-1 layer kernel costs: configs[1] (4096x9216 fp32, 32x32 tiles, 10 % balanced)\n")
    print("| build | cold us / launch | warm us / launch |")
    print("|---|---|---|")
    for rep in range(2):
        for bits, what in ABLATIONS:
            lib = ablation_lib(bits)
            if not os.path.exists(lib):
                sys.exit("bench_timeline.py: %s is not built (run with --build-ablations first)" % lib)
            out = subprocess.run([sys.executable, os.path.abspath(__file__), "--time-one", lib], stdout=subprocess.PIPE, text=True, check=True).stdout
            r = json.loads(out.strip().splitlines()[-1])
            print("| %s%s | %.2f | %.2f |" % (what, " (second pass)" if rep else "", r["cold"], r["warm"]), flush=True)


def time_one(lib):
    import json
    import numpy as np
    import torch
    from paper_1712_01084_amd import binding as B
    from paper_1712_01084_amd import workloads as WL
    import bench_util as BU
    B.LIB_PATH = lib
    p = WL.config2(seed=0)
    plan0 = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, B.PIVOT_F32, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol, p.bias,
                            act=p.act, device=0)
    nc = 40
    plans = [plan0] + [B.pivot_fc_plan_clone(plan0) for _ in range(nc - 1)]
    xs = [torch.from_numpy(p.x.copy()).cuda() for _ in range(nc)]
    ys = [torch.empty((1, p.M), dtype=torch.float32, device="cuda") for _ in range(nc)]
    ws = torch.zeros(4096, dtype=torch.uint8, device="cuda")

    def step(rot):
        return lambda i, s: B.pivot_fc_run(plans[i % nc if rot else 0], xs[i % nc if rot else 0].data_ptr(), p.K,
                                           ys[i % nc if rot else 0].data_ptr(), p.M, 1, ws.data_ptr(), ws.numel(), s)
    cold = BU.graph_time(step(True), 80, replays=12, repeats=3)
    warm = BU.graph_time(step(False), 100, replays=10, repeats=3)
    print(json.dumps({"cold": cold, "warm": warm}))


def run_case(label, p, ncopies, bursts=14, **plan_kw):
    import numpy as np
    import torch
    from paper_1712_01084_amd import binding as B
    from paper_1712_01084_amd import workloads as WL
    wd = B.PIVOT_F32 if p.wdtype == WL.F32 else B.PIVOT_F16
    plan0 = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol, p.bias,
                            act=p.act, device=0, **plan_kw)
    plans = [plan0] + [B.pivot_fc_plan_clone(plan0) for _ in range(ncopies - 1)]
    v = B.pivot_fc_plan_host_view(plan0)
    name = B.pivot_fc_kernel_name(plan0, 1)
    nwg, nw = v["nchunks"] * v["row_slices"], v["wg_waves"]
    if "fc_gemv_kernel" in name:
        nw = int(name.split(",")[-2])                       # the wavefront count of the instantiation launched
    xs = [torch.from_numpy(p.x.copy()).cuda() for _ in range(ncopies)]
    ys = [torch.empty((1, p.M), dtype=torch.float32, device="cuda") for _ in range(ncopies)]
    wsb = max(256, B.pivot_fc_workspace_bytes(plan0, 1))
    ws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
    tr = torch.zeros((nwg * nw, 8), dtype=torch.int64, device="cuda")
    os.environ["PIVOT_TRACE_PTR"] = str(tr.data_ptr())      # read by the trace build at every launch
    st = torch.cuda.current_stream().cuda_stream
    res, k = [], 0
    for burst in range(bursts):
        n = (ncopies if ncopies > 1 else 24) + burst         # back to back; the stamps of the last launch survive
        for _ in range(n):
            j = k % ncopies
            k += 1
            B.pivot_fc_run(plans[j], xs[j].data_ptr(), p.K, ys[j].data_ptr(), p.M, 1, ws.data_ptr(), wsb, st)
        torch.cuda.synchronize()
        t = tr.cpu().numpy().astype(np.float64)
        if burst >= 2:
            res.append((t - t[:, 0].min()) / 100.0)          # 100 MHz ticks -> us since the first wavefront started
    r = np.stack(res)                                         # [burst][workgroup * wave][stamp]
    print("\n### %s\n" % label)
    print("kernel `%s`, %d workgroups x %d wavefronts, %d tiles per work item, %s; %d bursts\n"
          % (name, nwg, nw, v["chunk_tiles"], "cache-cold (rotating through %d copies)" % ncopies if ncopies > 1 else "warm (one copy)",
             len(res)))
    print("| stamp | median us | 90th percentile | latest wavefront (mean over bursts) |")
    print("|---|---|---|---|")
    for i, ph in enumerate(PHASES):
        a = r[:, :, i]
        print("| %d %s | %.2f | %.2f | %.2f |" % (i, ph, np.median(a), np.percentile(a, 90), a.max(axis=1).mean()))
    wg_end = r[:, :, 7].reshape(len(res), nwg, nw).max(axis=2)      # when each workgroup's last wavefront is done
    print("\nworkgroup end: median %.2f us, 90th percentile %.2f, slowest %.2f (mean over bursts)"
          % (np.median(wg_end), np.percentile(wg_end, 90), wg_end.max(axis=1).mean()), flush=True)
    for h in plans:
        B.pivot_fc_plan_destroy(h)
    del xs, ys
    torch.cuda.empty_cache()


CHAIN_PHASES = ["item started", "every load issued", "own x-segments staged (tagged input: producers' pairs arrived)",
                "last weight consumed", "sums of all waves in LDS", "stores of the outputs issued (the finishing wavefront)"]


def run_chain(label, probs, ncopies, bursts=12):
    """The one-launch chain kernel: per layer, the stamps of every wavefront of the last launch of each burst."""
    import numpy as np
    import torch
    from paper_1712_01084_amd import binding as B
    from paper_1712_01084_amd import workloads as WL
    wd = B.PIVOT_F32 if probs[0].wdtype == WL.F32 else B.PIVOT_F16
    sets = []
    for c in range(ncopies):
        plans = ([B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol, p.bias,
                                  act=p.act, device=0) for p in probs] if not sets
                 else [B.pivot_fc_plan_clone(h) for h in sets[0][0]])
        sets.append((plans, B.pivot_mlp_plan(plans, 0)))
    views = [B.pivot_fc_plan_host_view(h) for h in sets[0][0]]
    assert B.pivot_mlp_plan_host_view(sets[0][1], views)["one_launch"] == 1
    xs = [torch.from_numpy(probs[0].x.copy()).cuda() for _ in range(ncopies)]
    M = probs[-1].M
    yd = torch.empty((1, M), dtype=torch.float32, device="cuda")
    wsb = max(256, B.pivot_mlp_workspace_bytes(sets[0][1], 1))
    ws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
    L = len(probs)
    tr = torch.zeros((L, 1024, 8, 8), dtype=torch.int64, device="cuda")
    os.environ["PIVOT_CHAIN_TRACE_PTR"] = str(tr.data_ptr())
    st = torch.cuda.current_stream().cuda_stream
    res, k = [], 0
    for burst in range(bursts):
        n = (ncopies if ncopies > 1 else 16) + burst
        for _ in range(n):
            j = k % ncopies
            k += 1
            B.pivot_mlp_run(sets[j][1], xs[j].data_ptr(), probs[0].K, yd.data_ptr(), M, 1, ws.data_ptr(), wsb, st)
        torch.cuda.synchronize()
        if burst >= 2:
            res.append(tr.cpu().numpy().astype(np.float64))
    assert all(B.pivot_mlp_status(m, st) == 0 for _, m in sets)
    r = np.stack(res)                                         # [burst][layer][wg][wave][stamp]
    t0 = np.array([b[0][b[0][:, :, 0] > 0][:, 0].min() for b in r])       # first wavefront of layer 1
    print("\n### %s\n" % label)
    print("%s, %d bursts; us since the first wavefront started; per stamp: median over wavefronts / 90th percentile / latest\n"
          % ("cache-cold (rotating through %d copies of the chain)" % ncopies if ncopies > 1 else "warm (one copy)", len(res)))
    print("| layer (work items) | " + " | ".join("%d %s" % (i, n) for i, n in enumerate(CHAIN_PHASES)) + " |")
    print("|---|" + "---|" * len(CHAIN_PHASES))
    for l in range(L):
        nit = views[l]["nchunks"] * views[l]["row_slices"]
        cells = []
        for i in range(len(CHAIN_PHASES)):
            waves = slice(0, 1) if i == 5 else slice(None)        # the outputs are stored by the first wavefront
            a = np.stack([(r[b, l, :nit, waves, i] - t0[b]) / 100.0 for b in range(len(res))])
            cells.append("%.2f / %.2f / %.2f" % (np.median(a), np.percentile(a, 90), a.reshape(len(res), -1).max(axis=1).mean()))
        print("| %d (%d) | %s |" % (l + 1, nit, " | ".join(cells)), flush=True)
    for plans, mlp in sets:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)
    torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true")
    ap.add_argument("--build-ablations", action="store_true")
    ap.add_argument("--ablations", action="store_true")
    ap.add_argument("--time-one", default=None, help=argparse.SUPPRESS)
    ap.add_argument("--cases", default="cfg2,cfg4l1")
    ap.add_argument("--lib", default=TRACE_LIB)
    args = ap.parse_args()
    if args.build:
        build()
        return
    if args.build_ablations:
        build_ablations()
        return
    if args.time_one:
        time_one(args.time_one)
        return
    if args.ablations:
        time_ablations()
        return
    import torch
    from paper_1712_01084_amd import binding as B
    from paper_1712_01084_amd import workloads as WL
    if not os.path.exists(args.lib):
        sys.exit("bench_timeline.py: %s is not built (run with --build first)" % args.lib)
    if not torch.cuda.is_available():
        sys.exit("bench_timeline.py: no GPU visible")
    B.LIB_PATH = args.lib
    B.lib()
    cases = set(args.cases.split(","))
    print("# In-kernel timeline of the batch-1 layer kernel (100 MHz device clock, us since the first wavefront's start)")
    if "cfg2" in cases:
        p = WL.config2(seed=0)
        run_case("configs[1]: 4096x9216 fp32, 32x32 tiles, 10 % balanced, cold", p, 40)
        run_case("configs[1]: 4096x9216 fp32, 32x32 tiles, 10 % balanced, warm", p, 1)
    if "cfg4l1" in cases:
        p = WL.config4(seed=0)[0]
        run_case("configs[3] layer 1: 4096x25088 fp32, 32x32 tiles, 10 % balanced, cold", p, 16)
        run_case("configs[3] layer 1: 4096x25088 fp32, 32x32 tiles, 10 % balanced, warm", p, 1)
    if "cfg4" in cases:
        for elim in (False, True):
            probs = WL.config4(seed=0, eliminated=elim)
            tag = "eliminated" if elim else "composed"
            run_chain("configs[3] chain 25088-4096-4096-1000 fp32 in one launch, %s boundaries, cold" % tag, probs, 12)
            if not elim:
                run_chain("configs[3] chain in one launch, %s boundaries, warm" % tag, probs, 1)
    if "cfg1" in cases:
        p = WL.config1(seed=0)
        run_case("configs[0]: 1024x1024 fp32, 16x16 tiles, 25 % uniform, cold", p, 200)
    if "cfg3d" in cases:
        p = WL.config3(seed=0, frac=1.0)
        run_case("configs[2] dense control: 4096x4096 fp16, 64x16 tiles, cold", p, 18)


if __name__ == "__main__":
    main()
