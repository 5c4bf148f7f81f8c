#!/usr/bin/env python3
"""The paper's three tile layouts (Section 4.1.1: BRC, BCR, CBR) on one MI355X,
the analog of its layout comparison (Section 4.1.2, Table 2): the same pruned
layer, batch 1, through the row-major kernel (BRC; with and without row
slicing) and through the column-major kernels (BCR, CBR), cache-cold and warm,
GPU-side time from replays of captured graphs.

    python bench_layouts.py [--cases cfg1,cfg2,...]

Under `rocprofv3 --pmc FETCH_SIZE` the per-kernel counter of this script gives
the bytes each layout really fetches (load efficiency = algorithmic / fetched).
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

COLD_FOOTPRINT = 2 * (256 + 32) * (1 << 20)
LAYOUTS = (("BRC", B.PIVOT_BRC, 0), ("BRC unsliced", B.PIVOT_BRC, 1), ("BCR", B.PIVOT_BCR, 1), ("CBR", B.PIVOT_CBR, 1))


def cases():
    yield "cfg1 1024x1024 f32 16x16 25%", WL.config1()
    yield "cfg2 4096x9216 f32 32x32 10%", WL.config2()
    yield "cfg3 4096x4096 f16 64x16 25%", WL.config3(frac=0.25)
    yield "cfg3 4096x4096 f16 64x16 100%", WL.config3(frac=1.0)
    yield "cfg4 layer 1 4096x25088 f32 32x32 10%", WL.config4()[0]
    yield "grid 4096 25% f32 (4 blocks of 1024, 64x64 tiles)", WL.paper_grid_case(4096, 0.25)
    yield "cfg5 gates 8192x3072 f16 16x32 zipf", _with_x(WL.config5(steps=1).fc)


def _with_x(p):
    p.x = np.random.default_rng(5).standard_normal((1, p.K)).astype(p.Wp.dtype)
    return p


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cases", default="")
    ap.add_argument("--no-cold", action="store_true")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    B.lib()
    st = torch.cuda.current_stream().cuda_stream
    rows = []
    for name, p in cases():
        if args.cases and not any(c in name for c in args.cases.split(",")):
            continue
        wd = B.PIVOT_F32 if p.wdtype == WL.F32 else B.PIVOT_F16
        alg = p.algorithmic_bytes(1)
        ncopies = int(max(2, min(300, -(-COLD_FOOTPRINT // alg))))
        for lname, layout, sl in LAYOUTS:
            plan0 = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol,
                                    p.bias, act=p.act, layout=layout, row_slices=sl, device=0)
            v = B.pivot_fc_plan_host_view(plan0)
            plans = [plan0] + ([] if args.no_cold else [B.pivot_fc_plan_clone(plan0) for _ in range(ncopies - 1)])
            xs = [torch.from_numpy(p.x[:1].copy()).cuda() for _ in range(len(plans))]
            yd = torch.empty((1, p.M), dtype=torch.float32, device="cuda")
            nws = max(256, B.pivot_fc_workspace_bytes(plan0, 1))
            ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
            B.pivot_workspace_init(ws.data_ptr(), nws, st)

            def go(rot):
                n = len(plans)
                return lambda i, s: B.pivot_fc_run(plans[i % n if rot else 0], xs[i % n if rot else 0].data_ptr(), p.K,
                                                   yd.data_ptr(), p.M, 1, ws.data_ptr(), nws, s)
            warm = BU.graph_time(go(False), 100, replays=4, repeats=3)
            cold = None if args.no_cold else BU.graph_time(go(True), len(plans) * max(1, 64 // len(plans)), replays=4, repeats=3)
            row = {"case": name, "layout": lname, "warm_us": round(warm, 2), "cold_us": None if cold is None else round(cold, 2),
                   "warm_GBs": round(alg / warm / 1e3, 1), "cold_GBs": None if cold is None else round(alg / cold / 1e3, 1),
                   "work_items": v["nchunks"] * v["row_slices"], "wg_waves": v["wg_waves"], "chunk_tiles": v["chunk_tiles"]}
            rows.append(row)
            print(json.dumps(row), flush=True)
            for h in plans:
                B.pivot_fc_plan_destroy(h)
            torch.cuda.empty_cache()
    print("\n| case | layout | warm us | warm GB/s | cold us | cold GB/s | work items x waves |")
    print("|---|---|---|---|---|---|---|")
    for r in rows:
        print("| %s | %s | %s | %s | %s | %s | %d x %d |" % (r["case"], r["layout"], r["warm_us"], r["warm_GBs"],
                                                            r["cold_us"], r["cold_GBs"], r["work_items"], r["wg_waves"]))


if __name__ == "__main__":
    main()
