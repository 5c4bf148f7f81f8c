#!/usr/bin/env python3
"""The paper's own experiment on one MI355X (Section 5, Table 1a): square
matrices of size 64..4096 with 1/fill identical square blocks on the diagonal,
fill-in 3.125 / 6.25 / 12.5 / 25 %, batch 1, fp32.  For each cell:

  * the pruned layer through pivot_fc_run with random permutations,
  * the same with identity permutations (the gather and the scatter become
    contiguous: the paper's permutation-overhead question, Section 5.1.1),
  * with --gather-off: the identity case once more through a build of the
    library that has no permutation code at all (-DPIVOT_ABLATE=32: the kernel
    reads one block column per tile instead of a gather index per column, takes
    the x-segment as BW contiguous elements, and stores a row at its own index
    without a look-up); --build-gather-off makes that build (no GPU needed), the
    timed run loads it in a child process and checks that its outputs have the
    bits of the identity case,
  * the same matrix dense through this library's dense kernel and rocBLAS,
  * the same matrix in CSR through this library's CSR kernel,

warm (same buffers every launch; these matrices are at most 16.8 MB and the
paper's 2,500-call averages are warm too), GPU-side time from replays of
captured graphs (bench_util.py).  Prints JSON lines and the analog
of Table 1a: speedup vs dense / vs CSR.

    python bench_paper_grid.py --build-gather-off          # once, here or on the GPU machine
    python bench_paper_grid.py [--wdtype f32] [--gather-off] [--extended]
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
import scipy.sparse as sp
import torch

from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL
import bench_util as BU


def gt(enqueue, n_launch=100):
    """GPU-side us per launch: replays of a captured graph of n_launch plain launches (bench_util.py)."""
    return BU.graph_time(enqueue, n_launch, replays=5, repeats=3)


def ev_eager(fn, iters):
    fn(20)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn(iters)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def natural_masked(p):
    """The pruned matrix in natural coordinates, storage dtype (input of the comparators)."""
    keep = np.repeat(np.repeat(p.tile_mask.astype(bool), p.bh, 0), p.bw, 1)[:p.M, :p.K]
    W = np.zeros_like(p.Wp)
    W[np.ix_(p.prow, p.pcol)] = np.where(keep, p.Wp, 0)
    return W


def gather_off_lib():
    from paper_1712_01084_amd import build as Bd
    return os.path.join(Bd.HERE, "libpivotfc_abl32.so")


def build_gather_off():
    from paper_1712_01084_amd import build as Bd
    print(Bd.build(out=gather_off_lib(), objdir=os.path.join(Bd.HERE, "_build_trace", "abl32"),
                   device_flags=Bd.DEVICE + ["-DPIVOT_ABLATE=32"], only=["pivot_gemv_f32.hip", "pivot_gemv_f16.hip", "pivot_launch.hip"]))


def y_digest(yd):
    import hashlib
    return hashlib.sha1(yd.cpu().numpy().tobytes()).hexdigest()[:16]


def gather_off_child(args, sizes, wdt, wd):
    """Runs in a process of its own with the build that has no permutation code: identity cases only."""
    B.LIB_PATH = gather_off_lib()
    B.lib()
    st = torch.cuda.current_stream().cuda_stream
    for size in sizes:
        for fill in WL.PAPER_GRID_FILLS:
            p = WL.paper_grid_case(size, fill, seed=args.seed, wdtype=wdt, perms="identity")
            plan = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol,
                                   p.bias, act=p.act, device=0)
            xd = torch.from_numpy(p.x).cuda()
            yd = torch.full((1, p.M), float("nan"), dtype=torch.float32, device="cuda")
            nws = max(256, B.pivot_fc_workspace_bytes(plan, 1))
            ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
            B.pivot_workspace_init(ws.data_ptr(), nws, st)
            t = gt(lambda i, s: B.pivot_fc_run(plan, xd.data_ptr(), p.K, yd.data_ptr(), p.M, 1, ws.data_ptr(), nws, s))
            torch.cuda.synchronize()
            print(json.dumps({"gather_off": True, "size": size, "fill": fill, "us": t, "y": y_digest(yd)}), flush=True)
            B.pivot_fc_plan_destroy(plan)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gather-off", action="store_true", help="add the build without permutation code (see --build-gather-off)")
    ap.add_argument("--build-gather-off", action="store_true")
    ap.add_argument("--gather-off-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--wdtype", default="f32", choices=["f32", "f16"])
    ap.add_argument("--iters", type=int, default=500)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--extended", action="store_true", help="also sizes 8192 and 16384 (beyond the paper's grid)")
    args = ap.parse_args()
    if args.build_gather_off:
        build_gather_off()
        return
    sizes = tuple(WL.PAPER_GRID_SIZES) + ((8192, 16384) if args.extended else ())
    assert torch.cuda.is_available(), "needs a GPU"
    wdt = WL.F32 if args.wdtype == "f32" else WL.F16
    wd = B.PIVOT_F32 if wdt == WL.F32 else B.PIVOT_F16
    if args.gather_off_child:
        gather_off_child(args, sizes, wdt, wd)
        return
    goff = {}
    if args.gather_off:
        import subprocess
        assert os.path.exists(gather_off_lib()), "run with --build-gather-off first"
        cmd = [sys.executable, os.path.abspath(__file__), "--gather-off-child", "--wdtype", args.wdtype, "--seed", str(args.seed)] \
            + (["--extended"] if args.extended else [])
        out = subprocess.run(cmd, stdout=subprocess.PIPE, text=True, check=True).stdout
        for line in out.splitlines():
            if line.startswith("{"):
                d = json.loads(line)
                goff[(d["size"], d["fill"])] = d
    B.lib()
    st = torch.cuda.current_stream().cuda_stream
    table = {}

    print(json.dumps({"case": "null kernel back to back", "us": round(gt(lambda i, s: B.pivot_null_run(s), 200), 2)}), flush=True)

    for size in sizes:
        for fill in WL.PAPER_GRID_FILLS:
            res = {}
            for perms in ("random", "identity"):
                p = WL.paper_grid_case(size, fill, seed=args.seed, wdtype=wdt, perms=perms)
                plan = B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd, p.Wp, B.PIVOT_W_PIVOTED, p.tile_mask, p.prow, p.pcol,
                                       p.bias, act=p.act, device=0)
                xd = torch.from_numpy(p.x).cuda()
                yd = torch.empty((1, p.M), dtype=torch.float32, device="cuda")
                nws = max(256, B.pivot_fc_workspace_bytes(plan, 1))
                ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
                B.pivot_workspace_init(ws.data_ptr(), nws, st)

                res["pbp_" + perms] = gt(lambda i, s: B.pivot_fc_run(plan, xd.data_ptr(), p.K, yd.data_ptr(), p.M, 1,
                                                                     ws.data_ptr(), nws, s))
                if perms == "identity" and goff:
                    torch.cuda.synchronize()
                    g = goff[(size, fill)]
                    assert g["y"] == y_digest(yd), "the build without permutation code computed other bits (%d, %g)" % (size, fill)
                    res["pbp_gather_off"] = g["us"]
                if perms == "random":
                    Wn = natural_masked(p)
                    xv = xd[0]
                    Wd_ = torch.from_numpy(Wn).cuda()
                    bd = torch.from_numpy(p.bias).cuda()

                    res["dense_own"] = gt(lambda i, s: B.pivot_dense_run(Wd_.data_ptr(), wd, p.M, p.K, xd.data_ptr(), p.K,
                                                                         bd.data_ptr(), yd.data_ptr(), p.M, 1, p.act, s))

                    # rocBLAS through torch inside a captured graph as well
                    side = BU.side_stream()
                    yt = torch.empty((p.M,), dtype=Wd_.dtype, device="cuda")
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.stream(side):
                        torch.mv(Wd_, xv, out=yt)
                        side.synchronize()
                        with torch.cuda.graph(g, stream=side):
                            for _ in range(100):
                                torch.mv(Wd_, xv, out=yt)
                    torch.cuda.synchronize()
                    res["dense_rocblas"] = BU.time_graph(g, 100, 5, repeats=3)
                    A = sp.csr_matrix(Wn.astype(np.float32))
                    rp = torch.from_numpy(A.indptr.astype(np.int32)).cuda()
                    ci = torch.from_numpy(A.indices.astype(np.int32)).cuda()
                    va = torch.from_numpy(A.data.astype(Wn.dtype)).cuda()
                    y1 = torch.empty((p.M,), dtype=torch.float32, device="cuda")

                    res["csr_own"] = gt(lambda i, s: B.pivot_csr_run(rp.data_ptr(), ci.data_ptr(), va.data_ptr(), wd, p.M, A.nnz,
                                                                     xv.data_ptr(), bd.data_ptr(), y1.data_ptr(), p.act, s))
                    res["tile"] = p.bh
                    res["block_edge"] = p.meta["block_edge"]
                B.pivot_fc_plan_destroy(plan)
            torch.cuda.empty_cache()
            dense = min(res["dense_own"], res["dense_rocblas"])
            row = {"size": size, "fill_pct": fill * 100, **{k: (round(v, 2) if isinstance(v, float) else v) for k, v in res.items()},
                   "speedup_vs_dense": round(dense / res["pbp_random"], 2),
                   "speedup_vs_csr": round(res["csr_own"] / res["pbp_random"], 2),
                   "perm_overhead_pct": round(100 * (res["pbp_random"] - res["pbp_identity"]) / res["pbp_random"], 1)}
            if "pbp_gather_off" in res:
                row["perm_overhead_vs_gather_off_pct"] = round(100 * (res["pbp_random"] - res["pbp_gather_off"]) / res["pbp_random"], 1)
            table[(size, fill)] = row
            print(json.dumps(row), flush=True)

    print("\nSpeedup of the PBP layer (random permutations) vs dense / vs CSR; linear would be "
          + " / ".join("%g" % (1 / f) for f in WL.PAPER_GRID_FILLS))
    print("| size \\\\ fill-in | " + " | ".join("%g %%" % (100 * f) for f in WL.PAPER_GRID_FILLS) + " |")
    print("|---|" + "---|" * len(WL.PAPER_GRID_FILLS))
    for size in sizes:
        print("| %d | " % size + " | ".join("%.2f / %.2f" % (table[(size, f)]["speedup_vs_dense"], table[(size, f)]["speedup_vs_csr"])
                                            for f in WL.PAPER_GRID_FILLS) + " |")
    if goff:
        print("\nPermutation overhead (Section 5.1.1): time per call in us with random permutations / with identity "
              "permutations / without permutation code, and the share of the first that the permutations cost")
        print("| size \\\\ fill-in | " + " | ".join("%g %%" % (100 * f) for f in WL.PAPER_GRID_FILLS) + " |")
        print("|---|" + "---|" * len(WL.PAPER_GRID_FILLS))
        for size in sizes:
            print("| %d | " % size + " | ".join("%.2f / %.2f / %.2f (%.0f %%)" % (
                table[(size, f)]["pbp_random"], table[(size, f)]["pbp_identity"], table[(size, f)]["pbp_gather_off"],
                table[(size, f)]["perm_overhead_vs_gather_off_pct"]) for f in WL.PAPER_GRID_FILLS) + " |")
    print("\nTime per call in us: PBP random perms / PBP identity perms / dense (best) / CSR")
    print("| size \\\\ fill-in | " + " | ".join("%g %%" % (100 * f) for f in WL.PAPER_GRID_FILLS) + " |")
    print("|---|" + "---|" * len(WL.PAPER_GRID_FILLS))
    for size in sizes:
        cells = []
        for f in WL.PAPER_GRID_FILLS:
            r = table[(size, f)]
            cells.append("%.2f / %.2f / %.2f / %.2f" % (r["pbp_random"], r["pbp_identity"], min(r["dense_own"], r["dense_rocblas"]), r["csr_own"]))
        print("| %d | " % size + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()
