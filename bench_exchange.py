#!/usr/bin/env python3
"""What one trip between two workgroups of a launch costs on this GPU: the unit
the one-launch forms (the chain of layers, Section 4.2, and the recurrent loop)
pay at every hand-over.  Runs pivot_exchange_probe_run a few times and prints
the one-way time of a 4-byte word for a pair of workgroups on one XCD and on two
XCDs, with the device-coherent accesses the kernels use and with two candidates
for a shorter path inside an XCD.

    python bench_exchange.py [--rounds 2000] [--reps 5]
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_1712_01084_amd import binding as B


def probe(rounds):
    """One run: dict of one-way microseconds per mechanism (None: the wait gave up), partners."""
    buf = torch.empty(B.PIVOT_PROBE_SCRATCH_BYTES + 256, dtype=torch.uint8, device="cuda")
    off = (-buf.data_ptr()) % 256
    B.pivot_exchange_probe_run(buf.data_ptr() + off, B.PIVOT_PROBE_SCRATCH_BYTES, rounds, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    out = buf[off:off + 64].cpu().numpy().view(np.int64)
    tab = buf[off + 1024:off + 2048].cpu().numpy().view(np.uint32)
    if out[0] != 1:
        raise RuntimeError("the probe did not run (status %d): workgroups not all resident, or one XCD only" % out[0])
    us = lambda ticks: None if ticks < 0 else ticks / 100.0 / (2 * rounds)       # 100 MHz clock, two trips per round
    return {"same_xcd_device_coherent": us(out[1]), "same_xcd_workgroup_scope": us(out[2]),
            "same_xcd_l1_invalidate_plain_load": us(out[6]), "other_xcd_device_coherent": us(out[3]),
            "partner_same": int(out[4]), "partner_other": int(out[5]), "xcd_of_workgroup": (tab.astype(np.int64) - 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rounds", type=int, default=2000)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    runs = [probe(args.rounds) for _ in range(args.reps)]
    x = runs[0]["xcd_of_workgroup"]
    n = int((x >= 0).sum())
    print("%d workgroups, one per compute unit; XCD of workgroups 0..15: %s" % (n, " ".join(str(v) for v in x[:16])))
    print("partners of workgroup 0: %d (same XCD), %d (other XCD); %d round trips per series, %d runs\n"
          % (runs[0]["partner_same"], runs[0]["partner_other"], args.rounds, args.reps))
    print("| pair, mechanism | us one way: median (min - max) |")
    print("|---|---|")
    rows = [("same XCD, device-coherent store and load", "same_xcd_device_coherent"),
            ("other XCD, device-coherent store and load", "other_xcd_device_coherent"),
            ("same XCD, plain store, L1 invalidate + plain load", "same_xcd_l1_invalidate_plain_load"),
            ("same XCD, workgroup-scope atomics", "same_xcd_workgroup_scope")]
    for label, key in rows:
        v = [r[key] for r in runs]
        if any(t is None for t in v):
            print("| %s | the wait gave up in %d of %d runs (the update was never seen) |" % (label, sum(t is None for t in v), len(v)))
        else:
            print("| %s | %.2f (%.2f - %.2f) |" % (label, float(np.median(v)), min(v), max(v)))


if __name__ == "__main__":
    main()
