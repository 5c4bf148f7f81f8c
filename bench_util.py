"""Timing helper shared by the benchmark scripts.

Launching through Python costs about 5 us of host time per call, more than
the GPU needs for the small layers, so a loop of eager calls measures the host.
The launches are therefore captured once into a HIP graph (plain kernel
launches only: the library enqueues no memset or copy nodes) and the graph is
replayed; HIP events around the replays give the GPU-side time per launch,
back to back on one stream.
"""
from __future__ import annotations

import numpy as np
import torch

_side = None


def side_stream():
    global _side
    if _side is None:
        _side = torch.cuda.Stream()
    return _side


def capture(enqueue, n_launch):
    """Graph of launches enqueue(0, s) .. enqueue(n_launch-1, s); `s` is the raw stream handle."""
    side = side_stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for i in range(min(n_launch, 8)):
            enqueue(i, side.cuda_stream)        # make sure every kernel is loaded before capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for i in range(n_launch):
                enqueue(i, side.cuda_stream)
    torch.cuda.synchronize()
    return g


def time_graph(g, n_launch, replays, warm_replays=2, repeats=1, stats=False):
    """us per launch: HIP events around `replays` replays of a graph of n_launch launches; the median over
    `repeats` such measurements (stats=True: the pair (median, min))."""
    for _ in range(warm_replays):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ts = []
    for _ in range(repeats):
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / (replays * n_launch))
    if stats:
        return float(np.median(ts)), float(min(ts))
    return float(np.median(ts))


def graph_time(enqueue, n_launch, replays=5, repeats=3, stats=False):
    g = capture(enqueue, n_launch)
    return time_graph(g, n_launch, replays, repeats=repeats, stats=stats)


_floor_cache = {}


def stream_floor(nbytes, footprint=2 * (256 + 32) * (1 << 20)):
    """(cold_us, warm_us) of ONE launch that only reads `nbytes` (pivot_stream_read_run): the measured ceiling
    for a single launch of that size.  Cold rotates through separate regions of >= `footprint` bytes in total."""
    from paper_1712_01084_amd import binding as B
    kb = max(1, int(nbytes) // 1024)
    if kb in _floor_cache:
        return _floor_cache[kb]
    n = kb * 1024
    stride = -(-n // 4096) * 4096
    ncopies = int(max(2, min(600, -(-footprint // n))))
    buf = torch.zeros(ncopies * stride, dtype=torch.uint8, device="cuda")
    out = torch.empty(2048, dtype=torch.float32, device="cuda")
    base = buf.data_ptr()
    cold = graph_time(lambda i, s: B.pivot_stream_read_run(base + (i % ncopies) * stride, n, out.data_ptr(), s),
                      ncopies * max(1, 64 // ncopies), replays=4)
    warm = graph_time(lambda i, s: B.pivot_stream_read_run(base, n, out.data_ptr(), s), 100, replays=6)
    del buf
    torch.cuda.empty_cache()
    _floor_cache[kb] = (cold, warm)
    return cold, warm
