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


def time_graph(g, n_launch, replays, warm_replays=2, repeats=1):
    """us per launch: HIP events around `replays` replays of a graph of n_launch launches."""
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
    return float(np.median(ts))


def graph_time(enqueue, n_launch, replays=5, repeats=3):
    g = capture(enqueue, n_launch)
    return time_graph(g, n_launch, replays, repeats=repeats)
