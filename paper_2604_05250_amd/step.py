"""Replaying one draft-then-verify cycle (Alg. 1) as a HIP graph.

The cycle is a fixed sequence of a dozen kernel launches on fixed buffers; for the small workloads the
launches themselves (host marshalling, launch latency between dependent kernels) are a sizeable part of
its time.  Capturing the sequence once and replaying it removes the host from the loop.  The library only
launches kernels on the caller's stream - no allocation, no memset, no synchronisation - so every call of
the binding can be captured as it is.
"""
from __future__ import annotations

from typing import Callable


def capture_step(fn: Callable[[], None], warmup: int = 2):
    """Run `fn` (calls of this package on fixed tensors) `warmup` times on a side stream, then record it once.
    The scratch memory of the recorded calls is one tensor allocated here, before the capture, at the largest
    size the warm-up calls asked for; the returned torch.cuda.CUDAGraph keeps it alive (`graph.dd_workspace`).
    `graph.replay()` enqueues the whole sequence on the current stream; replays of one graph share that scratch
    tensor and must not overlap each other."""
    import torch

    import paper_2604_05250_amd as dd
    side = torch.cuda.Stream()                    # default priority
    side.wait_stream(torch.cuda.current_stream())
    dd.reset_workspace_peak()
    with torch.cuda.stream(side):
        for _ in range(max(1, warmup)):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    ws = torch.empty(max(dd.workspace_peak(), 256), dtype=torch.uint8, device=torch.cuda.current_device())
    graph = torch.cuda.CUDAGraph()
    with dd.fixed_workspace(ws):
        with torch.cuda.graph(graph):
            fn()
    graph.dd_workspace = ws
    return graph
