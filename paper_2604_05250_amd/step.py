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
    """Run `fn` (calls of this package on fixed tensors) `warmup` times on a side stream, then record it once
    (the binding keeps one scratch tensor per stream; the one of the capture stream is allocated during capture
    and belongs to the graph's memory pool).  Returns the torch.cuda.CUDAGraph;
    `graph.replay()` enqueues the whole sequence on the current stream."""
    import torch
    side = torch.cuda.Stream()                    # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(max(1, warmup)):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    return graph
