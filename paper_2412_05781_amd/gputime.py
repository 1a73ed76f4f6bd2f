"""GPU timing helper for bench.py and the timing tables: average duration of one call, host launch cost excluded."""
from __future__ import annotations

import torch


def graph_time(fn, reps: int, replays: int = 4) -> float:
    """Seconds per call of fn(i): `reps` calls are captured in a HIP graph on a side stream and the graph is replayed
    between two HIP events recorded on that same stream (the stream the kernels run on); best of `replays` replays."""
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for i in range(2):
            fn(i)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for i in range(reps):
                fn(i)
        g.replay()
        side.synchronize()
        best = float("inf")
        for _ in range(replays):
            a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(side)
            g.replay()
            z.record(side)
            side.synchronize()
            best = min(best, a.elapsed_time(z))
    return best / reps * 1e-3
