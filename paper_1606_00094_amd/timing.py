"""Device-side timing helpers shared by bench.py and the tuning sweep.

Launches are captured into a HIP graph and the graph is replayed between HIP
events on the launch stream, so the figure holds kernel time and the device's
own kernel-to-kernel gap but no host launch overhead.

The card idles at a low clock and takes tens of milliseconds of load to reach
its working clock (a launch measured right after a host-side pause is 5-10 %
slower than the same launch in a busy stream), so every measurement first keeps
the device busy for `spin_ms` and then times replays enqueued back to back.
"""
import math

import torch


def graph_time_us(fn, launches=20, replays=5, best=False, spin_ms=50.0):
    """Microseconds per call of fn() (which must only enqueue work on torch's
    current stream), from replaying a captured graph of `launches` back-to-back
    calls: after `spin_ms` of untimed replays, `replays` timed replays enqueued
    without a host synchronisation in between; the mean of them, or the fastest
    with best=True (used to rank candidates in the sweep)."""
    fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(launches):
            fn()
    # one replay, timed, to size the spin-up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    first_ms = max(e0.elapsed_time(e1), 1e-3)
    for _ in range(min(20000, int(math.ceil(spin_ms / first_ms)))):
        g.replay()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
    marks[0].record()
    for i in range(replays):
        g.replay()
        marks[i + 1].record()
    torch.cuda.synchronize()
    times = [marks[i].elapsed_time(marks[i + 1]) * 1e3 / launches for i in range(replays)]
    del g
    return min(times) if best else sum(times) / len(times)
