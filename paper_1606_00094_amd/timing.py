"""Device-side timing helpers shared by bench.py and the tuning sweep.

Launches are captured into a HIP graph and the graph is replayed between two
HIP events on the launch stream, so the figure holds kernel time and the
device's own kernel-to-kernel gap but no host launch overhead.
"""
import torch


def graph_time_us(fn, launches=20, replays=5, best=False):
    """Microseconds per call of fn() (which must only enqueue work on torch's
    current stream), from replaying a captured graph of `launches` back-to-back
    calls: the mean over `replays` timed replays (after one untimed replay), or
    the fastest replay with best=True (used to rank candidates in the sweep)."""
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
    g.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / launches)
    del g
    return min(times) if best else sum(times) / len(times)
