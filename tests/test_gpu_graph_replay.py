"""The library under HIP graph capture, on the GPU.

bench.py and the tuning sweep time replays of captured graphs, and serving loops are the
callers conv_fwd_noalloc exists for; so a captured sequence of library calls must give, on
every replay, exactly what the same calls give eagerly on the same inputs.  Each case is
replayed three times, the input buffers rewritten between replays, with eager launches and
synchronisations of the program's own in between.  (The library enqueues kernels only: no
memory-set nodes end up in the graph.)
"""
import numpy as np
import pytest
import torch

import workloads
from paper_1606_00094_amd import binding

pytestmark = pytest.mark.gpu


def _capture(fn):
    fn()                                     # first call outside the capture (attribute set-up)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def _replays_equal_eager(fn, inputs, outputs, fresh_inputs):
    """fn reads `inputs` and writes `outputs` (device tensors).  Three replays of its captured
    graph, each on new input contents, against the eager call on those contents."""
    g = _capture(fn)
    for rep in range(3):
        for t, new in zip(inputs, fresh_inputs(rep)):
            t.copy_(new)
        for o in outputs:
            o.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        replayed = [o.clone() for o in outputs]
        for o in outputs:
            o.fill_(float("nan"))
        fn()                                 # eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(replayed, outputs):
            assert not torch.isnan(b).any()
            assert torch.equal(a, b), "replay %d differs from the eager call" % rep


def test_noalloc_split_layer_and_pooled_call_replay():
    """conv_fwd_noalloc on a layer whose choice splits the reduction (main kernel + reduction
    kernel through the static scratch array) followed by the convolution + pooling call."""
    dev = torch.device("cuda:0")
    l3, l5, N = workloads.CONV3, workloads.CONV5, 2
    x, f, b = workloads.make_layer_inputs(l3, N)
    _, f5, b5 = workloads.make_layer_inputs(l5, N)
    xd, fd, bd = (torch.from_numpy(a).to(dev) for a in (x, f, b))
    f5d, b5d = torch.from_numpy(f5).to(dev), torch.from_numpy(b5).to(dev)
    dims3 = (N, l3.C, l3.H, l3.W, l3.K, 3, 3, 1, 1)
    assert binding.conv_variant_name(binding.conv_selected_variant(*dims3)).split("/s")[1] != "1"
    mid = torch.empty((N, l3.K, 13, 13), dtype=torch.float32, device=dev)
    x5 = torch.empty((N, l5.C, 13, 13), dtype=torch.float32, device=dev)
    dims5 = (N, l5.C, 13, 13, l5.K, 3, 3, 1, 1)
    ws = torch.zeros(binding.conv_pool_fwd_workspace_bytes(*dims5, -1) // 4 + 1, dtype=torch.float32, device=dev)
    out = torch.empty((N, l5.K, 6, 6), dtype=torch.float32, device=dev)

    def fn():
        binding.conv_fwd_noalloc(xd, fd, bd, mid, 1, 1, True)
        binding.conv_pool_fwd_ex(x5, f5d, b5d, out, 1, 1, True, 3, 2, ws)

    rng = np.random.default_rng(workloads.BASE_SEED + 901)

    def fresh(rep):
        return (torch.from_numpy(rng.random(x.shape, dtype=np.float32)).to(dev),
                torch.from_numpy(rng.random(tuple(x5.shape), dtype=np.float32)).to(dev))

    _replays_equal_eager(fn, (xd, x5), (mid, out), fresh)


def test_half_precision_stack_replays():
    """The five-layer stack in half precision (first-layer kernel with its preparation launch,
    C8 layers with packed filters, both poolings) as one captured graph."""
    import bench
    dev = torch.device("cuda:0")
    N = 5
    img, params = workloads.make_stack_inputs(N)
    st = bench.F16Stack(N, img, params)
    final = st.acts[-1][0]
    rng = np.random.default_rng(workloads.BASE_SEED + 902)

    def fresh(rep):
        return (torch.from_numpy(rng.random(img.shape, dtype=np.float32)).to(dev).half(),)

    _replays_equal_eager(st.step, (st.x,), (final,), fresh)
