"""Benchmark of the forward convolution library on one MI355X.

A step is one pass of the hot path over every benchmark layer shape (first
layer, the four middle layers, the three pointwise and the two reduce layers)
at batch 32, each call = variant selection + tiled MFMA kernel (+ split
reduction) with fused bias + ReLU, inputs already resident in HBM.  `value` is
the algorithmic GFLOP/s of that pass (2 flops per multiply-accumulate, the
convention of the paper's SGEMM tables).  The same JSON line carries the
per-layer table at batch 1 and 32 with both roofline fractions (and the same
layers with half-precision storage, as context), the five-layer
stack at batch 1/5/20/32, the roofline of the dominant kernel measured with HIP
events, and the CPU oracle timed on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "conv fwd GFLOP/s (fp32) per layer at batch 1 and 32; % of fp32 MFMA/HBM roof"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class LayerProblem:
    """Device tensors of one (layer, N) problem, `copies` rotating sets."""

    def __init__(self, layer, N, copies=1, half=False):
        import torch
        import workloads
        from paper_1606_00094_amd import binding, roofline
        self.layer, self.N, self.half = layer, N, half
        dev = torch.device("cuda:0")
        x, f, b = workloads.make_layer_inputs(layer, N)
        P, Q = binding.conv_out_dims(layer.H, layer.W, layer.R, layer.S, layer.stride, layer.pad)
        self.dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
        self.flops = roofline.conv_flops(*self.dims)
        self.bytes = roofline.conv_bytes(*self.dims)
        if half:   # in, filt, out stored as fp16; the bias stays fp32
            self.bytes = (self.bytes - 4 * layer.K) // 2 + 4 * layer.K
        if half:
            self.variant = binding.conv_fwd_f16_selected_variant(*self.dims)
            need = binding.conv_fwd_f16_workspace_bytes(*self.dims, self.variant)
        else:
            self.variant = binding.conv_selected_variant(*self.dims)
            need = binding.conv_fwd_workspace_bytes(*self.dims, self.variant)
        self.ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)
        xd, fd, bd = (torch.from_numpy(a).to(dev) for a in (x, f, b))
        store = torch.float16 if half else torch.float32
        xd, fd = xd.to(store), fd.to(store)
        self.sets = []
        for c in range(copies):
            self.sets.append((xd if c == 0 else xd.clone(), fd if c == 0 else fd.clone(), bd,
                              torch.empty((N, layer.K, P, Q), dtype=store, device=dev)))
        self.k = 0

    def prepack(self):
        """Half precision, fp16-matrix-core tile: re-lay the filters once (deployment keeps its
        weights); launch() then runs the packed call.  Returns False when there is nothing to pack."""
        import torch
        from paper_1606_00094_amd import binding
        nbytes = binding.conv_f16_packed_filter_bytes(*self.dims, self.variant) if self.half else 0
        if not nbytes:
            return False
        self.packed = []
        for x, f, b, o in self.sets:
            pk = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=x.device)
            binding.conv_f16_pack_filters(f, pk, self.N, self.layer.H, self.layer.W, self.layer.stride,
                                          self.layer.pad, variant=self.variant)
            self.packed.append(pk)
        torch.cuda.synchronize()
        return True

    def to_c8(self):
        """Half precision on octet-interleaved activations (how a chain of half-precision layers
        keeps them): input converted once, filters packed once for the tile chosen for that
        layout; launch() then runs the layout call, C8 out where K allows.  Returns the tile's
        name, or None when no fp16-matrix-core tile serves the shape."""
        import torch
        from paper_1606_00094_amd import binding
        N, C, H, W, K = self.dims[:5]
        try:
            v = binding.conv_fwd_f16_c8_selected_variant(*self.dims) if self.half and C % 8 == 0 else -1
        except binding.BconvError:
            v = -1
        if v < 0:
            return None
        P, Q = self.sets[0][3].shape[2:]
        olay = binding.LAYOUT_C8 if K % 8 == 0 else binding.LAYOUT_NCHW
        nbytes = binding.conv_f16_packed_filter_bytes(*self.dims, v)
        self.c8 = []
        for x, f, b, o in self.sets:
            pk = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=x.device)
            binding.conv_f16_pack_filters(f, pk, N, H, W, self.layer.stride, self.layer.pad, variant=v)
            x8 = torch.empty((N, C // 8, H, W, 8), dtype=torch.float16, device=x.device)
            binding.f16_layout_convert(x, binding.LAYOUT_NCHW, x8, binding.LAYOUT_C8, (N, C, H, W))
            o8 = torch.empty((N, K // 8, P, Q, 8), dtype=torch.float16, device=x.device) if olay else o
            self.c8.append((x8, pk, o8, olay, v))
        torch.cuda.synchronize()
        return binding.conv_variant_name(v)

    def launch(self):
        from paper_1606_00094_amd import binding
        x, f, b, o = self.sets[self.k]
        if getattr(self, "c8", None):
            x8, pk, o8, olay, v = self.c8[self.k]
            self.k = (self.k + 1) % len(self.sets)
            binding.conv_fwd_f16_packed_layout_ex(x8, binding.LAYOUT_C8, pk, f.shape, b, o8, olay, tuple(x.shape),
                                                  self.layer.stride, self.layer.pad, True, variant=v)
            return
        if getattr(self, "packed", None):
            pk = self.packed[self.k]
            self.k = (self.k + 1) % len(self.sets)
            binding.conv_fwd_f16_packed_ex(x, pk, f.shape, b, o, self.layer.stride, self.layer.pad, True,
                                           variant=self.variant)
            return
        self.k = (self.k + 1) % len(self.sets)
        fn = binding.conv_fwd_f16_ex if self.half else binding.conv_fwd_ex
        fn(x, f, b, o, self.layer.stride, self.layer.pad, True, workspace=self.ws,
           variant=self.variant)


def time_launches(fn, reps, warm=3):
    """Average milliseconds per call of fn over `reps` back-to-back calls, by HIP
    events on torch's current stream (the stream the library launches on)."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def layer_row(prob, ms, mode):
    from paper_1606_00094_amd import binding, roofline
    t = ms * 1e-3
    return {
        "layer": prob.layer.name, "N": prob.N, "mode": mode,
        "variant": binding.conv_variant_name(prob.variant),
        "us": round(ms * 1e3, 2),
        "gflops": round(prob.flops / t / 1e9, 1),
        "frac_mfma": round(prob.flops / t / 1e12 / roofline.PEAK_FP32_MFMA_TFLOPS, 4),
        "gbps": round(prob.bytes / t / 1e9, 1),
        "frac_hbm": round(prob.bytes / t / 1e9 / roofline.PEAK_HBM_GBPS, 4),
    }


def recorded_traffic(prob):
    """HBM bytes per call (all its kernels) as measured with rocprofv3 FETCH_SIZE /
    WRITE_SIZE (two separate counter runs, scaled by a calibration copy) and recorded in
    profiles/traffic.json; None if there is no record for this layer and batch or the record
    was taken with another variant than the one running now."""
    from paper_1606_00094_amd import binding
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as fh:
            recs = json.load(fh)["records"]
    except (OSError, ValueError, KeyError):
        return None
    for rec in recs:
        if (rec.get("layer") == prob.layer.name and rec.get("N") == prob.N
                and rec.get("variant") == binding.conv_variant_name(prob.variant)):
            return rec.get("bytes")
    return None


def run_sgemm(n):
    """Square matrix product of size n through the sgemm entry point (the sizes of the
    paper's SGEMM tables; reported as context beside the pointwise layers)."""
    import torch
    import workloads
    from paper_1606_00094_amd import binding, roofline
    from paper_1606_00094_amd.timing import graph_time_us
    dev = torch.device("cuda:0")
    a, b = workloads.make_sgemm_inputs(n)
    ad, bd = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
    c = torch.empty((n, n), dtype=torch.float32, device=dev)
    need = binding.sgemm_workspace_bytes(n, n, n)
    ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)
    us = graph_time_us(lambda: binding.sgemm_ex(ad, bd, c, workspace=ws), launches=20)
    gf = roofline.sgemm_flops(n, n, n) / us / 1e3
    return {"size": n, "us": round(us, 2), "gflops": round(gf, 1),
            "frac_mfma": round(gf / 1e3 / roofline.PEAK_FP32_MFMA_TFLOPS, 4),
            "variant": binding.conv_variant_name(binding.conv_selected_variant(1, n, 1, n, n, 1, 1, 1, 0))}


def run_stack(N, reps):
    """Five-layer stack with 3x3/s2 max pooling after the first two layers (those two
    through the convolution + pooling call)."""
    import torch
    import workloads
    from paper_1606_00094_amd import binding, roofline
    dev = torch.device("cuda:0")
    img, params = workloads.make_stack_inputs(N)
    cur_shape = img.shape
    bufs, plan, flops = [torch.from_numpy(img).to(dev)], [], 0
    for li, (layer, (f, b)) in enumerate(zip(workloads.STACK, params)):
        n, c, h, w = cur_shape
        dims = (n, c, h, w, layer.K, layer.R, layer.S, layer.stride, layer.pad)
        P, Q = binding.conv_out_dims(h, w, layer.R, layer.S, layer.stride, layer.pad)
        pooled = li in workloads.STACK_POOL_AFTER
        v = binding.conv_pool_selected_variant(*dims, 3, 2) if pooled else binding.conv_selected_variant(*dims)
        need = (binding.conv_pool_fwd_workspace_bytes if pooled else binding.conv_fwd_workspace_bytes)(*dims, v)
        ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)
        shape = (n, layer.K) + (binding.conv_out_dims(P, Q, 3, 3, 2, 0) if pooled else (P, Q))
        out = torch.empty(shape, dtype=torch.float32, device=dev)
        plan.append((len(bufs) - 1, len(bufs), torch.from_numpy(f).to(dev), torch.from_numpy(b).to(dev),
                     layer, ws, v, pooled))
        bufs.append(out)
        flops += roofline.conv_flops(*dims)
        cur_shape = out.shape

    def step():
        for i, o, f, b, layer, ws, v, pooled in plan:
            if pooled:
                binding.conv_pool_fwd_ex(bufs[i], f, b, bufs[o], layer.stride, layer.pad, True, 3, 2, ws,
                                         variant=v)
            else:
                binding.conv_fwd_ex(bufs[i], f, b, bufs[o], layer.stride, layer.pad, True,
                                    workspace=ws, variant=v)

    ms = graph_time_us(step, launches=reps) * 1e-3
    return {"N": N, "ms": round(ms, 4), "gflops": round(flops / (ms * 1e-3) / 1e9, 1),
            "frac_mfma": round(flops / (ms * 1e-3) / 1e12 / roofline.PEAK_FP32_MFMA_TFLOPS, 4)}


class F16Stack:
    """The five-layer stack with half-precision storage, laid out for the fp16 matrix cores: the
    first layer (three channels, NCHW input) writes the octet-interleaved layout directly when
    its choice is a first-layer fp16-matrix-core tile (else NCHW, pooled there and converted
    once); both poolings and the other four layers run in that layout, filters packed beforehand.
    step() enqueues the whole chain."""

    def __init__(self, N, img, params):
        import torch
        import workloads
        from paper_1606_00094_amd import binding, roofline
        B = binding
        dev = torch.device("cuda:0")
        self.N, self.flops = N, 0
        half = lambda a: torch.from_numpy(a).to(dev).half()
        self.x = half(img)
        self.ops, self.acts = [], []     # acts: (tensor, layout, logical shape) after each conv (+ pool)
        cur, cur_shape, lay = self.x, tuple(img.shape), B.LAYOUT_NCHW
        for li, (layer, (f, b)) in enumerate(zip(workloads.STACK, params)):
            n, c, h, w = cur_shape
            dims = (n, c, h, w, layer.K, layer.R, layer.S, layer.stride, layer.pad)
            P, Q = B.conv_out_dims(h, w, layer.R, layer.S, layer.stride, layer.pad)
            self.flops += roofline.conv_flops(*dims)
            fd, bd = half(f), torch.from_numpy(b).to(dev)
            oshape = (n, layer.K, P, Q)
            if lay == B.LAYOUT_NCHW:     # first layer: NCHW in, straight into the layout the chain keeps
                v = B.conv_fwd_f16_selected_variant(*dims)
                need = B.conv_fwd_f16_workspace_bytes(*dims, v)
                ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)
                direct = B.conv_variant_name(v).startswith(("h16k11s4", "h16k7s2")) and layer.K % 8 == 0
                if direct:
                    out = torch.empty((n, layer.K // 8, P, Q, 8), dtype=torch.float16, device=dev)
                    self.ops.append(lambda cur=cur, fd=fd, bd=bd, out=out, l=layer, ws=ws, v=v, shp=cur_shape:
                                    B.conv_fwd_f16_layout_ex(cur, B.LAYOUT_NCHW, fd, bd, out, B.LAYOUT_C8, shp,
                                                             l.stride, l.pad, True, ws, variant=v))
                    lay = B.LAYOUT_C8
                else:
                    out = torch.empty(oshape, dtype=torch.float16, device=dev)
                    self.ops.append(lambda cur=cur, fd=fd, bd=bd, out=out, l=layer, ws=ws, v=v:
                                    B.conv_fwd_f16_ex(cur, fd, bd, out, l.stride, l.pad, True, workspace=ws,
                                                      variant=v))
            else:
                v = B.conv_fwd_f16_c8_selected_variant(*dims)
                pk = torch.empty(B.conv_f16_packed_filter_bytes(*dims, v) // 2, dtype=torch.float16, device=dev)
                B.conv_f16_pack_filters(fd, pk, n, h, w, layer.stride, layer.pad, variant=v)
                out = torch.empty((n, layer.K // 8, P, Q, 8), dtype=torch.float16, device=dev)
                self.ops.append(lambda cur=cur, pk=pk, fs=tuple(fd.shape), bd=bd, out=out, l=layer, v=v,
                                shp=cur_shape:
                                B.conv_fwd_f16_packed_layout_ex(cur, B.LAYOUT_C8, pk, fs, bd, out, B.LAYOUT_C8, shp,
                                                                l.stride, l.pad, True, variant=v))
            cur, cur_shape = out, oshape
            if li in workloads.STACK_POOL_AFTER:
                PP, PQ = B.conv_out_dims(P, Q, 3, 3, 2, 0)
                pshape = (n, layer.K, PP, PQ)
                pout = torch.empty(pshape if lay == B.LAYOUT_NCHW else (n, layer.K // 8, PP, PQ, 8),
                                   dtype=torch.float16, device=dev)
                self.ops.append(lambda cur=cur, pout=pout, lay=lay, shp=cur_shape:
                                B.maxpool_fwd_f16(cur, pout, lay, shp, 3, 2))
                cur, cur_shape = pout, pshape
            if lay == B.LAYOUT_NCHW:     # into the layout the rest of the chain keeps
                c8 = torch.empty((cur_shape[0], cur_shape[1] // 8) + cur_shape[2:] + (8,), dtype=torch.float16,
                                 device=dev)
                self.ops.append(lambda cur=cur, c8=c8, shp=cur_shape:
                                B.f16_layout_convert(cur, B.LAYOUT_NCHW, c8, B.LAYOUT_C8, shp))
                cur, lay = c8, B.LAYOUT_C8
            self.acts.append((cur, cur_shape))
        torch.cuda.synchronize()

    def step(self):
        for op in self.ops:
            op()

    def activations_nchw(self):
        """The input and each layer's (pooled) output as NCHW numpy arrays, after step()."""
        import torch
        from paper_1606_00094_amd import binding as B
        outs = [self.x.cpu().numpy()]
        for t, shape in self.acts:
            back = torch.empty(shape, dtype=torch.float16, device=t.device)
            B.f16_layout_convert(t, B.LAYOUT_C8, back, B.LAYOUT_NCHW, shape)
            torch.cuda.synchronize()
            outs.append(back.cpu().numpy())
        return outs


def run_stack_f16(N, reps):
    import workloads
    from paper_1606_00094_amd import roofline
    img, params = workloads.make_stack_inputs(N)
    st = F16Stack(N, img, params)
    ms = graph_time_us(st.step, launches=reps) * 1e-3
    return {"N": N, "ms": round(ms, 4), "gflops": round(st.flops / (ms * 1e-3) / 1e9, 1), "kernels": len(st.ops)}


def cpu_baseline(layers, N, min_seconds=10.0, max_passes=8):
    """The oracle as it stands, timed on this machine's host cores over whole passes of
    the same layer set at batch N, repeated until about min_seconds of CPU work."""
    import oracle
    import workloads
    from paper_1606_00094_amd import roofline
    oracle.build()
    problems = [(layer, workloads.make_layer_inputs(layer, N)) for layer in layers]
    flops, secs, passes = 0, 0.0, 0
    while passes < max_passes and secs < min_seconds:
        for layer, (x, f, b) in problems:
            t0 = time.perf_counter()
            oracle.conv_fwd(x, f, b, stride=layer.stride, pad=layer.pad, relu=True)
            secs += time.perf_counter() - t0
            flops += roofline.conv_flops(N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S,
                                         layer.stride, layer.pad)
        passes += 1
    return {"value": round(flops / secs / 1e9, 2), "unit": "GFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(secs, 2),
            "sample": "%d pass(es) over the %d benchmark layers at batch %d (%.1f GFLOP)"
                      % (passes, len(layers), N, flops / 1e9)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--spinup-ms", type=float, default=150.0,
                    help="untimed steps before the warm-up until the device has been busy this long")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--big-batch", type=int, default=128,
                    help="batch of the supplementary per-layer table (0: skip it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-layer-table", action="store_true")
    ap.add_argument("--no-stack", action="store_true",
                    help="skip the five-layer stacks and the matrix products (a profile of single layers)")
    ap.add_argument("--cpu-baseline-batch", type=int, default=32)
    ap.add_argument("--layers", default="", help="comma-separated layer names (default: all ten)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (--gpus %d refused)" % args.gpus)
        sys.exit(2)

    import torch
    import workloads
    from paper_1606_00094_amd import binding, roofline
    global graph_time_us
    from paper_1606_00094_amd.timing import graph_time_us
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the library has no CPU path")
        sys.exit(1)
    binding.lib()
    torch.cuda.set_device(0)

    layers = workloads.CONFIG_FIRST + workloads.CONFIG_MIDDLE + workloads.CONFIG_POINTWISE
    if args.layers:
        layers = [workloads.BY_NAME[n] for n in args.layers.split(",")]
    if args.calibration_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    probs = [LayerProblem(l, args.batch) for l in layers]
    total_flops = sum(p.flops for p in probs)

    def step():
        for p in probs:
            p.launch()

    # The card idles at a low clock and needs tens of milliseconds of load to reach its working
    # clock: untimed steps until it has been busy for --spinup-ms, then the W warm-up steps.
    spinup_steps = 0
    t_spin = time.perf_counter()
    while (time.perf_counter() - t_spin) * 1e3 < args.spinup_ms:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        spinup_steps += 10
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = max(e0.elapsed_time(e1) / args.steps, 0.0)
    # whole-job rate uses the host clock around the synchronised region
    value = total_flops / (wall_ms * 1e-3) / 1e9
    log("step: %.3f ms wall, %.3f ms by events, %.1f GFLOP/s" % (wall_ms, ms_per_step, value))

    # ---- per-layer table
    table = []
    per_layer_ms = {}
    for p in probs:
        ms = graph_time_us(p.launch, launches=10) * 1e-3
        per_layer_ms[p.layer.name] = ms
        table.append(layer_row(p, ms, "warm"))
    if not args.no_layer_table:
        for l in [workloads.TOY] + layers:
            p1 = LayerProblem(l, 1)
            table.append(layer_row(p1, graph_time_us(p1.launch, launches=20) * 1e-3, "warm"))
            # cold: rotate through enough distinct tensor sets that nothing stays in cache
            copies = int(min(192, max(2, (600 << 20) // max(1, p1.bytes))))
            pc = LayerProblem(l, 1, copies=copies)
            table.append(layer_row(pc, graph_time_us(pc.launch, launches=copies, replays=3) * 1e-3,
                                   "cold"))
            del p1, pc
    for row in table:
        log(json.dumps(row))

    # ---- the same layers at a production-size batch (context beside the metric's batch 1
    # and 32; not part of `value`): more rounds of workgroups, less lost to the last one
    table_big = []
    if not args.no_layer_table and args.big_batch > 0:
        for l in layers:
            pb = LayerProblem(l, args.big_batch)
            table_big.append(layer_row(pb, graph_time_us(pb.launch, launches=5, replays=3) * 1e-3, "warm"))
            del pb
    for row in table_big:
        log(json.dumps(row))

    # ---- the same layers with half-precision storage (fp32 arithmetic): same variants,
    # half the bytes; context beside the fp32 table, not part of `value`
    table_f16 = []
    if not args.no_layer_table:
        for l in layers:
            for N in (args.batch, 1):
                ph = LayerProblem(l, N, half=True)
                row = layer_row(ph, graph_time_us(ph.launch, launches=10 if N > 1 else 20) * 1e-3, "warm")
                row["storage"] = "f16"
                if ph.prepack():       # the same layer with the filters re-laid once, not per call
                    row["us_prepacked"] = round(graph_time_us(ph.launch, launches=10), 2)
                c8_tile = ph.to_c8()   # ... and with the activations octet-interleaved as well
                if c8_tile:
                    row["us_c8"] = round(graph_time_us(ph.launch, launches=10 if N > 1 else 20), 2)
                    row["variant_c8"] = c8_tile
                table_f16.append(row)
                del ph
    for row in table_f16:
        log(json.dumps(row))

    # ---- roofline of the dominant kernel (largest share of the step)
    dom = max(probs, key=lambda p: per_layer_ms[p.layer.name])
    dom_ms = graph_time_us(dom.launch, launches=20) * 1e-3
    achieved = dom.flops / (dom_ms * 1e-3) / 1e12
    roof = {"bound": "mfma", "achieved": round(achieved, 2), "peak": roofline.PEAK_FP32_MFMA_TFLOPS,
            "unit": "TFLOP/s", "frac": round(achieved / roofline.PEAK_FP32_MFMA_TFLOPS, 4),
            "traffic": recorded_traffic(dom), "kernel": binding.conv_variant_name(dom.variant),
            "layer": dom.layer.name, "N": dom.N, "us_per_launch": round(dom_ms * 1e3, 2)}

    stack = [] if args.no_layer_table or args.no_stack else [run_stack(n, 20) for n in (1, 5, 20, 32)]
    for row in stack:
        log(json.dumps({"stack": row}))

    stack16 = [] if args.no_layer_table or args.no_stack else [run_stack_f16(n, 20) for n in (1, 5, 20, 32)]
    for row in stack16:
        log(json.dumps({"stack_f16": row}))

    sgemm = [] if args.no_layer_table or args.no_stack else [run_sgemm(n) for n in workloads.SGEMM_SIZES]
    for row in sgemm:
        log(json.dumps({"sgemm": row}))

    # ---- one isolated call, host clock: from the call until the host sees it complete
    # (library host code + launch + kernel(s) + completion signal), median of 30
    single = []
    if not args.no_layer_table:
        for l, N in ((workloads.TOY, 1), (workloads.CONV3, 1), (workloads.CONV2, args.batch)):
            ps = LayerProblem(l, N)
            for _ in range(3):
                ps.launch()
            times = []
            for _ in range(30):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ps.launch()
                torch.cuda.synchronize()
                times.append(time.perf_counter() - t0)
            times.sort()
            single.append({"layer": l.name, "N": N, "wall_us": round(times[len(times) // 2] * 1e6, 1),
                           "min_us": round(times[0] * 1e6, 1)})
            del ps
    for row in single:
        log(json.dumps({"single_launch": row}))

    # what the machine at hand sustains, beside the published peaks: a register-only MFMA
    # loop through the library, and a large device-to-device copy
    measured = None
    if not args.no_layer_table:
        buf = torch.empty(512 * 256, dtype=torch.float32, device="cuda:0")
        flops = binding.bconv_debug_mfma_loop(buf, 512, 500)
        us = graph_time_us(lambda: binding.bconv_debug_mfma_loop(buf, 512, 500), launches=4)
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        cus = graph_time_us(lambda: dst.copy_(src), launches=4)
        measured = {"mfma_loop_tflops": round(flops / us / 1e6, 1),
                    "copy_256mib_gbps_read_plus_write": round(2 * src.numel() * 4 / cus / 1e3, 1)}
        del src, dst
        log(json.dumps({"measured_peaks": measured}))

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(layers, args.cpu_baseline_batch)
        log(json.dumps(cpu))

    # ---- the batch-1 half of the metric in compact form.  The layers whose roofline minimum
    # is a fraction of a microsecond (the weight- or activation-streaming ones) are quoted
    # cold (no tensor still in cache) against two denominators: the HBM roof (algorithmic
    # bytes / time / 8 TB/s) and the shortest time any single kernel takes in a replayed graph
    # on this machine (the toy layer, 0.9 MFLOP: launch gap + one prologue + one epilogue).
    by_key = {(r["layer"], r["N"], r["mode"]): r for r in table}
    floor_row = by_key.get((workloads.TOY.name, 1, "warm"))
    floor_us = floor_row["us"] if floor_row else None
    streaming = [l.name for l in (workloads.CONV3, workloads.CONV4, workloads.CONV5, workloads.PW_A,
                                  workloads.PW_B, workloads.PW_C)]

    def batch1_entry(name):
        r = by_key[(name, 1, "cold")]
        p1 = LayerProblem(workloads.BY_NAME[name], 1)
        e = {"layer": name, "us": r["us"], "gbps": r["gbps"], "frac": r["frac_hbm"],
             "frac_of_kernel_floor": round(floor_us / r["us"], 3) if floor_us else None,
             "kernels": 1 if r["variant"].endswith("/s1") or r["variant"] == "direct" else 2, "traffic": recorded_traffic(p1)}
        del p1
        return e

    roof1 = None
    rows1 = [batch1_entry(n) for n in streaming if (n, 1, "cold") in by_key]
    if rows1:
        roof1 = {"bound": "hbm", "peak": roofline.PEAK_HBM_GBPS, "unit": "GB/s", "mode": "cold",
                 "kernel_floor_us": floor_us,
                 "worst": min(rows1, key=lambda e: e["frac"]), "best": max(rows1, key=lambda e: e["frac"])}
    # per layer: [us at batch 32, fraction of the fp32 MFMA peak, us at batch 1 cold, GB/s,
    # fraction of the HBM peak, kernel floor / us]
    per_layer = {}
    for l in layers:
        r32 = by_key.get((l.name, args.batch, "warm"))
        r1 = by_key.get((l.name, 1, "cold"))
        per_layer[l.name] = [r32["us"], r32["frac_mfma"]] + (
            [r1["us"], r1["gbps"], r1["frac_hbm"], round(floor_us / r1["us"], 3)] if r1 and floor_us else [])
    # half-precision storage (context, not part of `value`): time per layer at the benchmark batch
    # and the largest one against the fp16 matrix peak (its kernel multiplies on those cores)
    per_layer_f16, roof16 = {}, None
    rows16 = [r for r in table_f16 if r["N"] == args.batch]
    for r in rows16:
        per_layer_f16[r["layer"]] = [r["us"], round(r["gflops"] / 1e3, 1), r.get("us_prepacked"), r.get("us_c8")]
    # ... and at batch 1 (per-call NCHW path, and C8 activations with packed filters)
    per_layer_f16_b1 = {r["layer"]: [r["us"], r.get("us_c8")] for r in table_f16 if r["N"] == 1}
    if rows16:
        # the largest layer of the native half-precision configuration (C8 activations, packed
        # filters) against the fp16 matrix peak; NCHW per-call figures where no such tile applies
        on_cores = [r for r in rows16 if r.get("us_c8")]
        if on_cores:
            big = max(on_cores, key=lambda r: r["us_c8"])
            us16, kern16, lay16 = big["us_c8"], big["variant_c8"], "C8 in/out, filters packed"
        else:
            big = max(rows16, key=lambda r: r["us"])
            us16, kern16, lay16 = big["us"], big["variant"], "NCHW"
        tf16 = big["gflops"] * big["us"] / us16 / 1e3
        roof16 = {"bound": "mfma", "dtype": "f16 storage, fp32 accumulate", "achieved": round(tf16, 1),
                  "peak": roofline.PEAK_FP16_MFMA_TFLOPS, "unit": "TFLOP/s",
                  "frac": round(tf16 / roofline.PEAK_FP16_MFMA_TFLOPS, 4), "layout": lay16,
                  "layer": big["layer"], "N": big["N"], "kernel": kern16, "us_per_launch": us16}
    full = {"layers": table, "layers_batch_%d" % args.big_batch: table_big, "layers_f16_storage": table_f16,
            "stack": stack, "stack_f16": stack16, "sgemm": sgemm, "single_launch": single, "measured_peaks": measured}
    log(json.dumps({"tables": full}))

    # The one line on stdout: the contract's fields first, the compact per-layer summary, then
    # the baseline and the two roofline objects last (a reader that keeps only the end of the
    # line still gets them).  The full tables went to stderr above.
    print(json.dumps({
        "metric": METRIC, "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "spinup_steps": spinup_steps,
        "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": ("one pass over the 10 benchmark conv layers (first layer, 4 middle, "
                                "3 pointwise, 2 reduce) at batch %d, bias + ReLU fused" % args.batch)
                               if not args.layers else
                               "layers %s at batch %d, bias + ReLU fused" % (args.layers, args.batch),
                   "batch": args.batch, "gflop_per_step": round(total_flops / 1e9, 2)},
        "per_layer_columns": ["us_b%d" % args.batch, "frac_mfma_b%d" % args.batch, "us_b1_cold", "gbps_b1",
                              "frac_hbm_b1", "kernel_floor_over_us_b1"],
        "per_layer": per_layer,
        "stack_ms": {str(r["N"]): r["ms"] for r in stack},
        "stack_f16_ms": {str(r["N"]): r["ms"] for r in stack16},
        "measured_peaks": measured,
        "per_layer_f16_columns": ["us_b%d" % args.batch, "tflops", "us_filters_prepacked", "us_c8_activations"], "per_layer_f16": per_layer_f16,
        "per_layer_f16_b1_columns": ["us_b1", "us_b1_c8_activations"], "per_layer_f16_b1": per_layer_f16_b1,
        "roofline_f16": roof16,
        "cpu_baseline": cpu, "roofline_batch1": roof1, "roofline": roof,
    }), flush=True)


if __name__ == "__main__":
    main()
