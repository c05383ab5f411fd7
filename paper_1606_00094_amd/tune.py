"""Offline tuning sweep: times every applicable variant (tile shape x reduction
split) on each benchmark layer shape and batch size and writes the per-shape
selection table the library compiles in.

This plays the role the paper gives to its per-operation choice of variant and
blocking constants (Section V: blocking chosen by heuristics and manual tuning,
automated tuning named as future work; Section VI: variant per convolution).

    python -m paper_1606_00094_amd.tune --out tune.json --table selection_table.inc

Each candidate is timed as a HIP graph of back-to-back launches (no host launch
overhead in the figure) and its output is compared with the direct kernel's.
"""
import argparse
import re
import json
import sys

import torch

import workloads
from paper_1606_00094_amd import binding, roofline
from paper_1606_00094_amd.timing import graph_time_us


def _split_of(name):
    return int(name.rsplit("/s", 1)[1])


def sweep_layer(layer, N, check=True, max_split=32, only=None):
    """Times every applicable variant (with `only`, a compiled regular expression: the
    variants whose name matches it, plus the one the library selects today)."""
    dev = torch.device("cuda:0")
    x, f, b = workloads.make_layer_inputs(layer, N)
    xd, fd, bd = (None if a is None else torch.from_numpy(a).to(dev) for a in (x, f, b))
    dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    P, Q = binding.conv_out_dims(layer.H, layer.W, layer.R, layer.S, layer.stride, layer.pad)
    out = torch.empty((N, layer.K, P, Q), dtype=torch.float32, device=dev)
    ref = torch.empty_like(out)
    binding.conv_fwd_ex(xd, fd, bd, ref, layer.stride, layer.pad, True, variant=0)
    flops = roofline.conv_flops(*dims)
    rows = []
    selected = binding.conv_selected_variant(*dims)
    for v in range(1, binding.conv_num_variants()):
        if not binding.conv_variant_applicable(*dims, v):
            continue
        if v != selected and _split_of(binding.conv_variant_name(v)) > max_split:
            continue
        if only is not None and v != selected and not only.search(binding.conv_variant_name(v)):
            continue
        need = binding.conv_fwd_workspace_bytes(*dims, v)
        ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)

        def run():
            binding.conv_fwd_ex(xd, fd, bd, out, layer.stride, layer.pad, True, workspace=ws,
                                variant=v)
        us = graph_time_us(run, best=True)
        ok = True
        if check:
            err = (out - ref).abs()
            ok = bool((err <= torch.clamp(ref.abs() * 1e-4, min=1e-5) * 2).all())
        rows.append({"variant": binding.conv_variant_name(v), "us": round(us, 2),
                     "tflops": round(flops / us / 1e6, 2), "ok": ok})
        del ws
    rows.sort(key=lambda r: r["us"])
    return rows


def sweep_layer_pooled(layer, N, max_split=32, ksz=3, pstride=2):
    """The same sweep through the convolution + pooling call: a variant that splits the
    reduction carries the pooling in its reduction kernel, one without pays a pooling
    kernel, so the ranking differs from the convolution's own."""
    dev = torch.device("cuda:0")
    x, f, b = workloads.make_layer_inputs(layer, N)
    xd, fd, bd = (torch.from_numpy(a).to(dev) for a in (x, f, b))
    dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    P, Q = binding.conv_out_dims(layer.H, layer.W, layer.R, layer.S, layer.stride, layer.pad)
    conv = torch.empty((N, layer.K, P, Q), dtype=torch.float32, device=dev)
    binding.conv_fwd_ex(xd, fd, bd, conv, layer.stride, layer.pad, True, variant=0)
    ref = torch.empty((N, layer.K) + binding.conv_out_dims(P, Q, ksz, ksz, pstride, 0),
                      dtype=torch.float32, device=dev)
    binding.maxpool_fwd(conv, ref, ksz, pstride)
    out = torch.empty_like(ref)
    rows = []
    for v in range(1, binding.conv_num_variants()):
        if not binding.conv_variant_applicable(*dims, v):
            continue
        if _split_of(binding.conv_variant_name(v)) > max_split:
            continue
        need = binding.conv_pool_fwd_workspace_bytes(*dims, v)
        ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)

        def run():
            binding.conv_pool_fwd_ex(xd, fd, bd, out, layer.stride, layer.pad, True, ksz, pstride, ws,
                                     variant=v)
        us = graph_time_us(run, best=True)
        err = (out - ref).abs()
        ok = bool((err <= torch.clamp(ref.abs() * 1e-4, min=1e-5) * 2).all())
        rows.append({"variant": binding.conv_variant_name(v), "us": round(us, 2), "ok": ok})
        del ws
    rows.sort(key=lambda r: r["us"])
    return rows


def main_pooled(args, batches, names):
    """--pool: rows for pool_selection_table.inc, for the layers a 3x3 / step-2 pooling
    follows; a row is written only where the pooled best beats the convolution's own
    choice run through the same call by more than 2 %."""
    layers = [l for l in workloads.POOLED_LAYERS if not names or l.name in names]
    results, table = [], []
    for layer in layers:
        for N in batches:
            rows = sweep_layer_pooled(layer, N, max_split=args.max_split or (32 if N <= 2 else 12 if N <= 8 else 6))
            good = [r for r in rows if r["ok"]]
            dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
            own = binding.conv_variant_name(binding.conv_selected_variant(*dims))
            own_us = next((r["us"] for r in rows if r["variant"] == own), None)
            best = good[0] if good else None
            results.append({"layer": layer.name, "N": N, "best": best, "all": rows,
                            "conv_choice": own, "conv_choice_us": own_us})
            print("%-18s N=%-3d pooled best %-26s %8.2f us; convolution's choice %s %s"
                  % (layer.name, N, best["variant"] if best else "-", best["us"] if best else 0, own,
                     "%.2f us" % own_us if own_us else "-"), flush=True)
            if best and own_us and best["variant"] != own and best["us"] < 0.98 * own_us:
                tile, split = best["variant"].split("/s")
                table.append('{%d, %d, %d, %d, %d, %d, %d, %d, %d, "%s", %s},  // %s N=%d: %.1f us (convolution\'s choice %s: %.1f)'
                             % (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride,
                                layer.pad, tile, split, layer.name, N, best["us"], own, own_us))
    with open(args.out, "w") as fh:
        json.dump(results, fh, indent=1)
    with open(args.table, "w") as fh:
        fh.write("// Variant choices for convolution + 3x3 / step-2 max pooling in one call, written by the\n"
                 "// offline tuning sweep (paper_1606_00094_amd/tune.py --pool).  Only shapes whose best\n"
                 "// pooled variant differs from the convolution's own choice are listed.\n"
                 "// Row: {N, C, H, W, K, R, S, stride, pad, \"tile\", nsplit},\n")
        fh.write("\n".join(table) + ("\n" if table else ""))
    return 0


def sweep_layer_f16(layer, N):
    """Half-precision storage: every tile on the fp16 matrix cores that applies, against what the
    half-precision entry points would run without them (the fp32 table's choice, widening)."""
    dev = torch.device("cuda:0")
    x, f, b = workloads.make_layer_inputs(layer, N)
    xd, fd = torch.from_numpy(x).to(dev).half(), torch.from_numpy(f).to(dev).half()
    bd = None if b is None else torch.from_numpy(b).to(dev)
    dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    P, Q = binding.conv_out_dims(layer.H, layer.W, layer.R, layer.S, layer.stride, layer.pad)
    out = torch.empty((N, layer.K, P, Q), dtype=torch.float16, device=dev)
    ref = torch.empty_like(out)
    base = binding.conv_selected_variant(*dims)
    need = binding.conv_fwd_f16_workspace_bytes(*dims, base)
    ws0 = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)
    binding.conv_fwd_f16_ex(xd, fd, bd, ref, layer.stride, layer.pad, True, workspace=ws0, variant=base)
    flops = roofline.conv_flops(*dims)
    rows = []
    for v in [base] + [v for v in range(1, binding.conv_num_variants())
                       if binding.conv_variant_name(v).startswith("h16")]:
        if not binding.conv_fwd_f16_variant_applicable(*dims, v):
            continue
        need = binding.conv_fwd_f16_workspace_bytes(*dims, v)
        ws = torch.zeros(max(1, (need + 3) // 4), dtype=torch.float32, device=dev)

        def run():
            binding.conv_fwd_f16_ex(xd, fd, bd, out, layer.stride, layer.pad, True, workspace=ws, variant=v)
        us = graph_time_us(run, best=True)
        err = (out.float() - ref.float()).abs()
        ok = bool((err <= torch.clamp(ref.float().abs() * 2.0 ** -9, min=1e-5)).all())
        rows.append({"variant": binding.conv_variant_name(v), "us": round(us, 2),
                     "tflops": round(flops / us / 1e6, 2), "ok": ok, "base": v == base})
        del ws
    rows.sort(key=lambda r: r["us"])
    return rows


def main_f16(args, batches, names):
    """--f16: rows for f16_selection_table.inc where an fp16-matrix-core tile beats the
    half-precision path's fallback by more than 2 %."""
    layers = [l for l in workloads.ALL_LAYERS + workloads.EXTRA_LAYERS if (l.name in names if names else l in workloads.ALL_LAYERS)]
    results, table = [], []
    for layer in layers:
        for N in batches:
            rows = sweep_layer_f16(layer, N)
            good = [r for r in rows if r["ok"]]
            base_us = next((r["us"] for r in rows if r["base"]), None)
            best = good[0] if good else None
            results.append({"layer": layer.name, "N": N, "best": best, "all": rows})
            print("%-18s N=%-3d f16 best %-22s %8.2f us %7.1f TFLOP/s; widening path %s (%d candidates, %d failed)"
                  % (layer.name, N, best["variant"] if best else "-", best["us"] if best else 0,
                     best["tflops"] if best else 0, "%.2f us" % base_us if base_us else "-", len(rows),
                     len(rows) - len(good)), flush=True)
            if best and not best["base"] and base_us and best["us"] < 0.98 * base_us:
                tile, split = best["variant"].split("/s")
                table.append('{%d, %d, %d, %d, %d, %d, %d, %d, %d, "%s", %s},  // %s N=%d: %.1f us (widening path %.1f)'
                             % (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride,
                                layer.pad, tile, split, layer.name, N, best["us"], base_us))
    with open(args.out, "w") as fh:
        json.dump(results, fh, indent=1)
    with open(args.table, "w") as fh:
        fh.write("// Variant choices of the half-precision entry points, written by the offline tuning sweep\n"
                 "// (paper_1606_00094_amd/tune.py --f16): rows where a tile on the fp16 matrix cores is the measured best.\n"
                 "// Row: {N, C, H, W, K, R, S, stride, pad, \"tile\", nsplit},\n")
        fh.write("\n".join(table) + ("\n" if table else ""))
    return 0


def sweep_layer_f16_c8(layer, N):
    """Octet-interleaved activations, filters packed beforehand: every fp16-matrix-core tile that
    applies, timed through conv_fwd_f16_packed_layout_ex (C8 out where K allows it) and checked
    against the NCHW path of the same tile, which it must equal bit for bit."""
    dev = torch.device("cuda:0")
    x, f, b = workloads.make_layer_inputs(layer, N)
    xd, fd = torch.from_numpy(x).to(dev).half(), torch.from_numpy(f).to(dev).half()
    bd = None if b is None else torch.from_numpy(b).to(dev)
    C, K, H, W = layer.C, layer.K, layer.H, layer.W
    dims = (N, C, H, W, K, layer.R, layer.S, layer.stride, layer.pad)
    P, Q = binding.conv_out_dims(H, W, layer.R, layer.S, layer.stride, layer.pad)
    rows = []
    if C % 8:
        return rows
    c8_out = K % 8 == 0
    ref = torch.empty((N, K, P, Q), dtype=torch.float16, device=dev)
    back = torch.empty_like(ref)
    x8 = torch.empty((N, C // 8, H, W, 8), dtype=torch.float16, device=dev)
    o8 = torch.empty((N, K // 8, P, Q, 8), dtype=torch.float16, device=dev) if c8_out else back
    binding.f16_layout_convert(xd, binding.LAYOUT_NCHW, x8, binding.LAYOUT_C8, (N, C, H, W))
    olay = binding.LAYOUT_C8 if c8_out else binding.LAYOUT_NCHW
    flops = roofline.conv_flops(*dims)
    for v in range(1, binding.conv_num_variants()):
        if not binding.conv_variant_name(v).startswith("h16"):
            continue
        nbytes = binding.conv_f16_packed_filter_bytes(*dims, v)
        if nbytes == 0:
            continue
        packed = torch.empty(nbytes // 2, dtype=torch.float16, device=dev)
        binding.conv_f16_pack_filters(fd, packed, N, H, W, layer.stride, layer.pad, variant=v)
        binding.conv_fwd_f16_packed_ex(xd, packed, fd.shape, bd, ref, layer.stride, layer.pad, True, variant=v)

        def run():
            binding.conv_fwd_f16_packed_layout_ex(x8, binding.LAYOUT_C8, packed, fd.shape, bd, o8, olay,
                                                  (N, C, H, W), layer.stride, layer.pad, True, variant=v)
        us = graph_time_us(run, best=True)
        if c8_out:
            binding.f16_layout_convert(o8, binding.LAYOUT_C8, back, binding.LAYOUT_NCHW, (N, K, P, Q))
        rows.append({"variant": binding.conv_variant_name(v), "us": round(us, 2),
                     "tflops": round(flops / us / 1e6, 2), "ok": bool(torch.equal(back, ref))})
        del packed
    rows.sort(key=lambda r: r["us"])
    return rows


def main_f16_c8(args, batches, names):
    """--f16-c8: rows for f16_c8_selection_table.inc, the best tile per (layer, batch)."""
    layers = [l for l in workloads.ALL_LAYERS + workloads.EXTRA_LAYERS if (l.name in names if names else l in workloads.ALL_LAYERS)]
    results, table = [], []
    for layer in layers:
        for N in batches:
            rows = sweep_layer_f16_c8(layer, N)
            good = [r for r in rows if r["ok"]]
            best = good[0] if good else None
            results.append({"layer": layer.name, "N": N, "best": best, "all": rows})
            print("%-18s N=%-3d C8 best %-22s %8.2f us %7.1f TFLOP/s (%d candidates, %d failed)"
                  % (layer.name, N, best["variant"] if best else "-", best["us"] if best else 0,
                     best["tflops"] if best else 0, len(rows), len(rows) - len(good)), flush=True)
            if best:
                tile, split = best["variant"].split("/s")
                table.append('{%d, %d, %d, %d, %d, %d, %d, %d, %d, "%s", %s},  // %s N=%d: %.1f us'
                             % (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride,
                                layer.pad, tile, split, layer.name, N, best["us"]))
    with open(args.out, "w") as fh:
        json.dump(results, fh, indent=1)
    with open(args.table, "w") as fh:
        fh.write("// Tile choices for half-precision layers on octet-interleaved (C8) activations, written by the\n"
                 "// offline tuning sweep (paper_1606_00094_amd/tune.py --f16-c8).\n"
                 "// Row: {N, C, H, W, K, R, S, stride, pad, \"tile\", nsplit},\n")
        fh.write("\n".join(table) + ("\n" if table else ""))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="tune.json")
    ap.add_argument("--table", default="selection_table.inc")
    ap.add_argument("--batches", default="1,5,20,32")
    ap.add_argument("--layers", default="")
    ap.add_argument("--extra", action="store_true",
                    help="also sweep the shapes kept out of the table (heuristic quality check)")
    ap.add_argument("--sgemm", action="store_true", help="also sweep the square matrix products")
    ap.add_argument("--pool", action="store_true",
                    help="sweep the convolution + pooling call instead (rows for pool_selection_table.inc)")
    ap.add_argument("--f16", action="store_true",
                    help="sweep the half-precision entry points' fp16-matrix-core tiles (rows for f16_selection_table.inc)")
    ap.add_argument("--f16-c8", action="store_true",
                    help="sweep those tiles on octet-interleaved activations (rows for f16_c8_selection_table.inc)")
    ap.add_argument("--max-split", type=int, default=0, help="largest reduction split to try (0: by batch)")
    ap.add_argument("--only", default="",
                    help="regular expression: sweep only the variants whose name matches, against "
                         "the variant selected today (a partial re-sweep after adding tiles)")
    args = ap.parse_args()
    batches = [int(t) for t in args.batches.split(",")]
    names = [t for t in args.layers.split(",") if t]
    if args.pool:
        return main_pooled(args, batches, names)
    if args.f16_c8:
        return main_f16_c8(args, batches, names)
    if args.f16:
        return main_f16(args, batches, names)
    # the square matrix products (batch 1 only) are swept when named, or with --sgemm
    pool = workloads.ALL_LAYERS + (workloads.SGEMM_LAYERS if args.sgemm or names else []) + \
        (workloads.EXTRA_LAYERS if args.extra or names else [])
    layers = [l for l in pool if not names or l.name in names]
    results, table = [], []
    for layer in layers:
        for N in (batches if not layer.name.startswith("sgemm_") else [1]):
            # large batches have enough tiles; deep reduction splits only cost traffic there
            big = layer.name.startswith("sgemm_") and layer.C >= 768
            rows = sweep_layer(layer, N, max_split=args.max_split or (4 if big else 32 if N <= 2 else 12 if N <= 8 else 6),
                               only=re.compile(args.only) if args.only else None)
            good = [r for r in rows if r["ok"]]
            best = good[0] if good else None
            # what the library would run for this shape (table row, else the heuristic)
            dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
            chosen = binding.conv_variant_name(binding.conv_selected_variant(*dims))
            chosen_us = next((r["us"] for r in rows if r["variant"] == chosen), None)
            results.append({"layer": layer.name, "N": N, "best": best, "all": rows,
                            "selected": chosen, "selected_us": chosen_us})
            print("%-18s N=%-3d best %-24s %9.2f us %7.2f TFLOP/s  (%d candidates, %d failed check)"
                  "  selected %s %s"
                  % (layer.name, N, best["variant"] if best else "-", best["us"] if best else 0,
                     best["tflops"] if best else 0, len(rows), len(rows) - len(good), chosen,
                     "%.2f us (x%.2f)" % (chosen_us, chosen_us / best["us"]) if chosen_us and best else "-"),
                  flush=True)
            if best:
                tile, split = best["variant"].split("/s")
                table.append('{%d, %d, %d, %d, %d, %d, %d, %d, %d, "%s", %s},  // %s N=%d: %.1f us'
                             % (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride,
                                layer.pad, tile, split, layer.name, N, best["us"]))
    with open(args.out, "w") as fh:
        json.dump(results, fh, indent=1)
    with open(args.table, "w") as fh:
        fh.write("// Per-shape variant choices, written by the offline tuning sweep\n"
                 "// (paper_1606_00094_amd/tune.py).  Row: {N, C, H, W, K, R, S, stride, pad, \"tile\", nsplit},\n")
        fh.write("\n".join(table) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
