#!/usr/bin/env python3
"""Benchmark of the channel-gated convolution layer on one MI355X.

Workload: the seven ImageNet-shaped ResNet-18 3x3 gated convolutions (batch 64, bf16, NHWC,
G = 4; four stride-1 and three stride-2 layers), seeded synthetic inputs with spatially
clustered gate maps at about 30 % firing.  One *step* is one forward pass of the whole gated
layer (base path, gate, conditional path, epilogue, decision bitmap) over all seven layers,
each on its own HBM-resident input.

Prints ONE JSON line: effective TOP/s (dense-equivalent operations / time, i.e. skipped work
counted as done), per-layer microseconds beside the same-shape dense MFMA convolution from
the same library, the roofline of the dominant kernel and the CPU oracle timed on the host.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_INT8_TOPS = 5000.0       # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--rho", type=float, default=0.30)
    ap.add_argument("--kind", default="coherent", choices=["coherent", "literal", "iid"])
    ap.add_argument("--no-dense", action="store_true", help="skip the dense comparator (for kernel profiles)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--variant", default="auto", choices=["auto", "blockskip", "compact", "rows"],
                    help="kernel family (auto = what the library picks)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "int8"],
                    help="bf16 (the headline workload) or int8 (int8 activations/weights, int32 sums, int8 requantised output)")
    ap.add_argument("--fused-epilogue", action="store_true",
                    help="scale/shift by decision + residual add + ReLU in the layer epilogue (bf16) instead of ReLU alone")
    ap.add_argument("--grouped", action="store_true",
                    help="channel grouping (output group i takes input group i as its base path) instead of the "
                         "default fixed base channels")
    ap.add_argument("--tau-c", type=float, default=0.0,
                    help="channel-wise gate: an image's output channel keeps its conditional path only if at "
                         "least this fraction of its activations fired (0 = off)")
    ap.add_argument("--layers", default="", help="comma-separated layer names to restrict the workload")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards over the batch "
              "with no exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1805_12549_amd import binding as B
    from paper_1805_12549_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    variant = {"auto": B.CG_VARIANT_AUTO, "tile": B.CG_VARIANT_TILE,
               "rows": B.CG_VARIANT_MFMA_ROWS}[args.variant]
    shapes = W.imagenet_shapes(n=args.batch)
    if args.layers:
        keep = set(args.layers.split(","))
        shapes = [s for s in shapes if s.name in keep]
    layers = []
    t_gen = time.perf_counter()
    for li, s in enumerate(shapes):
        i8 = args.dtype == "int8"
        eb = 1 if i8 else 2
        tdt = torch.int8 if i8 else torch.bfloat16
        inp = W.make_inputs(s, W.seed_for(4 if i8 else 3, li), kind=args.kind, rho=args.rho, round_bf16=not i8,
                            grouped=args.grouped)
        if i8:
            inp_f = inp
            inp = W.quantize_int8(inp_f)
            gate = W.calibrate_gate_int8(inp, args.rho, sample_images=8)
            rq = W.requant_params(inp, np.random.default_rng(li))
        else:
            gate = W.calibrate_gate(inp, args.rho, sample_images=8)
        x_bytes = s.n * s.h * s.w * s.c_in * eb
        y_bytes = s.m * s.c_out * eb
        nset = max(2, int(np.ceil(600e6 / (x_bytes + y_bytes))))      # rotate past the 256 MB infinity cache
        x0 = torch.from_numpy(inp.x).to(dev).to(tdt)
        xs = [x0] + [x0.clone() for _ in range(nset - 1)]
        ys = [torch.empty((s.n, s.ho, s.wo, s.c_out), dtype=tdt, device=dev) for _ in range(nset)]
        bms = [torch.empty((s.m, s.c_out // 32), dtype=torch.int32, device=dev) for _ in range(nset)]
        wb = torch.from_numpy(inp.w_base).to(dev).to(tdt)
        wc = torch.from_numpy(inp.w_cond).to(dev).to(tdt)
        wfull = torch.cat([wb, wc], dim=-1).contiguous()
        common = dict(n_max=s.n, h=s.h, w=s.w, c_in=s.c_in, c_out=s.c_out, in_dtype=B.CG_I8 if i8 else B.CG_BF16,
                      out_dtype=B.CG_I8 if i8 else B.CG_BF16, stride=s.stride, pad=s.pad, epilogue=B.CG_EPI_RELU,
                      variant=variant)
        res = None
        if args.fused_epilogue and not i8:
            erng = np.random.default_rng(1000 + li)
            common.update(epilogue=B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL,
                          scale0=erng.uniform(0.5, 1.5, s.c_out), shift0=erng.normal(0, 0.1, s.c_out),
                          scale1=erng.uniform(0.5, 1.5, s.c_out), shift1=erng.normal(0, 0.1, s.c_out))
            res = torch.randn((s.n, s.ho, s.wo, s.c_out), device=dev).to(torch.bfloat16)
        if i8:
            common.update(rq)
            gkw = dict(gate_thr_i32=gate)
        else:
            gkw = dict(gate_mean=gate.mean, gate_var=gate.var, delta=gate.delta)
        gated = B.GatedConv(c_base=s.c_base, w_base=wb, w_cond=wc, groups=s.groups if args.grouped else 0,
                            tau_c=args.tau_c, **gkw, **common)
        dense = None if args.no_dense else B.GatedConv(c_base=s.c_in, w_base=wfull, w_cond=None, **common)
        layers.append(dict(shape=s, inp=inp, gate=gate, xs=xs, ys=ys, bms=bms, gated=gated, dense=dense, nset=nset, res=res,
                           rq=rq if i8 else None))
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    # ---- firing rate and executed-block fraction (one untimed call with counts on) ----------
    for L in layers:
        s = L["shape"]
        _, bm, cnt = L["gated"].forward(L["xs"][0], residual=L["res"], y=L["ys"][0], bitmap=L["bms"][0], counts=True)
        torch.cuda.synchronize()
        c = cnt.cpu().numpy().view(np.uint32)
        fired = int(c[0]) | (int(c[1]) << 32)
        L["rho"] = fired / (s.m * s.c_out)
        d = W.unpack_bitmap(bm[: min(s.m, 8 * s.ho * s.wo)].cpu().numpy().view(np.uint32), s.c_out)
        L["beta_16x16"] = W.occupancy(d, 16, 16)
        L["beta_px"] = W.occupancy(d, 1, s.c_out)

    def run_layer(L, which, k):
        i = k % L["nset"]
        L[which].forward(L["xs"][i], residual=L["res"], y=L["ys"][i], bitmap=L["bms"][i] if which == "gated" else False,
                         counts=False)

    # ---- per-layer timing with events on the launch stream ----------------------------------
    def time_layer(L, which, rounds=3):
        for k in range(12):
            run_layer(L, which, k)
        torch.cuda.synchronize()
        best = []
        for _ in range(rounds):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            calls = 48          # the same for every layer, so kernel-trace averages weigh layers equally
            e0.record()
            for k in range(calls):
                run_layer(L, which, k)
            e1.record()
            e1.synchronize()
            best.append(e0.elapsed_time(e1) * 1e3 / calls)
        return float(np.median(best))

    for L in layers:
        L["us_gated"] = time_layer(L, "gated")
        L["us_dense"] = None if args.no_dense else time_layer(L, "dense")

    # ---- the timed region: K steps of all layers ---------------------------------------------
    step_counter = [0]

    def one_step():
        k = step_counter[0]
        for L in layers:
            run_layer(L, "gated", k)
        step_counter[0] += 1

    stream = torch.cuda.current_stream()
    graph = None
    period = 1
    if not args.no_graph:
        # a graph replays fixed buffers: capture one period of the buffer rotation
        period = min(12, min(L["nset"] for L in layers))
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            one_step()                      # eager once on the capture stream
            torch.cuda.synchronize()
            step_counter[0] = 0
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(period):
                    one_step()
        torch.cuda.synchronize()

    def run_steps(n):
        if graph is None:
            for _ in range(n):
                one_step()
        else:
            for _ in range(n // period):
                graph.replay()

    steps = args.steps
    warm = args.warmup
    if graph is not None:
        steps = max(period, (steps // period) * period)
        warm = max(period, (warm // period) * period)
    run_steps(warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    dense_ops = sum(2 * L["shape"].dense_macs for L in layers)
    value = dense_ops / (ms_per_step * 1e-3) / 1e12

    # ---- roofline of the dominant kernel (the fused MFMA layer kernel) -------------------------
    alg_flops = 0.0
    alg_bytes = 0.0
    for L in layers:
        s = L["shape"]
        kp, kr = 9 * s.c_base, 9 * (s.c_in - s.c_base)
        alg_flops += 2.0 * s.m * s.c_out * (kp + L["rho"] * kr)
        ebl = 1 if args.dtype == "int8" else 2
        alg_bytes += (s.n * s.h * s.w * s.c_in + s.m * s.c_out + s.c_out * 9 * s.c_in) * ebl + s.m * s.c_out / 8
    t_kernel_us = sum(L["us_gated"] for L in layers)
    achieved = alg_flops / (t_kernel_us * 1e-6) / 1e12
    traffic = None     # measured HBM bytes per launch, from the committed counter summary
    tfile = ROOT / "profiles" / "hbm_traffic_gated_conv_rows_kernel_imagenet_resnet18_bf16_n64.txt"
    peak = PEAK_INT8_TOPS if args.dtype == "int8" else PEAK_BF16_TFLOPS
    if (tfile.exists() and args.batch == 64 and not args.layers and args.kind == "coherent" and not args.grouped
            and args.dtype == "bf16"
            and args.tau_c == 0.0
            and layers[0]["gated"].variant == B.CG_VARIANT_MFMA_ROWS):
        m = re.search(r"^bytes_per_launch:\s*(\d+)", tfile.read_text(), re.M)
        traffic = int(m.group(1)) if m else None
    roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=peak,
                    unit="TOP/s" if args.dtype == "int8" else "TFLOP/s",
                    frac=round(achieved / peak, 4), traffic=traffic,
                    kernel={B.CG_VARIANT_MFMA: "gated_conv_mfma_kernel",
                            B.CG_VARIANT_MFMA_COMPACT: "gated_conv_compact_kernel",
                            B.CG_VARIANT_MFMA_ROWS: "gated_conv_rows_kernel"}.get(
                                layers[-1]["gated"].variant, "naive_kernel") + "<%s>" % args.dtype, avg_launch_us=round(t_kernel_us / len(layers), 2),
                    algorithmic_gflop_per_launch=round(alg_flops / len(layers) / 1e9, 3),
                    hbm_gbs_algorithmic=round(alg_bytes / (t_kernel_us * 1e-6) / 1e9, 1),
                    hbm_frac=round(alg_bytes / (t_kernel_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4))

    # ---- CPU oracle on the host cores ----------------------------------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import cg_oracle as O
        t_cpu = 0.0
        ops_cpu = 0
        for L in layers:
            s, inp, gate = L["shape"], L["inp"], L["gate"]
            if args.dtype == "int8":
                tc = time.perf_counter()
                O.forward_int8(inp.x, inp.w_base, inp.w_cond, gate, stride=s.stride, pad=s.pad, out_i8=True,
                               epilogue=O.RELU, want_partials=False, groups=s.groups if args.grouped else 1,
                               tau_c=float(np.float32(args.tau_c)), **L["rq"])
                t_cpu += time.perf_counter() - tc
                ops_cpu += 2 * s.dense_macs
                continue
            x64 = inp.x.astype(np.float64)
            wb64, wc64 = inp.w_base.astype(np.float64), inp.w_cond.astype(np.float64)
            tc = time.perf_counter()
            O.forward_float(x64, wb64, wc64, stride=s.stride, pad=s.pad, gate_mean=gate.mean, gate_var=gate.var,
                            delta=gate.delta, epilogue=O.RELU, want_partials=False,
                            groups=s.groups if args.grouped else 1, tau_c=float(np.float32(args.tau_c)))
            t_cpu += time.perf_counter() - tc
            ops_cpu += 2 * s.dense_macs
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = dict(value=round(ops_cpu / t_cpu / 1e12, 5), unit="TOP/s", cores=cores, kind="oracle",
                   seconds=round(t_cpu, 2),
                   sample="one pass of the full workload (all layers, batch %d), %s, both branches evaluated"
                          % (args.batch, "int32 sums" if args.dtype == "int8" else "fp64"))

    per_layer = []
    for L in layers:
        s = L["shape"]
        row = dict(layer=s.name, us_gated=round(L["us_gated"], 2), rho=round(L["rho"], 4),
                   beta_16px_x_16ch=round(L["beta_16x16"], 3), beta_pixel=round(L["beta_px"], 3),
                   eff_tops_gated=round(2 * s.dense_macs / L["us_gated"] / 1e6, 1))
        if L["us_dense"] is not None:
            row.update(us_dense=round(L["us_dense"], 2), tops_dense=round(2 * s.dense_macs / L["us_dense"] / 1e6, 1),
                       speedup=round(L["us_dense"] / L["us_gated"], 3))
        per_layer.append(row)

    out = {
        "metric": "gated-conv effective TOP/s (dense-equivalent ops/time) over the ImageNet ResNet-18 3x3 layers; "
                  "per-layer us beside the dense MFMA conv in config.per_layer",
        "value": round(value, 2), "unit": "TOP/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "ImageNet-shaped ResNet-18 gated 3x3 convs (configs[2]): batch %d, %s NHWC, G=4, "
                               "%s gate maps, target firing %.2f%s; step = all %d layers" %
                               (args.batch, args.dtype, args.kind, args.rho,
                                (", channel grouping" if args.grouped else "") +
                                (", fused scale/shift + residual + ReLU epilogue" if args.fused_epilogue else "") +
                                (", channel-wise gate tau_c=%.2f" % args.tau_c if args.tau_c > 0 else ""), len(layers)),
                   "launch": "hip graph replay" if graph is not None else "eager",
                   "sum_us_gated": round(t_kernel_us, 2),
                   "sum_us_dense": None if args.no_dense else round(sum(L["us_dense"] for L in layers), 2),
                   "per_layer": per_layer},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
