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

`--sweep` instead walks the firing rate and the base fraction (rho in {0.1 .. 0.9} x 1/G in
{1/2, 1/4, 1/8}, clustered and unclustered maps) and reports, per layer, the firing rate at
which the gated layer stops beating the dense convolution.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from dataclasses import replace
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_INT8_TOPS = 5000.0       # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0
KERNEL_OF = {4: "gated_conv_rows_kernel", 5: "gated_conv_tile_kernel", 1: "naive_kernel"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--rho", type=float, default=0.30)
    ap.add_argument("--kind", default=None, choices=["coherent", "literal", "iid"],
                    help="gate maps: spatially clustered across channels (coherent, the default), the literal recipe "
                         "(zero-mean weights: unclustered across channels) or i.i.d. inputs; --sweep walks coherent and "
                         "literal unless one is named")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense comparator (for kernel profiles)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--warm", action="store_true",
                    help="two buffer sets per layer instead of a rotation past the 256 MB Infinity Cache (warm-cache regime)")
    ap.add_argument("--variant", default="auto", choices=["auto", "rows", "tile"],
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
    ap.add_argument("--sweep", action="store_true",
                    help="firing rate x base fraction sweep with the crossover firing rate per layer (no timed steps)")
    return ap.parse_args()


def graph_of(fn, calls):
    """Captures `calls` consecutive invocations fn(0), fn(1), ... into a HIP graph."""
    import torch
    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        fn(0)                                   # eager once on the capture stream
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for k in range(calls):
                fn(k)
    torch.cuda.synchronize()
    return g


def time_graph_us(g, calls, rounds=5):
    """Median microseconds per call of a graph of `calls` calls, from events on the replay stream."""
    import numpy as np
    import torch
    g.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        e1.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / calls)
    return float(np.median(ts))


class Layer:
    """One gated layer with its dense comparator and enough rotated buffers to defeat the caches."""

    def __init__(self, args, s, li, rho, kind, variant, want_dense=True):
        import numpy as np
        import torch
        from paper_1805_12549_amd import binding as B
        from paper_1805_12549_amd import workloads as W
        dev = torch.device("cuda:0")
        i8 = args.dtype == "int8"
        eb = 1 if i8 else 2
        tdt = torch.int8 if i8 else torch.bfloat16
        self.shape, self.rq = s, None
        inp = W.make_inputs(s, W.seed_for(4 if i8 else 3, li), kind=kind, rho=rho, round_bf16=not i8,
                            grouped=args.grouped)
        if i8:
            inp = W.quantize_int8(inp)
            self.gate = W.calibrate_gate_int8(inp, rho, sample_images=8)
            self.rq = W.requant_params(inp, np.random.default_rng(li))
        else:
            self.gate = W.calibrate_gate(inp, rho, sample_images=8)
        self.inp = inp
        x_bytes = s.n * s.h * s.w * s.c_in * eb
        y_bytes = s.m * s.c_out * eb
        self.nset = min(24, max(2, int(np.ceil(600e6 / (x_bytes + y_bytes)))))    # rotate past the 256 MB infinity cache
        if args.warm:
            self.nset = 2
        x0 = torch.from_numpy(inp.x).to(dev).to(tdt)
        self.xs = [x0] + [x0.clone() for _ in range(self.nset - 1)]
        self.ys = [torch.empty((s.n, s.ho, s.wo, s.c_out), dtype=tdt, device=dev) for _ in range(self.nset)]
        self.bms = [torch.empty((s.m, s.c_out // 32), dtype=torch.int32, device=dev) for _ in range(self.nset)]
        wb = torch.from_numpy(inp.w_base).to(dev).to(tdt)
        wc = torch.from_numpy(inp.w_cond).to(dev).to(tdt)
        common = dict(n_max=s.n, h=s.h, w=s.w, c_in=s.c_in, c_out=s.c_out, in_dtype=B.CG_I8 if i8 else B.CG_BF16,
                      out_dtype=B.CG_I8 if i8 else B.CG_BF16, stride=s.stride, pad=s.pad, epilogue=B.CG_EPI_RELU,
                      variant=variant)
        self.res = None
        if args.fused_epilogue and not i8:
            erng = np.random.default_rng(1000 + li)
            common.update(epilogue=B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL,
                          scale0=erng.uniform(0.5, 1.5, s.c_out), shift0=erng.normal(0, 0.1, s.c_out),
                          scale1=erng.uniform(0.5, 1.5, s.c_out), shift1=erng.normal(0, 0.1, s.c_out))
            self.res = torch.randn((s.n, s.ho, s.wo, s.c_out), device=dev).to(torch.bfloat16)
        if i8:
            common.update(self.rq)
            gkw = dict(gate_thr_i32=self.gate)
        else:
            gkw = dict(gate_mean=self.gate.mean, gate_var=self.gate.var, delta=self.gate.delta)
        self.gated = B.GatedConv(c_base=s.c_base, w_base=wb, w_cond=wc, groups=s.groups if args.grouped else 0,
                                 tau_c=args.tau_c, **gkw, **common)
        self.dense = None
        if want_dense:
            wfull = torch.cat([wb, wc], dim=-1).contiguous()
            self.dense = B.GatedConv(c_base=s.c_in, w_base=wfull, w_cond=None, **common)

    def run(self, which, k):
        i = k % self.nset
        layer = self.gated if which == "gated" else self.dense
        layer.forward(self.xs[i], residual=self.res, y=self.ys[i], bitmap=self.bms[i] if which == "gated" else False,
                      counts=False)

    def measure_firing(self):
        import numpy as np
        import torch
        from paper_1805_12549_amd import workloads as W
        s = self.shape
        _, bm, cnt = self.gated.forward(self.xs[0], residual=self.res, y=self.ys[0], bitmap=self.bms[0], counts=True)
        torch.cuda.synchronize()
        c = cnt.cpu().numpy().view(np.uint32)
        fired = int(c[0]) | (int(c[1]) << 32)
        self.rho = fired / (s.m * s.c_out)
        d = W.unpack_bitmap(bm[: min(s.m, 8 * s.ho * s.wo)].cpu().numpy().view(np.uint32), s.c_out)
        self.beta_16x16 = W.occupancy(d, 16, 16)
        self.beta_px64 = W.occupancy(d, 1, 64)          # the kernels' granule: one pixel x one 64-channel block
        self.beta_px = W.occupancy(d, 1, s.c_out)

    def time_us(self, which):
        calls = max(self.nset, 24)
        g = graph_of(lambda k: self.run(which, k), calls)
        return time_graph_us(g, calls)

    def close(self):
        self.gated.close()
        if self.dense is not None:
            self.dense.close()


def crossover(rhos, us_gated, us_dense):
    """Firing rate at which the gated layer's time reaches the dense layer's (linear between samples)."""
    if us_gated[0] >= us_dense:
        return "< %.2f (never faster)" % rhos[0]
    for i in range(1, len(rhos)):
        if us_gated[i] >= us_dense:
            t = (us_dense - us_gated[i - 1]) / (us_gated[i] - us_gated[i - 1])
            return round(rhos[i - 1] + t * (rhos[i] - rhos[i - 1]), 3)
    return "> %.2f (always faster)" % rhos[-1]


# how often each 3x3 shape occurs among the sixteen residual-block convolutions of ResNet-18
CONVS_OF_SHAPE = {"64@56": 4, "128@28": 3, "256@14": 3, "512@7": 3}


def run_sweep(args, shapes, variant):
    import torch
    rhos = [0.1, 0.3, 0.5, 0.7, 0.9]
    rows = []
    for kind in (("coherent", "literal") if args.kind is None else (args.kind,)):
        first_row = len(rows)
        for li, s0 in enumerate(shapes):
            for G in (2, 4, 8):
                s = replace(s0, groups=G)
                us_dense, us_g, rho_meas, beta = None, [], [], []
                for rho in rhos:
                    L = Layer(args, s, li, rho, kind, variant, want_dense=us_dense is None)
                    L.measure_firing()
                    if us_dense is None:
                        us_dense = L.time_us("dense")
                    us_g.append(L.time_us("gated"))
                    rho_meas.append(round(L.rho, 3))
                    beta.append(round(L.beta_px64, 3))
                    kname = KERNEL_OF.get(L.gated.variant, "?")
                    L.close()
                    del L
                    torch.cuda.empty_cache()
                rows.append(dict(layer=s.name, maps=kind, base_fraction="1/%d" % G, kernel=kname, rho_target=rhos,
                                 rho=rho_meas, beta_pixel_x_64ch=beta, us_gated=[round(v, 2) for v in us_g],
                                 us_dense=round(us_dense, 2), crossover_rho=crossover(rho_meas, us_g, us_dense)))
                print("sweep %-9s %-13s 1/G=1/%d dense %6.2f us  gated %s  crossover %s" %
                      (kind, s.name, G, us_dense, " ".join("%6.2f" % v for v in us_g), rows[-1]["crossover_rho"]),
                      file=sys.stderr, flush=True)
        # the sixteen gated convolutions of the network together, per base fraction
        for G in (2, 4, 8):
            mine = [r for r in rows[first_row:] if r["base_fraction"] == "1/%d" % G and r["layer"] != "network"]
            if len(mine) != len(shapes) or len(shapes) != 7:
                continue
            mult = [CONVS_OF_SHAPE.get(r["layer"], 1) for r in mine]
            sum_g = [sum(m * r["us_gated"][i] for m, r in zip(mult, mine)) for i in range(len(rhos))]
            sum_d = sum(m * r["us_dense"] for m, r in zip(mult, mine))
            wsum = float(sum(m * s.m * s.c_out for m, s in zip(mult, shapes)))
            rho_net = [round(sum(m * r["rho"][i] * s.m * s.c_out for m, r, s in zip(mult, mine, shapes)) / wsum, 3)
                       for i in range(len(rhos))]
            rows.append(dict(layer="network", maps=kind, base_fraction="1/%d" % G,
                             what="sum over the 16 residual-block 3x3 convolutions of ResNet-18 (shape multiplicities "
                                  "4/3/3/3/1/1/1), each on its own input", rho_target=rhos, rho=rho_net,
                             us_gated=[round(v, 1) for v in sum_g], us_dense=round(sum_d, 1),
                             crossover_rho=crossover(rho_net, sum_g, sum_d)))
            print("sweep %-9s %-13s 1/G=1/%d dense %6.1f us  gated %s  crossover %s" %
                  (kind, "16 convs", G, sum_d, " ".join("%6.1f" % v for v in sum_g), rows[-1]["crossover_rho"]),
                  file=sys.stderr, flush=True)
    return rows


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
    torch.cuda.set_device(0)

    variant = {"auto": B.CG_VARIANT_AUTO, "tile": B.CG_VARIANT_TILE, "rows": B.CG_VARIANT_MFMA_ROWS}[args.variant]
    shapes = W.imagenet_shapes(n=args.batch)
    if args.layers:
        keep = set(args.layers.split(","))
        shapes = [s for s in shapes if s.name in keep]

    if args.sweep:
        rows = run_sweep(args, shapes, variant)
        args.kind = args.kind or "coherent + literal"
        print(json.dumps({"metric": "crossover firing rate of the gated layer against the dense convolution",
                          "n_gpus": 1, "dtype": args.dtype, "data": "synthetic",
                          "config": {"workload": "ImageNet-shaped ResNet-18 3x3 layers, batch %d, %s, %s; firing rate x "
                                                 "base fraction sweep, clustered (coherent) and unclustered (literal) maps"
                                                 % (args.batch, args.dtype, "scale/shift by decision + residual + ReLU"
                                                    if args.fused_epilogue else "ReLU epilogue"),
                                     "cache": "warm" if args.warm else "cold (buffers rotated past the Infinity Cache)",
                                     "sweep": rows}}), flush=True)
        return

    args.kind = args.kind or "coherent"
    layers = [Layer(args, s, li, args.rho, args.kind, variant, want_dense=not args.no_dense)
              for li, s in enumerate(shapes)]
    torch.cuda.synchronize()
    for L in layers:
        L.measure_firing()

    # ---- per-layer time: each layer's calls captured in a graph of its own, HIP events on the replay stream
    for L in layers:
        L.us_gated = L.time_us("gated")
        L.us_dense = None if args.no_dense else L.time_us("dense")

    # ---- the timed region: exactly K steps of all layers -----------------------------------------
    steps, warm = max(1, args.steps), max(0, args.warmup)

    def one_step(k):
        for L in layers:
            L.run("gated", k)

    if args.no_graph:
        def run_steps(n):
            for k in range(n):
                one_step(k)
    else:
        # a graph replays fixed buffers: one period of the buffer rotation per graph, plus one graph
        # for the remainder, so that exactly the number of steps asked for is run
        period = min(12, min(L.nset for L in layers))
        big = graph_of(one_step, period)
        rem_graphs = {}
        for n in (steps, warm):
            if n % period and n % period not in rem_graphs:
                rem_graphs[n % period] = graph_of(one_step, n % period)

        def run_steps(n):
            for _ in range(n // period):
                big.replay()
            if n % period:
                rem_graphs[n % period].replay()
    run_steps(warm)
    torch.cuda.synchronize()
    # K steps take a few milliseconds: the K-step region is timed several times (at least 50 ms in all)
    # and the median is reported
    t0 = time.perf_counter()
    run_steps(steps)
    torch.cuda.synchronize()
    first = time.perf_counter() - t0
    repeats = int(min(200, max(3, np.ceil(0.05 / max(first, 1e-6)))))
    times = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(steps)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    ms_per_step = float(np.median(times)) * 1e3 / steps

    dense_ops = sum(2 * L.shape.dense_macs for L in layers)
    value = dense_ops / (ms_per_step * 1e-3) / 1e12

    # ---- roofline of the dominant kernel (the fused MFMA layer kernel) -------------------------
    alg_flops = 0.0
    alg_bytes = 0.0
    ebl = 1 if args.dtype == "int8" else 2
    for L in layers:
        s = L.shape
        kp, kr = 9 * s.c_base, 9 * (s.c_in - s.c_base)
        alg_flops += 2.0 * s.m * s.c_out * (kp + L.rho * kr)
        alg_bytes += (s.n * s.h * s.w * s.c_in + s.m * s.c_out + s.c_out * 9 * s.c_in) * ebl + s.m * s.c_out / 8
    t_kernel_us = sum(L.us_gated for L in layers)
    achieved = alg_flops / (t_kernel_us * 1e-6) / 1e12
    kernel = KERNEL_OF.get(layers[-1].gated.variant, "?")
    traffic, traffic_from = None, None     # HBM bytes per launch come from the committed counter summary
    tfile = ROOT / "profiles" / ("hbm_traffic_%s_imagenet_resnet18_bf16_n64.txt" % kernel)
    peak = PEAK_INT8_TOPS if args.dtype == "int8" else PEAK_BF16_TFLOPS
    default_workload = (args.batch == 64 and not args.layers and args.kind == "coherent" and not args.grouped
                        and args.dtype == "bf16" and args.tau_c == 0.0 and args.variant == "auto"
                        and not args.fused_epilogue and abs(args.rho - 0.30) < 1e-9)
    if tfile.exists() and default_workload:
        m = re.search(r"^bytes_per_launch:\s*(\d+)", tfile.read_text(), re.M)
        if m:
            traffic = int(m.group(1))
            traffic_from = "profiles/" + tfile.name + " (rocprofv3 --pmc; not measured in this run)"
    roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=peak,
                    unit="TOP/s" if args.dtype == "int8" else "TFLOP/s",
                    frac=round(achieved / peak, 4), traffic=traffic, traffic_from=traffic_from,
                    kernel=kernel + "<%s>" % args.dtype, avg_launch_us=round(t_kernel_us / len(layers), 2),
                    timing="HIP events around graph replays of each layer's launches, on the replay stream",
                    algorithmic_gflop_per_launch=round(alg_flops / len(layers) / 1e9, 3),
                    algorithmic_mb_per_launch=round(alg_bytes / len(layers) / 1e6, 2),
                    hbm_gbs_algorithmic=round(alg_bytes / (t_kernel_us * 1e-6) / 1e9, 1),
                    hbm_frac=round(alg_bytes / (t_kernel_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4))

    # ---- CPU oracle on the host cores ----------------------------------------------------------
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(args, layers)

    per_layer = []
    for L in layers:
        s = L.shape
        row = dict(layer=s.name, kernel=KERNEL_OF.get(L.gated.variant, "?"), us_gated=round(L.us_gated, 2),
                   rho=round(L.rho, 4), beta_16px_x_16ch=round(L.beta_16x16, 3), beta_pixel_x_64ch=round(L.beta_px64, 3),
                   beta_pixel=round(L.beta_px, 3), eff_tops_gated=round(2 * s.dense_macs / L.us_gated / 1e6, 1))
        if L.us_dense is not None:
            row.update(us_dense=round(L.us_dense, 2), tops_dense=round(2 * s.dense_macs / L.us_dense / 1e6, 1),
                       speedup=round(L.us_dense / L.us_gated, 3))
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
                   "launch": "eager" if args.no_graph else "hip graph replay",
                   "cache": "warm (two buffer sets per layer)" if args.warm else "cold (buffers rotated past the 256 MB Infinity Cache)",
                   "timed_region": "exactly %d steps, timed %d times, median" % (steps, repeats),
                   "sum_us_gated": round(t_kernel_us, 2),
                   "sum_us_dense": None if args.no_dense else round(sum(L.us_dense for L in layers), 2),
                   "per_layer": per_layer},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


def cpu_baseline(args, layers):
    """The oracle on the host cores, on the same layers at the same batch: the parity build as it
    stands (both branches of Eq. 1 evaluated, double precision) and, beside it, the build that
    skips the conditional sum where the gate is closed (-O3, single-precision accumulators) with
    its dense counterpart (every gate open)."""
    import numpy as np
    from oracle import cg_oracle as O
    i8 = args.dtype == "int8"
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t_par = t_skip = t_dense = 0.0
    ops = 0
    for L in layers:
        s, inp, gate = L.shape, L.inp, L.gate
        groups = s.groups if args.grouped else 1
        ops += 2 * s.dense_macs
        if i8:
            tc = time.perf_counter()
            O.forward_int8(inp.x, inp.w_base, inp.w_cond, gate, stride=s.stride, pad=s.pad, out_i8=True,
                           epilogue=O.RELU, want_partials=False, groups=groups, tau_c=float(np.float32(args.tau_c)),
                           **L.rq)
            t_par += time.perf_counter() - tc
            if args.tau_c == 0.0:
                tc = time.perf_counter()
                O.forward_skip(inp.x, inp.w_base, inp.w_cond, thr=gate, stride=s.stride, pad=s.pad, groups=groups,
                               timed_build=True)
                t_skip += time.perf_counter() - tc
                tc = time.perf_counter()
                O.forward_skip(inp.x, inp.w_base, inp.w_cond, thr=np.full(s.c_out, np.iinfo(np.int32).min, np.int32),
                               stride=s.stride, pad=s.pad, groups=groups, timed_build=True)
                t_dense += time.perf_counter() - tc
            continue
        x64 = inp.x.astype(np.float64)
        wb64, wc64 = inp.w_base.astype(np.float64), inp.w_cond.astype(np.float64)
        tc = time.perf_counter()
        O.forward_float(x64, wb64, wc64, stride=s.stride, pad=s.pad, gate_mean=gate.mean, gate_var=gate.var,
                        delta=gate.delta, epilogue=O.RELU, want_partials=False, groups=groups,
                        tau_c=float(np.float32(args.tau_c)))
        t_par += time.perf_counter() - tc
        if args.tau_c == 0.0:
            kw = dict(stride=s.stride, pad=s.pad, gate_mean=gate.mean, gate_var=gate.var, groups=groups, timed_build=True)
            tc = time.perf_counter()
            O.forward_skip(x64, wb64, wc64, delta=gate.delta, **kw)
            t_skip += time.perf_counter() - tc
            tc = time.perf_counter()
            O.forward_skip(x64, wb64, wc64, delta=np.full(s.c_out, -np.inf), **kw)
            t_dense += time.perf_counter() - tc
    cpu = dict(value=round(ops / t_par / 1e12, 5), unit="TOP/s", cores=cores, kind="oracle", seconds=round(t_par, 2),
               sample="one pass of the full workload (all layers, batch %d), %s, both branches evaluated"
                      % (args.batch, "int32 sums" if i8 else "fp64"))
    if t_skip > 0:
        cpu["timed_build"] = dict(
            flags=" ".join(O.TIMED_FLAGS), cores=cores,
            gated=dict(value=round(ops / t_skip / 1e12, 5), unit="TOP/s", seconds=round(t_skip, 2),
                       what="conditional sum only where the gate fired; dense-equivalent ops / time"),
            dense=dict(value=round(ops / t_dense / 1e12, 5), unit="TOP/s", seconds=round(t_dense, 2),
                       what="the same code with every gate open"),
            speedup_gated_over_dense=round(t_dense / t_skip, 3))
    return cpu


if __name__ == "__main__":
    main()
