"""Times gated 1x1 convolutions and gated fully connected layers (h = w = k = 1) beside the dense
layer of the same shape, through the C ABI (large-tile matrix-core kernel), and prints one JSON line.

    python -m paper_1805_12549_amd.pointwise_probe [--rho 0.3] [--kind coherent]

The shapes are MobileNet-style point-wise layers and classifier-sized fully connected layers; inputs
are seeded and synthetic as in the 3x3 benchmark (clustered gate maps by default), buffers are rotated
past the Infinity Cache and every layer's calls are replayed as a HIP graph.
"""
import argparse
import json

import numpy as np
import torch

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W

SHAPES = [
    W.LayerShape("pw_128>128@28_n64", 64, 28, 28, 128, 128, pad=0, k=1),
    W.LayerShape("pw_256>256@14_n64", 64, 14, 14, 256, 256, pad=0, k=1),
    W.LayerShape("pw_512>512@7_n64", 64, 7, 7, 512, 512, pad=0, k=1),
    W.LayerShape("pw_1024>1024@14_n64", 64, 14, 14, 1024, 1024, pad=0, k=1),
    W.LayerShape("pw_512>512@14_n256", 256, 14, 14, 512, 512, pad=0, k=1),
    W.LayerShape("fc_512>1024_n64", 64, 1, 1, 512, 1024, pad=0, k=1),
    W.LayerShape("fc_4096>4096_n1024", 1024, 1, 1, 4096, 4096, pad=0, k=1),
    W.LayerShape("fc_4096>4096_n8192", 8192, 1, 1, 4096, 4096, pad=0, k=1),
]


def graph_us(fn, nset, rounds=5):
    calls = max(nset, 12)
    calls = (calls // nset) * nset
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn(0)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for k in range(calls):
                fn(k % nset)
    torch.cuda.synchronize()
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


def one(s, li, rho, kind):
    dev = torch.device("cuda:0")
    inp = W.make_inputs(s, W.seed_for(6, li), kind=kind, rho=rho, round_bf16=True)
    gate = W.calibrate_gate(inp, rho, sample_images=8 if s.h * s.w >= 49 else None)
    nset = min(24, max(2, int(np.ceil(600e6 / ((s.n * s.h * s.w * s.c_in + s.m * s.c_out) * 2)))))
    x0 = torch.from_numpy(inp.x).to(dev).to(torch.bfloat16)
    xs = [x0] + [x0.clone() for _ in range(nset - 1)]
    ys = [torch.empty((s.n, s.ho, s.wo, s.c_out), dtype=torch.bfloat16, device=dev) for _ in range(nset)]
    bms = [torch.empty((s.m, s.c_out // 32), dtype=torch.int32, device=dev) for _ in range(nset)]
    wb = torch.from_numpy(inp.w_base).to(dev).to(torch.bfloat16)
    wc = torch.from_numpy(inp.w_cond).to(dev).to(torch.bfloat16)
    common = dict(n_max=s.n, h=s.h, w=s.w, c_in=s.c_in, c_out=s.c_out, in_dtype=B.CG_BF16, out_dtype=B.CG_BF16,
                  stride=s.stride, pad=s.pad, kh=s.k, kw=s.k, epilogue=B.CG_EPI_RELU)
    gated = B.GatedConv(c_base=s.c_base, w_base=wb, w_cond=wc, gate_mean=gate.mean, gate_var=gate.var,
                        delta=gate.delta, **common)
    dense = B.GatedConv(c_base=s.c_in, w_base=torch.cat([wb, wc], -1).contiguous(), w_cond=None, **common)
    _, _, cnt = gated.forward(xs[0], y=ys[0], bitmap=bms[0], counts=True)
    torch.cuda.synchronize()
    c = cnt.cpu().numpy().view(np.uint32)
    fired = (int(c[0]) | (int(c[1]) << 32)) / (s.m * s.c_out)
    us_g = graph_us(lambda k: gated.forward(xs[k], y=ys[k], bitmap=bms[k], counts=False), nset)
    us_d = graph_us(lambda k: dense.forward(xs[k], y=ys[k], bitmap=False, counts=False), nset)
    gflop = 2.0 * s.m * s.c_out * s.c_in / 1e9
    row = dict(layer=s.name, kernel_family=gated.variant, rho=round(fired, 3), us_gated=round(us_g, 2),
               us_dense=round(us_d, 2), tflops_dense=round(gflop / us_d * 1e3, 1),
               speedup=round(us_d / us_g, 3))
    gated.close()
    dense.close()
    return row


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rho", type=float, default=0.30)
    ap.add_argument("--kind", default="coherent", choices=["coherent", "literal", "iid"])
    args = ap.parse_args()
    assert torch.cuda.is_available(), "pointwise_probe needs a GPU"
    rows = [one(s, li, args.rho, args.kind) for li, s in enumerate(SHAPES)]
    print(json.dumps({"what": "gated 1x1 / fully connected layers beside the dense layer of the same shape, bf16, us per call",
                      "maps": args.kind, "rho_target": args.rho, "layers": rows}))


if __name__ == "__main__":
    main()
