"""Small driver for HBM-traffic counters (run under ``rocprofv3 --pmc FETCH_SIZE`` and again under
``--pmc WRITE_SIZE``): launches a plain device copy of known size (the calibration kernel) and then one
cold-cache gated forward of every layer of the benchmark workload.

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out/fetch -o r -- python3 -m paper_1805_12549_amd.traffic_probe
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d out/write -o r -- python3 -m paper_1805_12549_amd.traffic_probe
    python -m paper_1805_12549_amd.profile_summary --traffic out/fetch/r_counter_collection.csv out/write/r_counter_collection.csv
"""
import sys

import torch

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W

COPY_BYTES = 256 << 20


def main(batch=64, rho=0.30):
    dev = torch.device("cuda:0")
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    flush = torch.empty(768 << 20, dtype=torch.uint8, device=dev)
    layers = []
    for li, s in enumerate(W.imagenet_shapes(n=batch)):
        inp = W.make_inputs(s, W.seed_for(3, li), kind="coherent", rho=rho, round_bf16=True)
        gate = W.calibrate_gate(inp, rho, sample_images=8)
        x = torch.from_numpy(inp.x).to(dev).to(torch.bfloat16)
        wb = torch.from_numpy(inp.w_base).to(dev).to(torch.bfloat16)
        wc = torch.from_numpy(inp.w_cond).to(dev).to(torch.bfloat16)
        layer = B.GatedConv(n_max=s.n, h=s.h, w=s.w, c_in=s.c_in, c_out=s.c_out, c_base=s.c_base, w_base=wb, w_cond=wc,
                            in_dtype=B.CG_BF16, out_dtype=B.CG_BF16, stride=s.stride, pad=s.pad,
                            gate_mean=gate.mean, gate_var=gate.var, delta=gate.delta)
        y = torch.empty((s.n, s.ho, s.wo, s.c_out), dtype=torch.bfloat16, device=dev)
        bm = torch.empty((s.m, s.c_out // 32), dtype=torch.int32, device=dev)
        layers.append((layer, x, y, bm))
    torch.cuda.synchronize()
    for _ in range(2):
        dst.copy_(src)                       # calibration: reads and writes COPY_BYTES
        torch.cuda.synchronize()
    for layer, x, y, bm in layers:
        flush.fill_(1)                       # push the layer's tensors out of the 256 MB infinity cache
        torch.cuda.synchronize()
        layer.forward(x, y=y, bitmap=bm, counts=False)
        torch.cuda.synchronize()
    print("traffic_probe done: copy of %d bytes, %d gated layers" % (COPY_BYTES, len(layers)), flush=True)


if __name__ == "__main__":
    main()
