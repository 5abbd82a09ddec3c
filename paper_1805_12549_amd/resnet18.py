"""A channel-gated ResNet-18 forward pass assembled from the C-ABI entry points.

Orchestration only: every layer runs in the HIP library (input convolution, max pooling, sixteen
gated 3x3 convolutions with fused scale/shift / residual / ReLU, three 1x1 stride-2 shortcut
convolutions, average pooling + fully connected layer).  Weights are random (there is no trained
network here); scale/shift pairs and gate statistics are calibrated on a few synthetic images so
that activations keep a stable range and about a fraction `rho` of the gates fire in every layer.

    python -m paper_1805_12549_amd.resnet18 --batch 64 --size 224 --rho 0.3
"""
from __future__ import annotations

import argparse
import json
import time
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from . import binding as B
from . import workloads as W


@dataclass
class ConvSpec:
    name: str
    c_in: int
    c_out: int
    hw: int          # input height = width
    stride: int
    relu: bool
    residual: bool   # adds the block input (or its shortcut) before the ReLU


def conv_specs(size: int) -> List[ConvSpec]:
    """The sixteen 3x3 convolutions of ResNet-18's residual blocks for a size x size input."""
    hw = ((size + 2 * 3 - 7) // 2 + 1 - 1) // 2 + 1          # after the input layer and the max pooling
    specs = []
    c = 64
    for stage, c_out in enumerate((64, 128, 256, 512)):
        for blk in range(2):
            stride = 2 if (stage > 0 and blk == 0) else 1
            specs.append(ConvSpec("l%d.%d.a" % (stage + 1, blk), c, c_out, hw, stride, True, False))
            hw = (hw - 1) // stride + 1
            specs.append(ConvSpec("l%d.%d.b" % (stage + 1, blk), c_out, c_out, hw, 1, True, True))
            c = c_out
    return specs


class _Shortcut:
    """A block's 1x1 stride-2 shortcut convolution with its scale/shift (cg_pointwise_conv)."""

    def __init__(self, spec, w, scale, shift):
        self.spec, self.w, self.scale, self.shift = spec, w, scale, shift

    def forward(self, x, bitmap=False, counts=False):
        s = self.spec
        n = x.shape[0]
        ho = (s.hw - 1) // 2 + 1
        y = torch.empty((n, ho, ho, s.c_out), dtype=torch.bfloat16, device=x.device)
        B.cg_pointwise_conv(x.data_ptr(), self.w.data_ptr(), self.scale.data_ptr(), self.shift.data_ptr(), y.data_ptr(),
                            n, s.hw, s.hw, s.c_in, s.c_out, 2, False, torch.cuda.current_stream().cuda_stream)
        return y, None, None

    def close(self):
        pass


def _t(a, dtype=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype).contiguous()


class GatedResNet18:
    """size x size RGB input, batch up to n_max.  groups = G of the gated layers (base path = C_in/G
    channels); grouped: channel grouping (Sec. 3.3).  rho = 0 builds the dense network (every 3x3
    layer with c_base == c_in)."""

    def __init__(self, n_max: int, size: int = 224, classes: int = 1000, groups: int = 4, rho: float = 0.3,
                 grouped: bool = False, seed: int = W.BASE_SEED + 5000, calib_images: int = 4):
        self.n_max, self.size, self.classes, self.groups, self.rho, self.grouped = n_max, size, classes, groups, rho, grouped
        self.gated = rho > 0
        rng = np.random.Generator(np.random.PCG64(seed))
        self.rng = rng
        k = 7
        self.w_in = _t(W.bf16_round((rng.standard_normal((64, k, k, 3)) * np.sqrt(2.0 / (k * k * 3))).astype(np.float32)))
        self.hw_in = (size + 2 * 3 - 7) // 2 + 1
        self.hw_pool = (self.hw_in - 1) // 2 + 1
        self.specs = conv_specs(size)
        self.layers: List[Optional[B.GatedConv]] = [None] * len(self.specs)
        self.shortcuts = {}
        self.records = {}       # per layer: the host-side parameters it was built with (for checks)
        self.scale_in = torch.ones(64, dtype=torch.float32, device="cuda")
        self.shift_in = torch.zeros(64, dtype=torch.float32, device="cuda")
        self.w_fc = _t(W.bf16_round((rng.standard_normal((classes, 512)) / np.sqrt(512)).astype(np.float32)))
        self.b_fc = _t(np.zeros(classes, np.float32), torch.float32)
        self._calibrate(calib_images)

    # -- building blocks -------------------------------------------------------------------------
    def _stream(self):
        return torch.cuda.current_stream().cuda_stream

    def _input_layer(self, x, keep_conv=True):
        """The input convolution and the max pooling; keep_conv=False runs them fused (the pooled tensor only)."""
        n = x.shape[0]
        if not keep_conv:
            p = torch.empty((n, self.hw_pool, self.hw_pool, 64), dtype=torch.bfloat16, device="cuda")
            B.cg_conv7x7s2_maxpool(x.data_ptr(), self.w_in.data_ptr(), self.scale_in.data_ptr(), self.shift_in.data_ptr(),
                                   p.data_ptr(), n, self.size, self.size, 64, 3, True, self._stream())
            return None, p
        y = torch.empty((n, self.hw_in, self.hw_in, 64), dtype=torch.bfloat16, device="cuda")
        B.cg_small_cin_conv(x.data_ptr(), self.w_in.data_ptr(), self.scale_in.data_ptr(), self.shift_in.data_ptr(),
                            y.data_ptr(), n, self.size, self.size, 3, 64, 7, 2, 3, True, self._stream())
        p = torch.empty((n, self.hw_pool, self.hw_pool, 64), dtype=torch.bfloat16, device="cuda")
        B.cg_maxpool3x3s2(y.data_ptr(), p.data_ptr(), n, self.hw_in, self.hw_in, 64, self._stream())
        return y, p

    def _make_conv(self, spec: ConvSpec, wfull, scale, shift, gate, n_max):
        """wfull: float32 [C_out,3,3,C_in] (bf16-rounded).  gate None: dense layer."""
        c_base = spec.c_in // self.groups if gate is not None else spec.c_in
        wb, wc = W.split_weights(wfull, c_base, self.grouped and gate is not None)
        epi = B.CG_EPI_AFFINE | (B.CG_EPI_RELU if spec.relu else 0) | (B.CG_EPI_RESIDUAL if spec.residual else 0)
        kw = {}
        if gate is not None:
            kw = dict(gate_mean=gate.mean, gate_var=gate.var, delta=gate.delta,
                      groups=self.groups if self.grouped else 0)
        return B.GatedConv(n_max=n_max, h=spec.hw, w=spec.hw, c_in=spec.c_in, c_out=spec.c_out, c_base=c_base,
                           w_base=_t(wb), w_cond=_t(wc) if gate is not None else None, in_dtype=B.CG_BF16,
                           out_dtype=B.CG_BF16, stride=spec.stride, pad=1, epilogue=epi, scale0=scale, shift0=shift,
                           scale1=scale, shift1=shift, **kw)

    def _make_shortcut(self, spec: ConvSpec, w, scale, shift, n_max):
        return _Shortcut(spec, _t(w), _t(scale, torch.float32), _t(shift, torch.float32))

    # -- calibration: scale/shift and gate statistics from a few synthetic images ---------------------
    @staticmethod
    def _norm(y, target_std=1.0, target_mean=0.25):
        """Per-channel scale/shift that bring the given pre-activation sums to the target statistics."""
        f = y.float().reshape(-1, y.shape[-1])
        mean, std = f.mean(0).cpu().numpy().astype(np.float64), f.std(0).cpu().numpy().astype(np.float64)
        scale = target_std / np.maximum(std, 1e-6)
        return scale.astype(np.float32), (target_mean - mean * scale).astype(np.float32)

    def _calibrate(self, n_cal: int):
        rng = self.rng
        size = self.size
        xin = np.maximum(rng.standard_normal((n_cal, size, size, 3), dtype=np.float32), 0)
        field = W._smooth_field(rng, n_cal, size, size, sigma=size / 14.0)      # large-scale structure
        lo, hi = field.min(axis=(1, 2), keepdims=True), field.max(axis=(1, 2), keepdims=True)
        xin = W.bf16_round(xin * ((field - lo) / np.maximum(hi - lo, 1e-12))[..., None].astype(np.float32))
        self.calib_input = xin
        x = _t(xin)
        # input layer: normalise its sums
        self.scale_in.fill_(1.0)
        self.shift_in.zero_()
        n = n_cal
        y = torch.empty((n, self.hw_in, self.hw_in, 64), dtype=torch.bfloat16, device="cuda")
        B.cg_small_cin_conv(x.data_ptr(), self.w_in.data_ptr(), 0, 0, y.data_ptr(), n, size, size, 3, 64, 7, 2, 3, False,
                            self._stream())
        torch.cuda.synchronize()
        sc, sh = self._norm(y)
        self.scale_in.copy_(torch.from_numpy(sc))
        self.shift_in.copy_(torch.from_numpy(sh))
        _, cur = self._input_layer(x)
        block_in = cur
        for i, spec in enumerate(self.specs):
            std = np.sqrt(2.0 / (9 * spec.c_in))
            wfull = rng.standard_normal((spec.c_out, 3, 3, spec.c_in), dtype=np.float32) * np.float32(std)
            c_base = spec.c_in // self.groups
            if self.gated:       # the positive DC term on the base weights that makes the gates follow the input magnitude
                if self.grouped:
                    cpg = spec.c_out // self.groups
                    for g in range(self.groups):
                        wfull[g * cpg:(g + 1) * cpg, ..., g * c_base:(g + 1) * c_base] += np.float32(2.0 * std)
                else:
                    wfull[..., :c_base] += np.float32(2.0 * std)
            wfull = W.bf16_round(wfull)
            ones, zeros = np.ones(spec.c_out, np.float32), np.zeros(spec.c_out, np.float32)
            # 1. the plain sums of the dense layer on the calibration images give scale / shift
            probe_spec = ConvSpec(spec.name, spec.c_in, spec.c_out, spec.hw, spec.stride, False, False)
            probe = self._make_conv(probe_spec, wfull, ones, zeros, None, n_cal)
            s_dense, _, _ = probe.forward(cur, bitmap=False, counts=False)
            torch.cuda.synchronize()
            probe.close()
            scale, shift = self._norm(s_dense, target_std=0.7 if spec.residual else 1.0)
            # 2. gate statistics from a library convolution of the base path on the same inputs
            gate = None
            if self.gated:
                wb, wc = W.split_weights(wfull, c_base, self.grouped)
                shape = W.LayerShape(spec.name, n_cal, spec.hw, spec.hw, spec.c_in, spec.c_out, stride=spec.stride,
                                     groups=self.groups)
                inp = W.LayerInputs(shape, "net", cur.float().cpu().numpy(), wb, wc, self.grouped)
                gate = W.calibrate_gate(inp, self.rho, sample_images=None)
            layer = self._make_conv(spec, wfull, scale, shift, gate, self.n_max)
            self.layers[i] = layer
            self.records[spec.name] = dict(spec=spec, wfull=wfull, scale=scale, shift=shift, gate=gate)
            # the residual operand of the block's second convolution
            res = None
            if spec.residual:
                first = self.specs[i - 1]
                if first.stride == 2:
                    wsc = W.bf16_round(rng.standard_normal((spec.c_out, 1, 1, first.c_in), dtype=np.float32)
                                       * np.float32(np.sqrt(2.0 / first.c_in)))
                    sc_spec = ConvSpec(first.name + ".sc", first.c_in, spec.c_out, first.hw, 2, False, False)
                    probe = self._make_shortcut(sc_spec, wsc, ones, zeros, n_cal)
                    s_sc, _, _ = probe.forward(block_in, bitmap=False, counts=False)
                    torch.cuda.synchronize()
                    probe.close()
                    ssc, shc = self._norm(s_sc, target_std=0.7, target_mean=0.0)
                    self.shortcuts[i] = self._make_shortcut(sc_spec, wsc, ssc, shc, self.n_max)
                    self.records[sc_spec.name] = dict(spec=sc_spec, w=wsc, scale=ssc, shift=shc)
                    res, _, _ = self.shortcuts[i].forward(block_in, bitmap=False, counts=False)
                else:
                    res = block_in
            out, _, _ = layer.forward(cur, residual=res, bitmap=False, counts=False)
            torch.cuda.synchronize()
            cur = out
            if spec.residual:
                block_in = cur

    # -- forward ---------------------------------------------------------------------------------------
    def forward(self, x, trace: Optional[dict] = None, want_counts: bool = False):
        """x: [n, size, size, 3] bf16 device tensor -> logits [n, classes] fp32.  trace: filled with every
        layer's input / residual / output / bitmap (device tensors) when given."""
        n = x.shape[0]
        stem, cur = self._input_layer(x, keep_conv=trace is not None)
        if trace is not None:
            trace["input"] = dict(x=x, y=stem, pooled=cur)
        block_in = cur
        fired = 0.0
        for i, spec in enumerate(self.specs):
            res = None
            if spec.residual:
                if i in self.shortcuts:
                    res, _, _ = self.shortcuts[i].forward(block_in, bitmap=False, counts=False)
                    if trace is not None:
                        trace[self.specs[i - 1].name + ".sc"] = dict(x=block_in, y=res)
                else:
                    res = block_in
            need = trace is not None or want_counts
            out, bm, cnt = self.layers[i].forward(cur, residual=res, bitmap=need and self.gated, counts=need and self.gated)
            if trace is not None:
                trace[spec.name] = dict(x=cur, residual=res, y=out, bitmap=bm, counts=cnt)
            cur = out
            if spec.residual:
                block_in = cur
        hw = cur.shape[1] * cur.shape[2]
        logits = torch.empty((n, self.classes), dtype=torch.float32, device="cuda")
        B.cg_avgpool_fc(cur.data_ptr(), self.w_fc.data_ptr(), self.b_fc.data_ptr(), logits.data_ptr(), n, hw, 512,
                        self.classes, self._stream())
        if trace is not None:
            trace["fc"] = dict(x=cur, y=logits)
        return logits

    def close(self):
        for layer in list(self.layers) + list(self.shortcuts.values()):
            if layer is not None:
                layer.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--size", type=int, default=224)
    ap.add_argument("--rho", type=float, default=0.3, help="target firing rate of the gates; 0 = dense network")
    ap.add_argument("--grouped", action="store_true")
    ap.add_argument("--steps", type=int, default=20)
    args = ap.parse_args()
    torch.cuda.set_device(0)
    out = {}
    for tag, rho in (("gated", args.rho), ("dense", 0.0)):
        net = GatedResNet18(args.batch, args.size, rho=rho, grouped=args.grouped and rho > 0)
        rng = np.random.default_rng(1)
        x = _t(np.tile(net.calib_input, (-(-args.batch // net.calib_input.shape[0]), 1, 1, 1))[:args.batch])
        for _ in range(3):
            net.forward(x)
        torch.cuda.synchronize()
        # the forward pass only enqueues kernels on the current stream: capture it once, replay it
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            net.forward(x)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                logits = net.forward(x)
        torch.cuda.synchronize()
        eager = net.forward(x)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(eager, logits), "graph replay differs from the eager pass"
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        fired = None
        if rho > 0:
            tr = {}
            net.forward(x, trace=tr)
            torch.cuda.synchronize()
            tot = act = 0
            for spec in net.specs:
                c = tr[spec.name]["counts"].cpu().numpy().view(np.uint32)
                tot += int(c[0]) | (int(c[1]) << 32)
                act += tr[spec.name]["y"].numel()
            fired = tot / act
        out[tag] = dict(images_per_s=round(args.batch / dt, 1), ms_per_batch=round(dt * 1e3, 3), fired=fired)
        net.close()
    print(json.dumps(dict(network="ResNet-18, %dx%d, batch %d, bf16, random weights, synthetic images" %
                          (args.size, args.size, args.batch), **out)))


if __name__ == "__main__":
    main()
