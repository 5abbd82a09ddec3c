"""Seeded synthetic inputs for the channel-gated convolution layer.

This module only *makes inputs*: activations, weights, gate statistics and
thresholds, quantised copies.  It contains none of the layer's own arithmetic
and is the one module that both the GPU tests/bench and the CPU oracle's tests
may share.  Gate statistics are calibrated with a library convolution
(``torch.nn.functional.conv2d`` on the CPU) over a few images; they are inputs
to the layer like any other, so neither the oracle nor the GPU library is
involved in producing them.

The layer shapes are those of ResNet-18 (the network the paper evaluates in its
experiments section); no dataset item or trained weight is reproduced, every
tensor is drawn from ``numpy.random.Generator(PCG64(seed))``.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 180512549


@dataclass(frozen=True)
class LayerShape:
    name: str
    n: int
    h: int
    w: int
    c_in: int
    c_out: int
    stride: int = 1
    pad: int = 1
    groups: int = 4          # G; the base path takes c_in // G channels
    k: int = 3

    @property
    def c_base(self) -> int:
        return self.c_in // self.groups

    @property
    def ho(self) -> int:
        return (self.h + 2 * self.pad - self.k) // self.stride + 1

    @property
    def wo(self) -> int:
        return (self.w + 2 * self.pad - self.k) // self.stride + 1

    @property
    def m(self) -> int:
        return self.n * self.ho * self.wo

    @property
    def dense_macs(self) -> int:
        return self.m * self.c_out * self.k * self.k * self.c_in

    def with_batch(self, n: int) -> "LayerShape":
        return replace(self, n=n)


def config1_shape() -> LayerShape:
    return LayerShape("c16_32x32_f32", 1, 32, 32, 16, 16)


def cifar_shapes(n: int = 128) -> List[LayerShape]:
    return [LayerShape("cifar_64@32", n, 32, 32, 64, 64),
            LayerShape("cifar_128@16", n, 16, 16, 128, 128),
            LayerShape("cifar_256@8", n, 8, 8, 256, 256),
            LayerShape("cifar_512@4", n, 4, 4, 512, 512)]


def imagenet_shapes(n: int = 64, groups: int = 4, with_stride2: bool = True) -> List[LayerShape]:
    s = [LayerShape("64@56", n, 56, 56, 64, 64, groups=groups),
         LayerShape("128@28", n, 28, 28, 128, 128, groups=groups),
         LayerShape("256@14", n, 14, 14, 256, 256, groups=groups),
         LayerShape("512@7", n, 7, 7, 512, 512, groups=groups)]
    if with_stride2:
        s += [LayerShape("64>128@56s2", n, 56, 56, 64, 128, stride=2, groups=groups),
              LayerShape("128>256@28s2", n, 28, 28, 128, 256, stride=2, groups=groups),
              LayerShape("256>512@14s2", n, 14, 14, 256, 512, stride=2, groups=groups)]
    return s


def resnet18_gated_convs(n: int = 256, groups: int = 4) -> List[LayerShape]:
    """The 16 residual-block 3x3 convolutions of ImageNet ResNet-18, in order."""
    out = []
    for i in range(4):
        out.append(LayerShape("l1.%d" % i, n, 56, 56, 64, 64, groups=groups))
    for c_in, c_out, hw, tag in ((64, 128, 56, "l2"), (128, 256, 28, "l3"), (256, 512, 14, "l4")):
        out.append(LayerShape(tag + ".0", n, hw, hw, c_in, c_out, stride=2, groups=groups))
        for i in range(1, 4):
            out.append(LayerShape("%s.%d" % (tag, i), n, hw // 2, hw // 2, c_out, c_out, groups=groups))
    return out


def seed_for(config: int, layer_index: int) -> int:
    return BASE_SEED + 1000 * config + layer_index


# ----------------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------------

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bfloat16, returned as float32."""
    return bf16_to_f32(bf16_bits(a))


# ----------------------------------------------------------------------------
# activations and weights
# ----------------------------------------------------------------------------

def _smooth_field(rng: np.random.Generator, n: int, h: int, w: int, sigma: float = 4.0) -> np.ndarray:
    from scipy.ndimage import gaussian_filter
    u = rng.random((n, h, w))
    return np.stack([gaussian_filter(u[i], sigma=sigma, mode="reflect") for i in range(n)])


@dataclass
class LayerInputs:
    shape: LayerShape
    kind: str
    x: np.ndarray        # float32 [N,H,W,C_in]
    w_base: np.ndarray   # float32 [C_out,3,3,C_base]
    w_cond: np.ndarray   # float32 [C_out,3,3,C_in-C_base]
    grouped: bool = False   # channel grouping: output group i has input group i as its base channels


def split_weights(wfull: np.ndarray, c_base: int, grouped: bool):
    """[C_out,k,k,C_in] weights in input-channel order -> (w_base, w_cond) in the layer's layouts.
    Ungrouped: the first c_base input channels are every output channel's base channels.  Grouped:
    with G = C_in / c_base groups, output channel co of group i = co // (C_out/G) takes input
    channels [i*c_base, (i+1)*c_base) as base and the others, in order, as conditional channels."""
    c_out, c_in = wfull.shape[0], wfull.shape[-1]
    if not grouped:
        return np.ascontiguousarray(wfull[..., :c_base]), np.ascontiguousarray(wfull[..., c_base:])
    g = c_in // c_base
    cpg = c_out // g
    own = (np.arange(c_out) // cpg)[:, None] * c_base + np.arange(c_base)[None, :]       # [C_out, c_base]
    mask = np.ones((c_out, c_in), bool)
    np.put_along_axis(mask, own, False, axis=1)
    rest = np.nonzero(mask)[1].reshape(c_out, c_in - c_base)                               # increasing per row
    idx_b = np.broadcast_to(own[:, None, None, :], wfull.shape[:3] + (c_base,))
    idx_r = np.broadcast_to(rest[:, None, None, :], wfull.shape[:3] + (c_in - c_base,))
    return (np.ascontiguousarray(np.take_along_axis(wfull, idx_b, axis=-1)),
            np.ascontiguousarray(np.take_along_axis(wfull, idx_r, axis=-1)))


def make_inputs(shape: LayerShape, seed: int, kind: str = "iid", rho: float = 0.3,
                round_bf16: bool = False, dc: float = 2.0, grouped: bool = False) -> LayerInputs:
    """kind: 'iid'      x = relu(N(0,1)), Kaiming-normal weights;
             'literal'  x additionally scaled by a smooth per-image magnitude field
                        (min-max normalised Gaussian-blurred uniform noise, sigma 4 px);
             'coherent' field sharpened into on/off regions covering min(1, rho+0.10)
                        of the pixels and a positive DC term added to the base weights,
                        so that the gates of different output channels fire together
                        (the spatially clustered maps of the paper's intensity figure).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    s = shape
    x = np.maximum(rng.standard_normal((s.n, s.h, s.w, s.c_in), dtype=np.float32), 0)
    std = np.sqrt(2.0 / (s.k * s.k * s.c_in))
    wfull = (rng.standard_normal((s.c_out, s.k, s.k, s.c_in), dtype=np.float32) * np.float32(std))
    if kind in ("literal", "coherent"):
        f = _smooth_field(rng, s.n, s.h, s.w)
        if kind == "literal":
            lo = f.min(axis=(1, 2), keepdims=True)
            hi = f.max(axis=(1, 2), keepdims=True)
            mfield = (f - lo) / np.maximum(hi - lo, 1e-12)
        else:
            on = min(1.0, rho + 0.10)
            q = np.quantile(f, 1.0 - on) if on < 1.0 else f.min() - 1.0
            mfield = np.clip((f - q) / 0.05 + 0.5, 0.0, 1.0)
            if grouped:
                cpg = s.c_out // s.groups
                for i in range(s.groups):      # the DC term sits on each output group's own base weights
                    wfull[i * cpg:(i + 1) * cpg, ..., i * s.c_base:(i + 1) * s.c_base] += np.float32(dc * std)
            else:
                wfull[..., : s.c_base] += np.float32(dc * std)
        x = x * mfield[..., None].astype(np.float32)
    elif kind != "iid":
        raise ValueError(kind)
    if round_bf16:
        x = bf16_round(x)
        wfull = bf16_round(wfull)
    w_base, w_cond = split_weights(wfull, s.c_base, grouped)
    return LayerInputs(s, kind, np.ascontiguousarray(x), w_base, w_cond, grouped)


# ----------------------------------------------------------------------------
# gate statistics (inputs of the layer; calibrated with a library convolution)
# ----------------------------------------------------------------------------

def _library_partial_sums(x: np.ndarray, w_base: np.ndarray, stride: int, pad: int,
                          grouped: bool = False) -> np.ndarray:
    """Base-path sums over the given images from torch's CPU convolution (its grouped convolution
    for a grouped layer), float64, [n,ho,wo,c_out]."""
    import torch
    c_base = w_base.shape[-1]
    groups = x.shape[-1] // c_base if grouped else 1
    xin = x if grouped else x[..., :c_base]
    xt = torch.from_numpy(np.ascontiguousarray(xin, dtype=np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w_base, dtype=np.float64)).permute(0, 3, 1, 2)
    p = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad, groups=groups)
    return p.permute(0, 2, 3, 1).contiguous().numpy()


@dataclass
class GateParams:
    mean: np.ndarray     # float64 [C_out]
    var: np.ndarray      # float64 [C_out], population variance
    delta: np.ndarray    # float64 [C_out]
    eps: float = 0.0


def calibrate_gate(inp: LayerInputs, rho: float, sample_images: Optional[int] = 8) -> GateParams:
    """Per-output-channel mean / population variance of the base partial sums over the
    first ``sample_images`` images, and one Delta (broadcast over channels) equal to the
    (1-rho) quantile of the normalised sums, so that about a fraction rho of gates fire."""
    s = inp.shape
    k = s.n if sample_images is None else min(s.n, sample_images)
    p = _library_partial_sums(inp.x[:k], inp.w_base, s.stride, s.pad, inp.grouped).reshape(-1, s.c_out)
    mean = p.mean(axis=0)
    var = p.var(axis=0)
    z = (p - mean) / np.sqrt(np.maximum(var, 1e-300))
    if rho <= 0.0:
        d = np.inf
    elif rho >= 1.0:
        d = -np.inf
    else:
        zs = np.sort(z.reshape(-1))
        kth = int(round(rho * zs.size))
        kth = min(max(kth, 1), zs.size)
        d = zs[zs.size - kth]        # the kth largest fires (ties fire too)
    return GateParams(mean, var, np.full(s.c_out, d, dtype=np.float64))


# ----------------------------------------------------------------------------
# int8 quantisation (symmetric; per-tensor activations, per-channel weights)
# ----------------------------------------------------------------------------

@dataclass
class Int8Inputs:
    shape: LayerShape
    x: np.ndarray        # int8 [N,H,W,C_in], values 0..127
    w_base: np.ndarray   # int8
    w_cond: np.ndarray   # int8
    s_x: float
    s_w: np.ndarray      # float64 [C_out]
    grouped: bool = False


def quantize_int8(inp: LayerInputs) -> Int8Inputs:
    s_x = float(inp.x.max()) / 127.0 if inp.x.max() > 0 else 1.0
    xq = np.clip(np.rint(inp.x / np.float32(s_x)), 0, 127).astype(np.int8)
    wmax = np.maximum(np.abs(inp.w_base).max(axis=(1, 2, 3)), np.abs(inp.w_cond).max(axis=(1, 2, 3))
                      if inp.w_cond.shape[-1] else 0.0)
    s_w = np.maximum(wmax.astype(np.float64), 1e-30) / 127.0
    sw4 = s_w.astype(np.float32)[:, None, None, None]
    wb = np.clip(np.rint(inp.w_base / sw4), -127, 127).astype(np.int8)
    wc = np.clip(np.rint(inp.w_cond / sw4), -127, 127).astype(np.int8)
    return Int8Inputs(inp.shape, xq, wb, wc, s_x, s_w, inp.grouped)


def calibrate_gate_int8(q: Int8Inputs, rho: float, sample_images: Optional[int] = 8) -> np.ndarray:
    """Integer threshold per output channel: ceil(E + Delta*sigma) of the integer base sums."""
    s = q.shape
    k = s.n if sample_images is None else min(s.n, sample_images)
    p = _library_partial_sums(q.x[:k].astype(np.float64), q.w_base.astype(np.float64), s.stride, s.pad, q.grouped)
    p = p.reshape(-1, s.c_out)
    mean = p.mean(axis=0)
    sd = np.sqrt(p.var(axis=0))
    if rho <= 0.0:
        return np.full(s.c_out, np.iinfo(np.int32).max, np.int32)
    if rho >= 1.0:
        return np.full(s.c_out, np.iinfo(np.int32).min, np.int32)
    z = (p - mean) / np.maximum(sd, 1e-300)
    zs = np.sort(z.reshape(-1))
    kth = min(max(int(round(rho * zs.size)), 1), zs.size)
    d = zs[zs.size - kth]
    t = np.ceil(mean + d * sd)
    return np.clip(t, np.iinfo(np.int32).min, np.iinfo(np.int32).max).astype(np.int32)


def requant_params(q: Int8Inputs, rng: np.random.Generator, shift: int = 16) -> Dict[str, np.ndarray]:
    """Plausible fixed-point requantisation constants: multiplier ~ s_x*s_w/s_y in Q(shift)."""
    s = q.shape
    k_total = s.k * s.k * s.c_in
    s_y = max(q.s_x * float(q.s_w.mean()) * np.sqrt(k_total) * 64.0 / 127.0, 1e-30)
    mult = np.clip(np.rint(q.s_x * q.s_w / s_y * (1 << shift)), 1, 2 ** 30).astype(np.int32)
    mult0 = np.clip(np.rint(mult * rng.uniform(0.9, 1.5, s.c_out)), 1, 2 ** 30).astype(np.int32)
    bias = rng.integers(-8, 9, s.c_out).astype(np.int32)
    return dict(rq_mult0=mult0, rq_mult1=mult, rq_bias=bias, rq_shift=shift)


# ----------------------------------------------------------------------------
# diagnostics on a decision map (reported beside timings)
# ----------------------------------------------------------------------------

def unpack_bitmap(bitmap: np.ndarray, c_out: int) -> np.ndarray:
    """[M, ceil(c_out/32)] uint32 words -> [M, c_out] uint8 decisions."""
    b = np.ascontiguousarray(bitmap, dtype=np.uint32)
    bits = np.unpackbits(b.view(np.uint8).reshape(b.shape[0], -1), axis=1, bitorder="little")
    return bits[:, :c_out]


def occupancy(d: np.ndarray, pixel_tile: int, channel_tile: int) -> float:
    """Fraction of (pixel_tile consecutive pixels x channel_tile channels) blocks holding a fired gate."""
    m, c = d.shape
    mp = -(-m // pixel_tile) * pixel_tile
    cp = -(-c // channel_tile) * channel_tile
    pad = np.zeros((mp, cp), np.uint8)
    pad[:m, :c] = d
    blk = pad.reshape(mp // pixel_tile, pixel_tile, cp // channel_tile, channel_tile).max(axis=(1, 3))
    return float(blk.mean())
