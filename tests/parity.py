"""Helpers of the GPU parity tests: run one layer through the C ABI (via the ctypes
binding) and through the CPU oracle on the same seeded inputs, and compare under
the stated rule.

Rule.  int8 path: y, bitmap, counts bit-identical.  Float paths: a decision may
differ from the oracle's only where the oracle's normalised margin |z - Delta| is
below 1e-3 (such flips are counted and reported); every output must be within
atol 1e-3 + rtol 2e-3 of the fp64 oracle value *for the decision the GPU took*
(the oracle keeps both branches); with a bf16 output buffer one bf16 ulp of the
reference is added to the allowance.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from oracle import cg_oracle as O
from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W

RTOL, ATOL, MARGIN = 2e-3, 1e-3, 1e-3


@dataclass
class Report:
    name: str
    fired_frac: float
    flips: int
    max_err: float
    variant: int

    def __str__(self):
        return "%s: variant=%d fired=%.3f flips=%d max_abs_err=%.3g" % (
            self.name, self.variant, self.fired_frac, self.flips, self.max_err)


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(dtype).contiguous()


def bf16_ulp(v):
    a = np.maximum(np.abs(v), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def run_float(inp: W.LayerInputs, gate: W.GateParams, *, in_dtype=B.CG_BF16, out_dtype=B.CG_F32,
              epilogue=B.CG_EPI_RELU, variant=B.CG_VARIANT_AUTO, affine=None, residual=None, delta_hi=None,
              n_run=None, name="", check_counts=True, shuffle=False, tau_c=0.0, tile_hint=0):
    """Runs the GPU library and the oracle; asserts parity; returns a Report.  A grouped input set
    (inp.grouped) runs the layer with channel grouping; shuffle stores y channel-shuffled."""
    s = inp.shape
    groups = s.groups if inp.grouped else 1
    tdt = torch.bfloat16 if in_dtype == B.CG_BF16 else torch.float32
    odt = torch.bfloat16 if out_dtype == B.CG_BF16 else torch.float32
    x = _dev(inp.x, tdt)
    wb = _dev(inp.w_base, tdt)
    wc = _dev(inp.w_cond, tdt) if inp.w_cond.shape[-1] else None
    aff = affine or {}
    k = inp.w_base.shape[1]
    layer = B.GatedConv(n_max=s.n, h=s.h, w=s.w, c_in=s.c_in, c_out=s.c_out, c_base=inp.w_base.shape[-1],
                        w_base=wb, w_cond=wc, in_dtype=in_dtype, out_dtype=out_dtype, kh=k, kw=k,
                        stride=s.stride, pad=s.pad, epilogue=epilogue, variant=variant,
                        gate_mean=gate.mean if gate else None, gate_var=gate.var if gate else None,
                        delta=gate.delta if gate else None, delta_hi=delta_hi, gate_eps=gate.eps if gate else 0.0,
                        groups=groups, shuffle=shuffle, tau_c=tau_c, tile_hint=tile_hint, **aff)
    n = s.n if n_run is None else n_run
    res_dev = None
    res_host = None
    if residual is not None:
        # the residual lives in the output dtype on the device; the oracle sees the stored values
        res_dev = _dev(residual[:n], odt)
        res_host = res_dev.to(torch.float32).cpu().numpy().astype(np.float64)
    y, bitmap, counts = layer.forward(x[:n], residual=res_dev)
    torch.cuda.synchronize()
    y = y.to(torch.float32).cpu().numpy().astype(np.float64)
    bitmap = bitmap.cpu().numpy().view(np.uint32)
    counts = counts.cpu().numpy().view(np.uint32)
    variant_used = layer.variant
    layer.close()

    # the library's float tables are fp32: hand the oracle the same fp32-rounded statistics
    f32 = lambda a: None if a is None else np.asarray(a, np.float32).astype(np.float64)
    ref = O.forward_float(
        inp.x[:n], inp.w_base, inp.w_cond if wc is not None else None, stride=s.stride, pad=s.pad,
        gate_mean=f32(gate.mean) if gate else None, gate_var=f32(gate.var) if gate else None,
        delta=f32(gate.delta) if gate else None, delta_hi=f32(delta_hi),
        gate_eps=float(np.float32(gate.eps)) if gate else 0.0,
        scale0=f32(aff.get("scale0")), shift0=f32(aff.get("shift0")),
        scale1=f32(aff.get("scale1")), shift1=f32(aff.get("shift1")),
        residual=res_host, epilogue=epilogue, want_partials=False, groups=groups, shuffle=shuffle,
        tau_c=float(np.float32(tau_c)))
    need = None
    if tau_c > 0 and gate is not None:
        need = float(np.ceil(float(np.float32(tau_c)) * (s.ho * s.wo)))
    return compare_float(name or s.name, y, bitmap, counts, ref, s.c_out, out_dtype, variant_used, check_counts,
                         stored_groups=groups if shuffle else 0, chan_need=need)


def compare_float(name, y, bitmap, counts, ref, c_out, out_dtype, variant_used, check_counts=True,
                  stored_groups=0, chan_need=None):
    """stored_groups = G > 0: y holds the channels shuffled (channel j of group i at j*G + i) while
    the decisions keep the natural order.  chan_need = the fired count an (image, channel) needs to
    keep its conditional path under the channel-wise gate: where the oracle's count is within the
    number of that channel's marginal activations of it, the whole channel may go either way."""
    d_gpu = W.unpack_bitmap(bitmap, c_out).reshape(ref["d"].shape)
    d_ref = ref["d"]
    flip = d_gpu != d_ref
    nflip = int(flip.sum())
    if nflip:
        marginal = ref["margin"] < MARGIN
        allowed = marginal
        if chan_need is not None:
            n_img = d_ref.shape[0]
            pre = ref["pre_counts"].reshape(n_img, c_out).astype(np.int64)
            slack = marginal.reshape(n_img, -1, c_out).sum(axis=1)
            borderline = np.abs(pre - chan_need) <= slack
            allowed = marginal | borderline[:, None, None, :]
        bad_flip = flip & ~allowed
        assert not bad_flip.any(), "%s: %d decision flips outside the margin %g (worst margin %.3g)" % (
            name, int(bad_flip.sum()), MARGIN, float(ref["margin"][bad_flip].max()))
    # unused bitmap bits must be zero
    if c_out % 32:
        assert (bitmap[:, -1] >> np.uint32(c_out % 32) == 0).all(), "%s: unused bitmap bits set" % name
    flip_y = flip
    if stored_groups:
        sh = flip.shape
        flip_y = flip.reshape(sh[:-1] + (stored_groups, c_out // stored_groups)).swapaxes(-1, -2).reshape(sh)
    want = np.where(flip_y, ref["y_other"], ref["y"])
    tol = ATOL + RTOL * np.abs(want)
    if out_dtype == B.CG_BF16:
        tol = tol + bf16_ulp(want)
    err = np.abs(y - want)
    bad = err > tol
    assert not bad.any(), "%s: %d outputs out of tolerance, worst err %.4g (want %.6g got %.6g)" % (
        name, int(bad.sum()), float(err[bad].max()), float(want[bad][0]), float(y[bad][0]))
    if check_counts:
        total = int(counts[0]) | (int(counts[1]) << 32)
        assert total == int(d_gpu.sum()), "%s: total count %d != bitmap popcount %d" % (name, total, int(d_gpu.sum()))
        per = d_gpu.reshape(d_gpu.shape[0], -1, c_out).sum(axis=1).reshape(-1)
        assert np.array_equal(counts[2:], per.astype(np.uint32)), "%s: per-(image,channel) counts differ" % name
    return Report(name, float(d_gpu.mean()), nflip, float(err.max()) if err.size else 0.0, variant_used)


def run_int8(q: W.Int8Inputs, thr, *, out_i8=False, epilogue=B.CG_EPI_RELU, variant=B.CG_VARIANT_AUTO,
             rq=None, residual=None, rq_res_mult=0, n_run=None, name="", shuffle=False, tau_c=0.0, tile_hint=0):
    s = q.shape
    groups = s.groups if q.grouped else 1
    x = _dev(q.x, torch.int8)
    wb = _dev(q.w_base, torch.int8)
    wc = _dev(q.w_cond, torch.int8) if q.w_cond.shape[-1] else None
    rq = rq or {}
    k = q.w_base.shape[1]
    layer = B.GatedConv(n_max=s.n, h=s.h, w=s.w, c_in=s.c_in, c_out=s.c_out, c_base=q.w_base.shape[-1],
                        w_base=wb, w_cond=wc, in_dtype=B.CG_I8, out_dtype=B.CG_I8 if out_i8 else B.CG_I32,
                        kh=k, kw=k, stride=s.stride, pad=s.pad, epilogue=epilogue, variant=variant,
                        gate_thr_i32=thr, rq_res_mult=rq_res_mult, groups=groups, shuffle=shuffle, tau_c=tau_c,
                        tile_hint=tile_hint, **rq)
    n = s.n if n_run is None else n_run
    res_dev = _dev(residual[:n], torch.int8) if residual is not None else None
    y, bitmap, counts = layer.forward(x[:n], residual=res_dev)
    torch.cuda.synchronize()
    y = y.cpu().numpy().astype(np.int32)
    bitmap = bitmap.cpu().numpy().view(np.uint32)
    counts = counts.cpu().numpy().view(np.uint32)
    variant_used = layer.variant
    layer.close()
    ref = O.forward_int8(q.x[:n], q.w_base, q.w_cond if wc is not None else None, thr, stride=s.stride, pad=s.pad,
                         out_i8=out_i8, residual=residual[:n] if residual is not None else None,
                         rq_res_mult=rq_res_mult, epilogue=epilogue, want_partials=False, groups=groups,
                         shuffle=shuffle, tau_c=float(np.float32(tau_c)), **rq)
    nm = name or s.name
    assert np.array_equal(bitmap, ref["bitmap"]), "%s: bitmap differs in %d words" % (
        nm, int((bitmap != ref["bitmap"]).sum()))
    assert np.array_equal(counts, ref["counts"]), "%s: counts differ" % nm
    neq = y != ref["y"]
    assert not neq.any(), "%s: %d outputs differ (first: got %d want %d)" % (
        nm, int(neq.sum()), int(y[neq][0]), int(ref["y"][neq][0]))
    return Report(nm, float(ref["d"].mean()), 0, 0.0, variant_used)
