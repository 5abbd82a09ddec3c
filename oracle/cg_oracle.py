"""ctypes front end of the CPU oracle (``cg_ref.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the CPU-baseline leg
of the benchmark may import this module; the GPU library never does, and this
module imports nothing from the GPU package.

The arithmetic lives in ``cg_ref.c``; this file only widens inputs to the types
the C code takes (double for the float path, int8 for the integer path),
allocates outputs and fills the problem struct.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "cg_ref.c"
_LIB = _HERE / "libcg_ref.so"

RELU, AFFINE, RESIDUAL = 1, 2, 4


def build(force: bool = False) -> Path:
    """Compile cg_ref.c with gcc (plain -O2, OpenMP over output rows)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_pd = C.POINTER(C.c_double)
_pi8 = C.POINTER(C.c_int8)
_pi32 = C.POINTER(C.c_int32)
_pu8 = C.POINTER(C.c_uint8)
_pu32 = C.POINTER(C.c_uint32)
_pu64 = C.POINTER(C.c_uint64)


class _Problem(C.Structure):
    _fields_ = [
        ("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("c_in", C.c_int32),
        ("c_out", C.c_int32), ("c_base", C.c_int32),
        ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
        ("is_int", C.c_int32), ("out_i8", C.c_int32), ("epilogue", C.c_uint32),
        ("two_sided", C.c_int32), ("groups", C.c_int32), ("shuffle", C.c_int32),
        ("tau_c", C.c_double),
        ("x", _pd), ("w_base", _pd), ("w_cond", _pd),
        ("gate_mean", _pd), ("gate_var", _pd), ("delta", _pd), ("delta_hi", _pd),
        ("gate_eps", C.c_double),
        ("scale0", _pd), ("shift0", _pd), ("scale1", _pd), ("shift1", _pd),
        ("residual", _pd),
        ("xi", _pi8), ("wi_base", _pi8), ("wi_cond", _pi8),
        ("thr", _pi32), ("rq_mult0", _pi32), ("rq_mult1", _pi32), ("rq_bias", _pi32),
        ("rq_shift", C.c_int32), ("residual_i8", _pi8), ("rq_res_mult", C.c_int32),
        ("P", _pd), ("R", _pd), ("y", _pd), ("y_other", _pd), ("margin", _pd),
        ("Pi", _pi32), ("Ri", _pi32), ("yi", _pi32), ("yi_other", _pi32),
        ("d", _pu8), ("bitmap", _pu32), ("counts", _pu32), ("macs", _pu64),
        ("pre_counts", _pu32),
    ]


_LIB_TIMED = _HERE / "libcg_ref_timed.so"
TIMED_FLAGS = ["-O3", "-march=native", "-fopenmp", "-DCG_REF_ACC=float"]


def build_timed(force: bool = False) -> Path:
    """The same source built for the CPU timing of the benchmark: -O3 -march=native and
    single-precision accumulators in cg_ref_forward_skip.  Never used for parity."""
    if force or not _LIB_TIMED.exists() or _LIB_TIMED.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB_TIMED.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(["gcc", *TIMED_FLAGS, "-fPIC", "-shared", "-std=c11", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB_TIMED)
    return _LIB_TIMED


_lib = None
_lib_timed = None


def _load_timed():
    global _lib_timed
    if _lib_timed is None:
        build_timed()
        _lib_timed = C.CDLL(str(_LIB_TIMED))
        _lib_timed.cg_ref_forward_skip.argtypes = [C.POINTER(_Problem)]
        _lib_timed.cg_ref_forward_skip.restype = C.c_int
    return _lib_timed


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(str(_LIB))
        _lib.cg_ref_forward.argtypes = [C.POINTER(_Problem)]
        _lib.cg_ref_forward.restype = C.c_int
        _lib.cg_ref_forward_skip.argtypes = [C.POINTER(_Problem)]
        _lib.cg_ref_forward_skip.restype = C.c_int
    return _lib


def out_hw(h, w, kh, kw, stride, pad):
    ho = (h + 2 * pad - kh) // stride + 1 if h + 2 * pad - kh >= 0 else 0
    wo = (w + 2 * pad - kw) // stride + 1 if w + 2 * pad - kw >= 0 else 0
    return ho, wo


def _as(a, dtype):
    return None if a is None else np.ascontiguousarray(np.asarray(a), dtype=dtype)


def _ptr(a, ptype):
    return None if a is None else a.ctypes.data_as(ptype)


def forward_float(x, w_base, w_cond, *, stride=1, pad=1, gate_mean=None, gate_var=None, delta=None,
                  delta_hi=None, gate_eps=0.0, scale0=None, shift0=None, scale1=None, shift1=None,
                  residual=None, epilogue=RELU, want_partials=True, groups=1, shuffle=False, tau_c=0.0):
    """Float path.  x [N,H,W,C_in]; w_base [C_out,kh,kw,C_base]; w_cond [C_out,kh,kw,C_in-C_base]
    (None or zero-width for a dense layer).  Every array is widened to float64 exactly.
    groups > 1: channel grouping (output group i uses input group i as base), optionally with the
    output channels of y stored shuffled.  tau_c > 0: channel-wise gate (an image's output channel
    keeps its conditional path only if at least tau_c of its activations fired); out["pre_counts"]
    holds the sums it thresholds."""
    lib = _load()
    x = _as(x, np.float64)
    w_base = _as(w_base, np.float64)
    n, h, w, c_in = x.shape
    c_out, kh, kw, c_base = w_base.shape
    c_r = c_in - c_base
    if c_r > 0:
        w_cond = _as(w_cond, np.float64)
        assert w_cond.shape == (c_out, kh, kw, c_r), w_cond.shape
    else:
        w_cond = None
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    shape = (n, ho, wo, c_out)
    words = (c_out + 31) // 32
    keep = dict(x=x, w_base=w_base, w_cond=w_cond)
    for name, v in (("gate_mean", gate_mean), ("gate_var", gate_var), ("delta", delta), ("delta_hi", delta_hi),
                    ("scale0", scale0), ("shift0", shift0), ("scale1", scale1), ("shift1", shift1)):
        v = _as(v, np.float64)
        if v is not None:
            if v.ndim == 0:
                v = np.full(c_out, float(v))
            assert v.shape == (c_out,), (name, v.shape)
        keep[name] = v
    residual = _as(residual, np.float64)
    if residual is not None:
        assert residual.shape == shape
    out = dict(
        y=np.empty(shape), y_other=np.empty(shape), margin=np.empty(shape),
        d=np.empty(shape, np.uint8), bitmap=np.empty((n * ho * wo, words), np.uint32),
        counts=np.empty(2 + n * c_out, np.uint32))
    if want_partials:
        out["P"] = np.empty(shape)
        out["R"] = np.empty(shape)
    macs = C.c_uint64(0)
    p = _Problem()
    p.n, p.h, p.w, p.c_in, p.c_out, p.c_base = n, h, w, c_in, c_out, c_base
    p.kh, p.kw, p.stride, p.pad = kh, kw, stride, pad
    p.is_int, p.out_i8, p.epilogue = 0, 0, epilogue
    p.two_sided = 1 if delta_hi is not None else 0
    p.groups, p.shuffle = int(groups), int(bool(shuffle))
    p.tau_c = float(tau_c)
    out["pre_counts"] = np.empty(n * c_out, np.uint32)
    p.pre_counts = _ptr(out["pre_counts"], _pu32)
    p.gate_eps = gate_eps
    for name in ("x", "w_base", "w_cond", "gate_mean", "gate_var", "delta", "delta_hi",
                 "scale0", "shift0", "scale1", "shift1"):
        setattr(p, name, _ptr(keep[name], _pd))
    p.residual = _ptr(residual, _pd)
    for name in ("y", "y_other", "margin", "P", "R"):
        if name in out:
            setattr(p, name, _ptr(out[name], _pd))
    p.d = _ptr(out["d"], _pu8)
    p.bitmap = _ptr(out["bitmap"], _pu32)
    p.counts = _ptr(out["counts"], _pu32)
    p.macs = C.pointer(macs)
    rc = lib.cg_ref_forward(C.byref(p))
    if rc != 0:
        raise ValueError("cg_ref_forward rejected the problem (rc=%d)" % rc)
    out["macs"] = int(macs.value)
    out["fired"] = int(out["counts"][0]) | (int(out["counts"][1]) << 32)
    return out


def forward_skip(x, w_base, w_cond, *, thr=None, stride=1, pad=1, gate_mean=None, gate_var=None, delta=None,
                 gate_eps=0.0, epilogue=RELU, groups=1, timed_build=False):
    """The layer as Eq. 1 executes it (cg_ref_forward_skip): the conditional sum is evaluated only
    where the gate fired.  Float path when ``thr`` is None (x, w widened to float64), else the int8
    path with the integer thresholds ``thr`` (raw int32 sums out).  timed_build: the -O3 build with
    single-precision accumulators that the benchmark times.  Returns y, d, bitmap, counts, macs."""
    lib = _load_timed() if timed_build else _load()
    is_int = thr is not None
    dt = np.int8 if is_int else np.float64
    x = _as(x, dt)
    w_base = _as(w_base, dt)
    n, h, w, c_in = x.shape
    c_out, kh, kw, c_base = w_base.shape
    w_cond = _as(w_cond, dt) if c_in > c_base else None
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    shape = (n, ho, wo, c_out)
    words = (c_out + 31) // 32
    out = dict(y=np.empty(shape, np.int32 if is_int else np.float64), d=np.empty(shape, np.uint8),
               bitmap=np.empty((n * ho * wo, words), np.uint32), counts=np.empty(2 + n * c_out, np.uint32))
    macs = C.c_uint64(0)
    p = _Problem()
    p.n, p.h, p.w, p.c_in, p.c_out, p.c_base = n, h, w, c_in, c_out, c_base
    p.kh, p.kw, p.stride, p.pad = kh, kw, stride, pad
    p.is_int, p.out_i8, p.epilogue = int(is_int), 0, epilogue
    p.groups = int(groups)
    p.gate_eps = gate_eps
    keep = []
    if is_int:
        thr = _as(thr, np.int32)
        p.xi, p.wi_base, p.wi_cond, p.thr = _ptr(x, _pi8), _ptr(w_base, _pi8), _ptr(w_cond, _pi8), _ptr(thr, _pi32)
        p.yi = _ptr(out["y"], _pi32)
    else:
        p.x, p.w_base, p.w_cond = _ptr(x, _pd), _ptr(w_base, _pd), _ptr(w_cond, _pd)
        for name, v in (("gate_mean", gate_mean), ("gate_var", gate_var), ("delta", delta)):
            v = _as(v, np.float64)
            keep.append(v)
            setattr(p, name, _ptr(v, _pd))
        p.y = _ptr(out["y"], _pd)
    p.d = _ptr(out["d"], _pu8)
    p.bitmap = _ptr(out["bitmap"], _pu32)
    p.counts = _ptr(out["counts"], _pu32)
    p.macs = C.pointer(macs)
    rc = lib.cg_ref_forward_skip(C.byref(p))
    if rc != 0:
        raise ValueError("cg_ref_forward_skip rejected the problem (rc=%d)" % rc)
    out["macs"] = int(macs.value)
    out["fired"] = int(out["counts"][0]) | (int(out["counts"][1]) << 32)
    return out


def forward_int8(x, w_base, w_cond, thr, *, stride=1, pad=1, out_i8=False, rq_mult0=None, rq_mult1=None,
                 rq_bias=None, rq_shift=0, residual=None, rq_res_mult=0, epilogue=RELU, want_partials=True,
                 groups=1, shuffle=False, tau_c=0.0):
    """Integer path: int8 inputs, int32 accumulation, int32 thresholds; exact."""
    lib = _load()
    x = _as(x, np.int8)
    w_base = _as(w_base, np.int8)
    n, h, w, c_in = x.shape
    c_out, kh, kw, c_base = w_base.shape
    c_r = c_in - c_base
    w_cond = _as(w_cond, np.int8) if c_r > 0 else None
    if w_cond is not None:
        assert w_cond.shape == (c_out, kh, kw, c_r)
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    shape = (n, ho, wo, c_out)
    words = (c_out + 31) // 32
    thr = _as(thr, np.int32)
    rq_mult0, rq_mult1, rq_bias = _as(rq_mult0, np.int32), _as(rq_mult1, np.int32), _as(rq_bias, np.int32)
    residual = _as(residual, np.int8)
    out = dict(
        y=np.empty(shape, np.int32), y_other=np.empty(shape, np.int32), margin=np.empty(shape),
        d=np.empty(shape, np.uint8), bitmap=np.empty((n * ho * wo, words), np.uint32),
        counts=np.empty(2 + n * c_out, np.uint32))
    if want_partials:
        out["P"] = np.empty(shape, np.int32)
        out["R"] = np.empty(shape, np.int32)
    macs = C.c_uint64(0)
    p = _Problem()
    p.n, p.h, p.w, p.c_in, p.c_out, p.c_base = n, h, w, c_in, c_out, c_base
    p.kh, p.kw, p.stride, p.pad = kh, kw, stride, pad
    p.is_int, p.out_i8, p.epilogue = 1, int(bool(out_i8)), epilogue
    p.groups, p.shuffle = int(groups), int(bool(shuffle))
    p.tau_c = float(tau_c)
    out["pre_counts"] = np.empty(n * c_out, np.uint32)
    p.pre_counts = _ptr(out["pre_counts"], _pu32)
    p.xi, p.wi_base, p.wi_cond = _ptr(x, _pi8), _ptr(w_base, _pi8), _ptr(w_cond, _pi8)
    p.thr = _ptr(thr, _pi32)
    p.rq_mult0, p.rq_mult1, p.rq_bias = _ptr(rq_mult0, _pi32), _ptr(rq_mult1, _pi32), _ptr(rq_bias, _pi32)
    p.rq_shift = rq_shift
    p.residual_i8 = _ptr(residual, _pi8)
    p.rq_res_mult = rq_res_mult
    p.yi, p.yi_other = _ptr(out["y"], _pi32), _ptr(out["y_other"], _pi32)
    p.margin = _ptr(out["margin"], _pd)
    if want_partials:
        p.Pi, p.Ri = _ptr(out["P"], _pi32), _ptr(out["R"], _pi32)
    p.d = _ptr(out["d"], _pu8)
    p.bitmap = _ptr(out["bitmap"], _pu32)
    p.counts = _ptr(out["counts"], _pu32)
    p.macs = C.pointer(macs)
    rc = lib.cg_ref_forward(C.byref(p))
    if rc != 0:
        raise ValueError("cg_ref_forward rejected the problem (rc=%d)" % rc)
    out["macs"] = int(macs.value)
    out["fired"] = int(out["counts"][0]) | (int(out["counts"][1]) << 32)
    return out


# ----------------------------------------------------------------------------
# dense pieces of a ResNet around the gated layers (plain definitions in cg_ref.c)
# ----------------------------------------------------------------------------

def dense_conv(x, w, *, stride=1, pad=0, scale=None, shift=None, relu=False):
    """x [N,H,W,C_in], w [C_out,k,k,C_in] -> [N,Ho,Wo,C_out] float64."""
    lib = _load()
    x, w = _as(x, np.float64), _as(w, np.float64)
    n, h, wd, c_in = x.shape
    c_out, k = w.shape[0], w.shape[1]
    assert w.shape == (c_out, k, k, c_in)
    scale, shift = _as(scale, np.float64), _as(shift, np.float64)
    ho, wo = out_hw(h, wd, k, k, stride, pad)
    y = np.empty((n, ho, wo, c_out))
    lib.cg_ref_dense_conv.argtypes = [_pd, _pd, _pd, _pd, _pd] + [C.c_int] * 9
    rc = lib.cg_ref_dense_conv(_ptr(x, _pd), _ptr(w, _pd), _ptr(scale, _pd), _ptr(shift, _pd), _ptr(y, _pd),
                               n, h, wd, c_in, c_out, k, stride, pad, int(bool(relu)))
    if rc != 0:
        raise ValueError("cg_ref_dense_conv rejected the problem")
    return y


def maxpool3x3s2(x):
    """x [N,H,W,C] -> [N,(H-1)//2+1,(W-1)//2+1,C] float64 (padding 1)."""
    lib = _load()
    x = _as(x, np.float64)
    n, h, wd, c = x.shape
    ho, wo = out_hw(h, wd, 3, 3, 2, 1)
    y = np.empty((n, ho, wo, c))
    lib.cg_ref_maxpool3x3s2.argtypes = [_pd, _pd] + [C.c_int] * 4
    if lib.cg_ref_maxpool3x3s2(_ptr(x, _pd), _ptr(y, _pd), n, h, wd, c) != 0:
        raise ValueError("cg_ref_maxpool3x3s2 rejected the problem")
    return y


def avgpool_fc(x, wfc, bias=None):
    """x [N,HW,C] (or [N,H,W,C]), wfc [classes,C] -> logits [N,classes] float64."""
    lib = _load()
    x, wfc, bias = _as(x, np.float64), _as(wfc, np.float64), _as(bias, np.float64)
    n, c = x.shape[0], x.shape[-1]
    hw = int(np.prod(x.shape[1:-1]))
    classes = wfc.shape[0]
    assert wfc.shape == (classes, c)
    out = np.empty((n, classes))
    lib.cg_ref_avgpool_fc.argtypes = [_pd, _pd, _pd, _pd] + [C.c_int] * 4
    if lib.cg_ref_avgpool_fc(_ptr(x, _pd), _ptr(wfc, _pd), _ptr(bias, _pd), _ptr(out, _pd), n, hw, c, classes) != 0:
        raise ValueError("cg_ref_avgpool_fc rejected the problem")
    return out
