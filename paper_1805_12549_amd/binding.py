"""ctypes binding of the C-ABI library (``include/cg_conv.h``), same names.

Argument marshalling only: every step of the layer runs in the HIP kernels of
``libcg_conv.so``.  There is no CPU fallback; importing this module raises if the
library has not been built (``python paper_1805_12549_amd/build.py``).
PyTorch appears only as the owner of device memory and streams: tensors are
reduced to raw device pointers before they cross the boundary.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional

import numpy as np

# The PyTorch wheel ships its own HIP runtime (soname libamdhip64.so.7).  The library and
# torch must share ONE runtime or the second one finds no device, so torch is imported
# first: the loader then resolves libcg_conv.so's libamdhip64.so.7 to the copy already mapped.
import torch  # noqa: F401,E402

_LIB_PATH = Path(__file__).resolve().parent / "libcg_conv.so"
if not _LIB_PATH.exists():
    raise ImportError(
        "%s is missing: build the HIP library first (python paper_1805_12549_amd/build.py or "
        "__graft_entry__.build()); there is no fallback path" % _LIB_PATH)
_lib = C.CDLL(str(_LIB_PATH))


def _hip_runtimes_mapped():
    seen = set()
    try:
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    seen.add(line.split()[-1])
    except OSError:
        pass
    return sorted(seen)


if len(_hip_runtimes_mapped()) > 1:
    raise ImportError("two HIP runtimes are mapped into this process (%s); import torch before anything "
                      "that loads libamdhip64" % ", ".join(_hip_runtimes_mapped()))

CG_OK, CG_EINVAL, CG_EUNSUPPORTED, CG_ENOMEM, CG_EHIP = 0, 1, 2, 3, 4
CG_F32, CG_BF16, CG_I8, CG_I32 = 0, 1, 2, 3
CG_EPI_RELU, CG_EPI_AFFINE, CG_EPI_RESIDUAL = 1, 2, 4
CG_VARIANT_AUTO, CG_VARIANT_NAIVE, CG_VARIANT_MFMA_ROWS, CG_VARIANT_TILE = 0, 1, 4, 5

EXPORTS = ("cg_conv_packed_bytes", "cg_conv_create", "cg_conv_workspace_bytes", "cg_conv_forward",
           "cg_conv_forward_noalloc",
           "cg_conv_destroy", "cg_conv_info", "cg_last_error", "cg_small_cin_conv", "cg_conv7x7s2_maxpool", "cg_pointwise_conv",
           "cg_maxpool3x3s2", "cg_avgpool_fc")

_pf = C.POINTER(C.c_float)
_pi = C.POINTER(C.c_int32)


class cg_conv_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("n_max", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("c_in", C.c_int32), ("c_out", C.c_int32),
        ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
        ("c_base", C.c_int32), ("in_dtype", C.c_int32), ("out_dtype", C.c_int32),
        ("epilogue", C.c_uint32), ("variant", C.c_int32), ("groups", C.c_int32),
        ("x_pixel_stride", C.c_int64),
        ("w_base", C.c_void_p), ("w_cond", C.c_void_p),
        ("gate_mean", _pf), ("gate_var", _pf), ("delta", _pf), ("delta_hi", _pf),
        ("gate_eps", C.c_float), ("shuffle", C.c_int32),
        ("gate_thr_i32", _pi),
        ("scale0", _pf), ("shift0", _pf), ("scale1", _pf), ("shift1", _pf),
        ("rq_mult0", _pi), ("rq_mult1", _pi), ("rq_bias", _pi),
        ("rq_shift", C.c_int32), ("rq_res_mult", C.c_int32),
        ("tau_c", C.c_float), ("tile_hint", C.c_int32),
        ("packed", C.c_void_p), ("packed_bytes", C.c_size_t),
    ]


_lib.cg_conv_packed_bytes.argtypes = [C.POINTER(cg_conv_desc)]
_lib.cg_conv_packed_bytes.restype = C.c_size_t
_lib.cg_conv_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(cg_conv_desc), C.c_void_p]
_lib.cg_conv_create.restype = C.c_int
_lib.cg_conv_workspace_bytes.argtypes = [C.c_void_p, C.c_int32]
_lib.cg_conv_workspace_bytes.restype = C.c_size_t
_lib.cg_conv_forward.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.cg_conv_forward.restype = C.c_int
_lib.cg_conv_forward_noalloc.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
_lib.cg_conv_forward_noalloc.restype = C.c_int
_lib.cg_conv_destroy.argtypes = [C.c_void_p]
_lib.cg_conv_destroy.restype = None
_lib.cg_conv_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
_lib.cg_conv_info.restype = C.c_int
_lib.cg_last_error.argtypes = []
_lib.cg_last_error.restype = C.c_char_p
_lib.cg_small_cin_conv.argtypes = [C.c_void_p] * 5 + [C.c_int32] * 9 + [C.c_void_p]
_lib.cg_small_cin_conv.restype = C.c_int
_lib.cg_conv7x7s2_maxpool.argtypes = [C.c_void_p] * 5 + [C.c_int32] * 6 + [C.c_void_p]
_lib.cg_conv7x7s2_maxpool.restype = C.c_int
_lib.cg_pointwise_conv.argtypes = [C.c_void_p] * 5 + [C.c_int32] * 7 + [C.c_void_p]
_lib.cg_pointwise_conv.restype = C.c_int
_lib.cg_maxpool3x3s2.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int32] * 4 + [C.c_void_p]
_lib.cg_maxpool3x3s2.restype = C.c_int
_lib.cg_avgpool_fc.argtypes = [C.c_void_p] * 4 + [C.c_int32] * 4 + [C.c_void_p]
_lib.cg_avgpool_fc.restype = C.c_int


class CGError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("cg_conv error %d: %s" % (code, text))
        self.code = code


def cg_last_error() -> str:
    return _lib.cg_last_error().decode()


def cg_conv_packed_bytes(desc: cg_conv_desc) -> int:
    return int(_lib.cg_conv_packed_bytes(C.byref(desc)))


def cg_conv_create(desc: cg_conv_desc, hip_stream: int = 0) -> int:
    """Returns the opaque handle (an integer address); raises CGError on failure."""
    h = C.c_void_p()
    rc = _lib.cg_conv_create(C.byref(h), C.byref(desc), C.c_void_p(hip_stream))
    if rc != CG_OK:
        raise CGError(rc, cg_last_error())
    return h.value


def cg_conv_workspace_bytes(handle: int, n: int) -> int:
    return int(_lib.cg_conv_workspace_bytes(C.c_void_p(handle), n))


def cg_conv_forward(handle: int, n: int, x: int, residual: int, y: int, bitmap: int, counts: int,
                    workspace: int, workspace_bytes: int, hip_stream: int = 0) -> None:
    """All tensor arguments are raw device addresses (0 = NULL)."""
    rc = _lib.cg_conv_forward(C.c_void_p(handle), n, C.c_void_p(x), C.c_void_p(residual), C.c_void_p(y),
                              C.c_void_p(bitmap), C.c_void_p(counts), C.c_void_p(workspace), workspace_bytes,
                              C.c_void_p(hip_stream))
    if rc != CG_OK:
        raise CGError(rc, cg_last_error())


def cg_conv_forward_noalloc(handle: int, n: int, x: int, residual: int, y: int, bitmap: int, counts: int,
                            hip_stream: int = 0) -> None:
    """cg_conv_forward without a workspace: the library's own fixed scratch array is used."""
    rc = _lib.cg_conv_forward_noalloc(C.c_void_p(handle), n, C.c_void_p(x), C.c_void_p(residual), C.c_void_p(y),
                                      C.c_void_p(bitmap), C.c_void_p(counts), C.c_void_p(hip_stream))
    if rc != CG_OK:
        raise CGError(rc, cg_last_error())


def cg_conv_destroy(handle: Optional[int]) -> None:
    _lib.cg_conv_destroy(C.c_void_p(handle))


def _check(rc: int) -> None:
    if rc != CG_OK:
        raise CGError(rc, cg_last_error())


def cg_small_cin_conv(x: int, w: int, scale: int, shift: int, y: int, n: int, h: int, wd: int, c_in: int,
                      c_out: int, k: int, stride: int, pad: int, relu: bool, hip_stream: int = 0) -> None:
    """Raw device addresses (0 = NULL for scale / shift)."""
    _check(_lib.cg_small_cin_conv(C.c_void_p(x), C.c_void_p(w), C.c_void_p(scale), C.c_void_p(shift), C.c_void_p(y),
                                  n, h, wd, c_in, c_out, k, stride, pad, int(bool(relu)), C.c_void_p(hip_stream)))


def cg_conv7x7s2_maxpool(x: int, w: int, scale: int, shift: int, y: int, n: int, h: int, wd: int, c_out: int,
                         pad: int, relu: bool, hip_stream: int = 0) -> None:
    _check(_lib.cg_conv7x7s2_maxpool(C.c_void_p(x), C.c_void_p(w), C.c_void_p(scale), C.c_void_p(shift), C.c_void_p(y),
                                     n, h, wd, c_out, pad, int(bool(relu)), C.c_void_p(hip_stream)))


def cg_pointwise_conv(x: int, w: int, scale: int, shift: int, y: int, n: int, h: int, wd: int, c_in: int, c_out: int,
                      stride: int, relu: bool, hip_stream: int = 0) -> None:
    _check(_lib.cg_pointwise_conv(C.c_void_p(x), C.c_void_p(w), C.c_void_p(scale), C.c_void_p(shift), C.c_void_p(y),
                                  n, h, wd, c_in, c_out, stride, int(bool(relu)), C.c_void_p(hip_stream)))


def cg_maxpool3x3s2(x: int, y: int, n: int, h: int, wd: int, c: int, hip_stream: int = 0) -> None:
    _check(_lib.cg_maxpool3x3s2(C.c_void_p(x), C.c_void_p(y), n, h, wd, c, C.c_void_p(hip_stream)))


def cg_avgpool_fc(x: int, wfc: int, bias: int, logits: int, n: int, hw: int, c: int, classes: int,
                  hip_stream: int = 0) -> None:
    _check(_lib.cg_avgpool_fc(C.c_void_p(x), C.c_void_p(wfc), C.c_void_p(bias), C.c_void_p(logits), n, hw, c, classes,
                              C.c_void_p(hip_stream)))


def cg_conv_info(handle: int):
    ho, wo = C.c_int32(), C.c_int32()
    v = _lib.cg_conv_info(C.c_void_p(handle), C.byref(ho), C.byref(wo))
    return v, ho.value, wo.value


# ----------------------------------------------------------------------------
# Convenience wrapper: fills the descriptor from numpy / torch objects and keeps the
# device buffers alive.  Still marshalling only.
# ----------------------------------------------------------------------------

def _host_f32(a, c_out):
    if a is None:
        return None
    v = np.ascontiguousarray(np.broadcast_to(np.asarray(a, dtype=np.float32), (c_out,)))
    return v


def _host_i32(a, c_out):
    if a is None:
        return None
    return np.ascontiguousarray(np.broadcast_to(np.asarray(a, dtype=np.int32), (c_out,)))


_TORCH_IN = {CG_F32: "float32", CG_BF16: "bfloat16", CG_I8: "int8"}
_TORCH_OUT = {CG_F32: "float32", CG_BF16: "bfloat16", CG_I8: "int8", CG_I32: "int32"}


class GatedConv:
    """One gated layer on the current torch device.

    w_base / w_cond: torch device tensors [C_out,kh,kw,C_base] / [C_out,kh,kw,C_in-C_base] in the
    input dtype (bf16 tensors for CG_BF16, int8 for CG_I8, float32 for CG_F32).
    groups > 1 selects channel grouping, shuffle the channel-shuffled store, tau_c > 0 the
    channel-wise gate (see cg_conv.h).
    """

    def __init__(self, *, n_max, h, w, c_in, c_out, c_base, w_base, w_cond, in_dtype, out_dtype,
                 kh=3, kw=3, stride=1, pad=1, epilogue=CG_EPI_RELU, variant=CG_VARIANT_AUTO,
                 gate_mean=None, gate_var=None, delta=None, delta_hi=None, gate_eps=0.0, gate_thr_i32=None,
                 scale0=None, shift0=None, scale1=None, shift1=None,
                 rq_mult0=None, rq_mult1=None, rq_bias=None, rq_shift=0, rq_res_mult=0,
                 x_pixel_stride=0, groups=0, shuffle=False, tau_c=0.0, tile_hint=0, stream=None):
        import torch
        self._torch = torch
        self.handle = None
        d = cg_conv_desc()
        d.struct_size = C.sizeof(cg_conv_desc)
        d.n_max, d.h, d.w, d.c_in, d.c_out = n_max, h, w, c_in, c_out
        d.kh, d.kw, d.stride, d.pad, d.c_base = kh, kw, stride, pad, c_base
        d.in_dtype, d.out_dtype, d.epilogue, d.variant = in_dtype, out_dtype, epilogue, variant
        d.x_pixel_stride = x_pixel_stride
        d.groups, d.shuffle = int(groups), int(bool(shuffle))
        d.tau_c = float(tau_c)
        d.tile_hint = int(tile_hint)
        self._keep = [w_base, w_cond]
        d.w_base = w_base.data_ptr()
        d.w_cond = w_cond.data_ptr() if (w_cond is not None and w_cond.numel()) else None
        host = {}
        for name, val, conv, ptype in (
                ("gate_mean", gate_mean, _host_f32, _pf), ("gate_var", gate_var, _host_f32, _pf),
                ("delta", delta, _host_f32, _pf), ("delta_hi", delta_hi, _host_f32, _pf),
                ("scale0", scale0, _host_f32, _pf), ("shift0", shift0, _host_f32, _pf),
                ("scale1", scale1, _host_f32, _pf), ("shift1", shift1, _host_f32, _pf),
                ("gate_thr_i32", gate_thr_i32, _host_i32, _pi), ("rq_mult0", rq_mult0, _host_i32, _pi),
                ("rq_mult1", rq_mult1, _host_i32, _pi), ("rq_bias", rq_bias, _host_i32, _pi)):
            arr = conv(val, c_out)
            host[name] = arr
            if arr is not None:
                setattr(d, name, arr.ctypes.data_as(ptype))
        d.gate_eps = gate_eps
        d.rq_shift, d.rq_res_mult = rq_shift, rq_res_mult
        need = cg_conv_packed_bytes(d)
        if need == 0:
            code = CG_EINVAL
            # distinguish unsupported from invalid through create's status
            d.packed, d.packed_bytes = None, 0
            h_ = C.c_void_p()
            code = _lib.cg_conv_create(C.byref(h_), C.byref(d), None)
            raise CGError(code, cg_last_error())
        dev = w_base.device
        self.packed = torch.empty(need + 256, dtype=torch.uint8, device=dev)
        base = self.packed.data_ptr()
        d.packed = (base + 255) & ~255
        d.packed_bytes = need
        self.stream = stream
        sptr = self._stream_ptr()
        self.handle = cg_conv_create(d, sptr)
        self.desc = d
        self.variant, self.ho, self.wo = cg_conv_info(self.handle)
        self.n_max, self.c_out, self.out_dtype = n_max, c_out, out_dtype
        self.words = (c_out + 31) // 32
        self._ws = None

    def _stream_ptr(self):
        s = self.stream if self.stream is not None else self._torch.cuda.current_stream()
        return s.cuda_stream

    def forward(self, x, residual=None, y=None, bitmap=True, counts=True):
        """x: torch device tensor [n,H,W,C_in] (contiguous NHWC).  Returns (y, bitmap, counts)."""
        torch = self._torch
        n = x.shape[0]
        dev = x.device
        if y is None:
            y = torch.empty((n, self.ho, self.wo, self.c_out), dtype=getattr(torch, _TORCH_OUT[self.out_dtype]),
                            device=dev)
        if bitmap is True:
            bitmap = torch.empty((n * self.ho * self.wo, self.words), dtype=torch.int32, device=dev)
        elif bitmap is False:
            bitmap = None
        if counts is True:
            counts = torch.empty(2 + n * self.c_out, dtype=torch.int32, device=dev)
        elif counts is False:
            counts = None
        need = cg_conv_workspace_bytes(self.handle, n)
        ws_ptr = 0
        if need:
            if self._ws is None or self._ws.numel() < need + 256:
                self._ws = torch.empty(need + 256, dtype=torch.uint8, device=dev)
            ws_ptr = (self._ws.data_ptr() + 255) & ~255
        cg_conv_forward(self.handle, n, x.data_ptr(), residual.data_ptr() if residual is not None else 0,
                        y.data_ptr(), bitmap.data_ptr() if bitmap is not None else 0,
                        counts.data_ptr() if counts is not None else 0, ws_ptr, need, self._stream_ptr())
        return y, bitmap, counts

    def close(self):
        if self.handle:
            cg_conv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
