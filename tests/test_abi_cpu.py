"""Host-side tests of the C ABI that need no GPU: the library loads, exports what the
header declares, and rejects bad arguments before touching HIP."""
import ctypes as C
import re
from pathlib import Path

import numpy as np
import pytest

from paper_1805_12549_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "cg_conv.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cg_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(B._lib, n) is not None


def make_desc(**over):
    d = B.cg_conv_desc()
    d.struct_size = C.sizeof(B.cg_conv_desc)
    d.n_max, d.h, d.w, d.c_in, d.c_out = 2, 8, 8, 16, 32
    d.kh = d.kw = 3
    d.stride, d.pad, d.c_base = 1, 1, 4
    d.in_dtype, d.out_dtype = B.CG_BF16, B.CG_F32
    d.epilogue = B.CG_EPI_RELU
    d.w_base, d.w_cond = 0x1000, 0x2000      # never dereferenced by validation
    keep = {}
    for name in ("gate_mean", "gate_var", "delta"):
        keep[name] = np.ones(32, np.float32)
        setattr(d, name, keep[name].ctypes.data_as(C.POINTER(C.c_float)))
    keep["thr"] = np.zeros(32, np.int32)
    d.gate_thr_i32 = keep["thr"].ctypes.data_as(C.POINTER(C.c_int32))
    for k, v in over.items():
        setattr(d, k, v)
    d._keep = keep
    return d


def test_valid_descriptor_sizes_packed_buffer():
    d = make_desc()
    need = B.cg_conv_packed_bytes(d)
    # at least the weights themselves
    assert need >= 32 * 9 * 16 * 2


@pytest.mark.parametrize("over,code", [
    (dict(struct_size=8), B.CG_EINVAL),
    (dict(n_max=0), B.CG_EINVAL),
    (dict(c_out=-1), B.CG_EINVAL),
    (dict(c_base=0), B.CG_EINVAL),
    (dict(c_base=17), B.CG_EINVAL),
    (dict(stride=0), B.CG_EINVAL),
    (dict(pad=-1), B.CG_EINVAL),
    (dict(kh=5, kw=5), B.CG_EUNSUPPORTED),
    (dict(kh=3, kw=1), B.CG_EUNSUPPORTED),
    (dict(in_dtype=7), B.CG_EINVAL),
    (dict(out_dtype=B.CG_I8), B.CG_EINVAL),
    (dict(in_dtype=B.CG_I8, out_dtype=B.CG_F32), B.CG_EINVAL),
    (dict(in_dtype=B.CG_I8, out_dtype=B.CG_I8, rq_shift=40), B.CG_EINVAL),
    (dict(epilogue=64), B.CG_EINVAL),
    (dict(variant=9), B.CG_EINVAL),
    (dict(x_pixel_stride=8), B.CG_EINVAL),
    (dict(w_base=None), B.CG_EINVAL),
    (dict(w_cond=None), B.CG_EINVAL),
    (dict(h=1, w=1, pad=0), B.CG_EINVAL),
    (dict(in_dtype=B.CG_F32, variant=B.CG_VARIANT_TILE), B.CG_EUNSUPPORTED),
    (dict(in_dtype=B.CG_F32, variant=B.CG_VARIANT_MFMA_ROWS), B.CG_EUNSUPPORTED),
    (dict(variant=2), B.CG_EINVAL),                     # retired kernel families
    (dict(variant=3), B.CG_EINVAL),
    (dict(groups=-1), B.CG_EINVAL),
    (dict(groups=2), B.CG_EINVAL),                      # c_base * groups != c_in
    (dict(groups=4, c_out=30), B.CG_EINVAL),            # groups does not divide c_out
    (dict(shuffle=1), B.CG_EINVAL),                     # shuffle without grouping
    (dict(groups=4, shuffle=2), B.CG_EINVAL),
    (dict(tau_c=-0.1), B.CG_EINVAL),
    (dict(tau_c=float("nan")), B.CG_EINVAL),
    (dict(tau_c=float("inf")), B.CG_EINVAL),
    (dict(tile_hint=1 << 12), B.CG_EINVAL),
    (dict(tile_hint=-1), B.CG_EINVAL),
])
def test_invalid_descriptors_are_rejected_without_a_gpu(over, code):
    d = make_desc(**over)
    assert B.cg_conv_packed_bytes(d) == 0
    h = C.c_void_p()
    rc = B._lib.cg_conv_create(C.byref(h), C.byref(d), None)
    assert rc == code, B.cg_last_error()
    assert h.value is None
    assert len(B.cg_last_error()) > 0


def test_grouped_descriptor_is_accepted():
    assert B.cg_conv_packed_bytes(make_desc(groups=4)) > 0
    assert B.cg_conv_packed_bytes(make_desc(groups=4, shuffle=1)) > 0
    assert B.cg_conv_packed_bytes(make_desc(groups=1)) == B.cg_conv_packed_bytes(make_desc())
    assert B.cg_conv_packed_bytes(make_desc(tau_c=0.25)) == B.cg_conv_packed_bytes(make_desc())


def test_missing_gate_statistics_and_nan():
    d = make_desc()
    d.delta = None
    assert B.cg_conv_packed_bytes(d) == 0
    d = make_desc()
    d._keep["gate_var"][3] = np.nan
    assert B.cg_conv_packed_bytes(d) == 0 and "channel 3" in B.cg_last_error()
    d = make_desc()
    d._keep["gate_var"][5] = -1.0
    assert B.cg_conv_packed_bytes(d) == 0 and "negative" in B.cg_last_error()
    d = make_desc(in_dtype=B.CG_I8, out_dtype=B.CG_I32)
    d.gate_thr_i32 = None
    assert B.cg_conv_packed_bytes(d) == 0


def test_packed_buffer_checks_precede_hip():
    d = make_desc()
    need = B.cg_conv_packed_bytes(d)
    h = C.c_void_p()
    d.packed, d.packed_bytes = None, need
    assert B._lib.cg_conv_create(C.byref(h), C.byref(d), None) == B.CG_EINVAL
    d.packed, d.packed_bytes = 0x10000, need - 1
    assert B._lib.cg_conv_create(C.byref(h), C.byref(d), None) == B.CG_EINVAL
    d.packed, d.packed_bytes = 0x10001, need
    assert B._lib.cg_conv_create(C.byref(h), C.byref(d), None) == B.CG_EINVAL
    assert "aligned" in B.cg_last_error()
    assert B._lib.cg_conv_create(None, C.byref(d), None) == B.CG_EINVAL


def test_null_handle_paths():
    B.cg_conv_destroy(None)
    assert B._lib.cg_conv_workspace_bytes(None, 1) == 0
    assert B._lib.cg_conv_info(None, None, None) == -1
    rc = B._lib.cg_conv_forward(None, 1, None, None, None, None, None, None, 0, None)
    assert rc == B.CG_EINVAL
    assert isinstance(B.cg_last_error(), str)


def test_dense_ops_validate_without_a_gpu():
    """cg_small_cin_conv / cg_maxpool3x3s2 / cg_avgpool_fc check their arguments before any HIP call."""
    for call, code in (
            (lambda: B.cg_small_cin_conv(0, 16, 0, 0, 16, 1, 8, 8, 3, 64, 7, 2, 3, True), B.CG_EINVAL),
            (lambda: B.cg_small_cin_conv(16, 16, 0, 0, 16, 1, 8, 8, 5, 64, 3, 1, 1, True), B.CG_EUNSUPPORTED),
            (lambda: B.cg_small_cin_conv(16, 16, 0, 0, 16, 1, 8, 8, 3, 48, 3, 1, 1, True), B.CG_EUNSUPPORTED),
            (lambda: B.cg_small_cin_conv(16, 16, 0, 0, 16, 1, 8, 8, 3, 64, 4, 1, 1, True), B.CG_EUNSUPPORTED),
            (lambda: B.cg_small_cin_conv(16, 16, 0, 0, 16, 1, 2, 2, 3, 64, 7, 2, 1, True), B.CG_EINVAL),
            (lambda: B.cg_small_cin_conv(16, 16, 0, 0, 17, 1, 8, 8, 3, 64, 3, 1, 1, True), B.CG_EINVAL),
            (lambda: B.cg_conv7x7s2_maxpool(16, 0, 0, 0, 16, 1, 32, 32, 64, 3, True), B.CG_EINVAL),
            (lambda: B.cg_conv7x7s2_maxpool(16, 16, 0, 0, 16, 1, 32, 32, 48, 3, True), B.CG_EUNSUPPORTED),
            (lambda: B.cg_conv7x7s2_maxpool(16, 16, 0, 0, 16, 1, 2, 2, 64, 1, True), B.CG_EINVAL),
            (lambda: B.cg_conv7x7s2_maxpool(16, 16, 0, 0, 16, 1, 32, 32, 64, 7, True), B.CG_EINVAL),
            (lambda: B.cg_pointwise_conv(16, 16, 0, 0, 0, 1, 8, 8, 64, 64, 2, False), B.CG_EINVAL),
            (lambda: B.cg_pointwise_conv(16, 16, 0, 0, 16, 1, 8, 8, 24, 64, 2, False), B.CG_EUNSUPPORTED),
            (lambda: B.cg_pointwise_conv(16, 16, 0, 0, 16, 1, 8, 8, 1024, 64, 2, False), B.CG_EUNSUPPORTED),
            (lambda: B.cg_pointwise_conv(16, 16, 0, 0, 16, 1, 8, 8, 64, 96, 2, False), B.CG_EUNSUPPORTED),
            (lambda: B.cg_pointwise_conv(16, 16, 0, 0, 16, 1, 8, 8, 64, 64, 0, False), B.CG_EINVAL),
            (lambda: B.cg_pointwise_conv(16, 16, 8, 0, 16, 1, 8, 8, 64, 64, 2, False), B.CG_EINVAL),
            (lambda: B.cg_maxpool3x3s2(16, 0, 1, 8, 8, 8), B.CG_EINVAL),
            (lambda: B.cg_maxpool3x3s2(16, 16, 1, 8, 8, 12), B.CG_EUNSUPPORTED),
            (lambda: B.cg_maxpool3x3s2(16, 16, 1, 0, 8, 8), B.CG_EINVAL),
            (lambda: B.cg_avgpool_fc(16, 0, 0, 16, 1, 4, 8, 2), B.CG_EINVAL),
            (lambda: B.cg_avgpool_fc(16, 16, 0, 16, 1, 0, 8, 2), B.CG_EINVAL),
            (lambda: B.cg_avgpool_fc(16, 16, 0, 16, 1, 4, 20000, 2), B.CG_EUNSUPPORTED)):
        with pytest.raises(B.CGError) as e:
            call()
        assert e.value.code == code, B.cg_last_error()
    # zero images: accepted, nothing to do
    B.cg_small_cin_conv(16, 16, 0, 0, 16, 0, 8, 8, 3, 64, 7, 2, 3, True)
    B.cg_pointwise_conv(16, 16, 0, 0, 16, 0, 8, 8, 64, 64, 2, False)
    B.cg_conv7x7s2_maxpool(16, 16, 0, 0, 16, 0, 32, 32, 64, 3, True)
    B.cg_maxpool3x3s2(16, 16, 0, 8, 8, 8)
    B.cg_avgpool_fc(16, 16, 0, 16, 0, 4, 8, 2)
