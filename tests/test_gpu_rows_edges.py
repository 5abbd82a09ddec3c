"""Edge cases of the row-tiled matrix-core kernel through the C ABI: partial batches, a large batch,
wide images, an input whose pixels are further apart than c_in, repeated calls."""
import numpy as np
import pytest
import torch

from oracle import cg_oracle as O
from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


@pytest.mark.parametrize("shape,n_run", [
    (W.LayerShape("pb_256@14", 5, 14, 14, 256, 256), 3),       # tiles straddle images, last tile ragged
    (W.LayerShape("pb_512@7", 9, 7, 7, 512, 512), 1),          # one image of nine
    (W.LayerShape("pb_128@28", 4, 28, 28, 128, 128), 3),
])
def test_partial_batch(shape, n_run):
    inp = W.make_inputs(shape, 8000 + shape.c_out, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    rep = _say(P.run_float(inp, gate, n_run=n_run, name="%s n=%d of %d" % (shape.name, n_run, shape.n)))
    assert rep.variant == B.CG_VARIANT_MFMA_ROWS
    q = W.quantize_int8(W.make_inputs(shape, 8100 + shape.c_out, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    _say(P.run_int8(q, thr, n_run=n_run, name="%s int8 n=%d" % (shape.name, n_run)))


def test_large_batch_and_wide_image():
    for shape in (W.LayerShape("big_128@28", 256, 28, 28, 128, 128), W.LayerShape("wide_64@112", 4, 112, 112, 64, 64),
                  W.LayerShape("tall_64", 2, 150, 20, 64, 128)):
        inp = W.make_inputs(shape, 8200 + shape.h, kind="coherent", rho=0.3, round_bf16=True)
        gate = W.calibrate_gate(inp, 0.30, sample_images=4)
        rep = _say(P.run_float(inp, gate, out_dtype=B.CG_BF16, name=shape.name))
        assert rep.variant == B.CG_VARIANT_MFMA_ROWS


def test_strided_input_pixels_and_repeatability():
    """x lives in a buffer with 160 elements per pixel of which the first 128 are the layer's channels."""
    shape = W.LayerShape("strided_128@14", 3, 14, 14, 128, 128)
    inp = W.make_inputs(shape, 8300, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    wide = torch.full((3, 14, 14, 160), 7.0, dtype=torch.bfloat16, device="cuda")
    wide[..., :128] = torch.from_numpy(inp.x).cuda().to(torch.bfloat16)
    layer = B.GatedConv(n_max=3, h=14, w=14, c_in=128, c_out=128, c_base=32, x_pixel_stride=160,
                        w_base=torch.from_numpy(inp.w_base).cuda().to(torch.bfloat16),
                        w_cond=torch.from_numpy(inp.w_cond).cuda().to(torch.bfloat16), in_dtype=B.CG_BF16,
                        out_dtype=B.CG_F32, gate_mean=gate.mean, gate_var=gate.var, delta=gate.delta)
    assert layer.variant == B.CG_VARIANT_MFMA_ROWS
    a = [t.clone() for t in layer.forward(wide)]
    b = layer.forward(wide)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    f32 = lambda v: np.asarray(v, np.float32).astype(np.float64)
    ref = O.forward_float(inp.x, inp.w_base, inp.w_cond, gate_mean=f32(gate.mean), gate_var=f32(gate.var),
                          delta=f32(gate.delta), want_partials=False)
    _say(P.compare_float("strided input", a[0].cpu().numpy().astype(np.float64), a[1].cpu().numpy().view(np.uint32),
                         a[2].cpu().numpy().view(np.uint32), ref, 128, B.CG_F32, layer.variant))
    layer.close()
