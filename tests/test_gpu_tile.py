"""GPU parity of the large-tile matrix-core kernel against the CPU oracle, through the C ABI:
every tile shape the library can pick (forced with the descriptor's tile_hint), 1x1 layers,
fully connected layers (h = w = k = 1, Sec. 3.1 footnote of the paper), degenerate output sizes,
one-chunk channel groups, tiles with more fired pixels than one conditional pass takes."""
import numpy as np
import pytest
import torch

from oracle import cg_oracle as O
from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu

TILE = B.CG_VARIANT_TILE


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


def hint(fp=0, wn=0, cps=0):
    return fp | (wn << 4) | (cps << 8)


FORCED = [
    W.LayerShape("t_64@56", 2, 56, 56, 64, 64),
    W.LayerShape("t_128@28", 3, 28, 28, 128, 128),
    W.LayerShape("t_256@14", 3, 14, 14, 256, 256),
    W.LayerShape("t_512@7", 5, 7, 7, 512, 512),
    W.LayerShape("t_128>256@28s2", 2, 28, 28, 128, 256, stride=2),
    W.LayerShape("t_ragged_19x23", 2, 19, 23, 64, 128),
    W.LayerShape("t_1x1", 2, 14, 14, 128, 128, pad=0, k=1),
]
SHAPES_OF_TILE = [(fp, wn) for fp in (4, 2, 1) for wn in (1, 2)]


def _run_both(shape, tile_hint, tag, rho=0.3):
    """bf16 (fp32 and bf16 outputs, a partial batch) and int8; returns the number of cases that ran."""
    ran = 0
    try:
        inp = W.make_inputs(shape, 1000 + shape.c_out + shape.h, kind="coherent", rho=rho, round_bf16=True)
        gate = W.calibrate_gate(inp, rho, sample_images=None)
        rep = _say(P.run_float(inp, gate, out_dtype=B.CG_F32, variant=TILE, tile_hint=tile_hint, name=tag + " bf16"))
        assert rep.variant == TILE
        _say(P.run_float(inp, gate, out_dtype=B.CG_BF16, variant=TILE, tile_hint=tile_hint, name=tag + " bf16 out",
                         n_run=max(1, shape.n - 1)))
        ran += 1
    except B.CGError as e:
        assert e.code == B.CG_EUNSUPPORTED      # a hint the shape cannot take
    if shape.c_base % 16 == 0:
        try:
            q = W.quantize_int8(W.make_inputs(shape, 2000 + shape.c_out + shape.h, kind="coherent", rho=0.35))
            thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
            rep = _say(P.run_int8(q, thr, variant=TILE, tile_hint=tile_hint, name=tag + " int8"))
            assert rep.variant == TILE
            ran += 1
        except B.CGError as e:
            assert e.code == B.CG_EUNSUPPORTED
    return ran


@pytest.mark.parametrize("fp,wn", SHAPES_OF_TILE, ids=["fp%d_wn%d" % c for c in SHAPES_OF_TILE])
def test_every_tile_shape(fp, wn):
    ran = 0
    for shape in FORCED:
        ran += _run_both(shape, hint(fp, wn), "%s fp=%d wn=%d" % (shape.name, fp, wn))
    assert ran >= 4          # most shapes take most tile shapes


@pytest.mark.parametrize("cps", [4, 1])
def test_stage_widths_of_3x3_layers(cps):
    """Stages of four 16-byte channel chunks, and of one (two taps share a K step)."""
    ran = 0
    for shape in (FORCED[1], FORCED[2], W.LayerShape("t_g8", 2, 14, 14, 64, 64, groups=8)):
        ran += _run_both(shape, hint(cps=cps), "%s cps=%d" % (shape.name, cps))
    assert ran >= 2


ONE_BY_ONE = [
    W.LayerShape("fc_512>1024_n64", 64, 1, 1, 512, 1024, pad=0, k=1),       # fully connected, batch 64
    W.LayerShape("fc_256>64_n130", 130, 1, 1, 256, 64, pad=0, k=1),         # ragged last row of the flat walk
    W.LayerShape("pw_256>256@14", 4, 14, 14, 256, 256, pad=0, k=1),         # MobileNet pointwise layer
    W.LayerShape("pw_128>256@9x11", 3, 9, 11, 128, 256, pad=0, k=1),
    W.LayerShape("pw_s2_128>128@14", 2, 14, 14, 128, 128, stride=2, pad=0, k=1),
    W.LayerShape("pw_g2_64>128@7", 5, 7, 7, 64, 128, pad=0, k=1, groups=2),
]


@pytest.mark.parametrize("shape", ONE_BY_ONE, ids=[s.name for s in ONE_BY_ONE])
def test_gated_1x1_and_fully_connected(shape):
    for variant in (B.CG_VARIANT_AUTO, TILE):
        inp = W.make_inputs(shape, 3000 + shape.c_out + shape.n, kind="iid", rho=0.3, round_bf16=True)
        gate = W.calibrate_gate(inp, 0.30, sample_images=None)
        rep = _say(P.run_float(inp, gate, variant=variant, name=shape.name + " bf16"))
        assert rep.variant == TILE and 0.1 < rep.fired_frac < 0.6
        q = W.quantize_int8(W.make_inputs(shape, 3100 + shape.c_out + shape.n, kind="iid", rho=0.35))
        thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
        rep = _say(P.run_int8(q, thr, variant=variant, name=shape.name + " int8"))
        assert rep.variant == TILE
    # a batch of one (the statistics of the gate come from the whole batch above)
    _say(P.run_float(inp, gate, variant=TILE, n_run=1, name=shape.name + " bf16 n=1"))
    _say(P.run_int8(q, thr, variant=TILE, n_run=1, name=shape.name + " int8 n=1"))


DEGENERATE = [
    W.LayerShape("d_3x3_pad0", 5, 3, 3, 64, 64, pad=0),           # Ho = Wo = 1
    W.LayerShape("d_1x1_pad1", 7, 1, 1, 64, 128),                 # a 1x1 image: only the centre tap is inside
    W.LayerShape("d_20x3_pad0", 3, 20, 3, 64, 64, pad=0),         # Wo = 1
    W.LayerShape("d_3x20_pad0", 3, 3, 20, 128, 64, pad=0),        # Ho = 1
    W.LayerShape("d_2x2_s2", 4, 2, 2, 64, 64, stride=2),          # Ho = Wo = 1 with stride 2
]


@pytest.mark.parametrize("variant", [B.CG_VARIANT_MFMA_ROWS, TILE], ids=["rows", "tile"])
@pytest.mark.parametrize("shape", DEGENERATE, ids=[s.name for s in DEGENERATE])
def test_output_height_or_width_of_one(shape, variant):
    """Division by an output size of one inside the kernels (the reciprocal does not fit 32 bits)."""
    inp = W.make_inputs(shape, 4000 + shape.h * 7 + shape.w, kind="iid", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    try:
        rep = _say(P.run_float(inp, gate, variant=variant, name=shape.name + " bf16"))
    except B.CGError as e:
        assert e.code == B.CG_EUNSUPPORTED
        pytest.skip("shape outside this kernel family")
    assert rep.variant == variant
    q = W.quantize_int8(W.make_inputs(shape, 4100 + shape.h * 7 + shape.w, kind="iid", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    _say(P.run_int8(q, thr, variant=variant, name=shape.name + " int8"))


def test_more_fired_pixels_than_one_conditional_pass():
    """Every gate fires: each tile walks the conditional stages twice (a pass takes half a tile's pixels)."""
    shape = W.LayerShape("t_allfire", 2, 28, 28, 128, 128)
    inp = W.make_inputs(shape, 5000, kind="iid", round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    for frac, delta in ((1.0, -np.inf), (0.8, None)):
        g = gate
        if delta is not None:
            g.delta[:] = delta
        else:
            g = W.calibrate_gate(inp, 0.8, sample_images=None)
        for fp in (4, 2, 1):
            rep = _say(P.run_float(inp, g, variant=TILE, tile_hint=hint(fp, 1), name="fired %.1f fp=%d" % (frac, fp)))
            assert abs(rep.fired_frac - frac) < 0.05
    q = W.quantize_int8(W.make_inputs(shape, 5001, kind="iid"))
    thr = np.full(128, np.iinfo(np.int32).min, np.int32)
    rep = _say(P.run_int8(q, thr, variant=TILE, tile_hint=hint(4, 1), name="int8 all fire"))
    assert rep.fired_frac == 1.0


def test_tile_epilogues_strided_input_and_repeatability():
    shape = W.LayerShape("t_epi", 3, 14, 14, 128, 128)
    inp = W.make_inputs(shape, 6100, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    rng = np.random.default_rng(61)
    aff = dict(scale0=rng.uniform(0.5, 1.5, 128), shift0=rng.normal(0, 0.1, 128),
               scale1=rng.uniform(0.5, 1.5, 128), shift1=rng.normal(0, 0.1, 128))
    res = rng.standard_normal((3, 14, 14, 128)).astype(np.float32)
    for out_dtype in (B.CG_F32, B.CG_BF16):
        _say(P.run_float(inp, gate, out_dtype=out_dtype, variant=TILE, affine=aff, residual=res,
                         epilogue=B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL, name="tile epilogue out=%d" % out_dtype))
    _say(P.run_float(inp, gate, variant=TILE, delta_hi=gate.delta + 0.8, name="tile two-sided gate"))
    # x in a buffer with 160 elements per pixel of which the first 128 are the layer's channels; two calls
    wide = torch.full((3, 14, 14, 160), 7.0, dtype=torch.bfloat16, device="cuda")
    wide[..., :128] = torch.from_numpy(inp.x).cuda().to(torch.bfloat16)
    layer = B.GatedConv(n_max=3, h=14, w=14, c_in=128, c_out=128, c_base=32, x_pixel_stride=160, variant=TILE,
                        w_base=torch.from_numpy(inp.w_base).cuda().to(torch.bfloat16),
                        w_cond=torch.from_numpy(inp.w_cond).cuda().to(torch.bfloat16), in_dtype=B.CG_BF16,
                        out_dtype=B.CG_F32, gate_mean=gate.mean, gate_var=gate.var, delta=gate.delta)
    a = [t.clone() for t in layer.forward(wide)]
    b = layer.forward(wide)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    f32 = lambda v: np.asarray(v, np.float32).astype(np.float64)
    ref = O.forward_float(inp.x, inp.w_base, inp.w_cond, gate_mean=f32(gate.mean), gate_var=f32(gate.var),
                          delta=f32(gate.delta), want_partials=False)
    _say(P.compare_float("tile strided input", a[0].cpu().numpy().astype(np.float64), a[1].cpu().numpy().view(np.uint32),
                         a[2].cpu().numpy().view(np.uint32), ref, 128, B.CG_F32, layer.variant))
    layer.close()
