"""GPU parity of the channel-wise gate (an image's output channel keeps its conditional path only
if at least a fraction tau_c of its activations fired) against the CPU oracle, through the C ABI:
plain and row-tiled kernels, bf16 and int8, with and without grouping, counts and bitmap after
the gate."""
import numpy as np
import pytest

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


SHAPES = [
    W.LayerShape("cg_128@28", 3, 28, 28, 128, 128),
    W.LayerShape("cg_256@14", 5, 14, 14, 256, 256),       # tiles straddle images
    W.LayerShape("cg_512@7", 9, 7, 7, 512, 512),          # several images per tile
    W.LayerShape("cg_128>256@28s2", 2, 28, 28, 128, 256, stride=2),
]


@pytest.mark.parametrize("variant", [B.CG_VARIANT_NAIVE, B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE],
                         ids=["plain", "rows", "tile"])
@pytest.mark.parametrize("shape", SHAPES, ids=[s.name for s in SHAPES])
def test_channel_gate_int8_bit_exact(shape, variant):
    q = W.quantize_int8(W.make_inputs(shape, 7000 + shape.c_out, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    fr = []
    for tau in (0.2, 0.35, 0.5, 0.9):
        rep = _say(P.run_int8(q, thr, variant=variant, tau_c=tau, name="%s int8 tau_c=%.2f" % (shape.name, tau)))
        assert rep.variant == variant
        fr.append(rep.fired_frac)
    assert fr[0] >= fr[1] >= fr[2] >= fr[3] and fr[0] > fr[3]      # the gate removes more as tau_c grows
    assert fr[0] > 0.05


@pytest.mark.parametrize("variant", [B.CG_VARIANT_NAIVE, B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE],
                         ids=["plain", "rows", "tile"])
@pytest.mark.parametrize("shape", SHAPES[:3], ids=[s.name for s in SHAPES[:3]])
def test_channel_gate_bf16(shape, variant):
    inp = W.make_inputs(shape, 7100 + shape.c_out, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    off = _say(P.run_float(inp, gate, variant=variant, name=shape.name + " bf16 tau_c=0"))
    for tau in (0.25, 0.4):
        rep = _say(P.run_float(inp, gate, variant=variant, tau_c=tau, out_dtype=B.CG_BF16,
                               name="%s bf16 tau_c=%.2f" % (shape.name, tau)))
        assert rep.variant == variant
        assert 0.02 < rep.fired_frac < off.fired_frac


def test_channel_gate_grouped_shuffled_with_epilogue():
    shape = W.LayerShape("cg_g_256@14", 3, 14, 14, 256, 256)
    rng = np.random.default_rng(5)
    q = W.quantize_int8(W.make_inputs(shape, 7200, kind="coherent", rho=0.35, grouped=True))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    rq = W.requant_params(q, rng)
    res = rng.integers(-128, 128, (shape.n, shape.ho, shape.wo, shape.c_out)).astype(np.int8)
    for variant in (B.CG_VARIANT_NAIVE, B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE):
        _say(P.run_int8(q, thr, variant=variant, tau_c=0.35, shuffle=True, out_i8=True, rq=rq, residual=res,
                        rq_res_mult=1 << 14, epilogue=B.CG_EPI_RESIDUAL | B.CG_EPI_RELU,
                        name="grouped shuffled requant tau_c=0.35 variant=%d" % variant))


def test_channel_gate_extremes():
    shape = SHAPES[0]
    q = W.quantize_int8(W.make_inputs(shape, 7300, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    base = _say(P.run_int8(q, thr, name="tau_c=0"))
    tiny = _say(P.run_int8(q, thr, tau_c=1e-6, name="tau_c=1e-6"))      # drops only channels that never fire
    assert tiny.fired_frac == base.fired_frac
    none = _say(P.run_int8(q, thr, tau_c=1.5, name="tau_c=1.5"))
    assert none.fired_frac == 0.0


def test_channel_gate_counts_without_bitmap_and_repeat():
    """Counts requested without a bitmap (the decisions then live in the workspace), called twice."""
    import torch
    shape = SHAPES[1]
    q = W.quantize_int8(W.make_inputs(shape, 7400, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    from oracle import cg_oracle as O
    ref = O.forward_int8(q.x, q.w_base, q.w_cond, thr, tau_c=float(np.float32(0.3)), want_partials=False)
    layer = B.GatedConv(n_max=shape.n, h=shape.h, w=shape.w, c_in=shape.c_in, c_out=shape.c_out, c_base=shape.c_base,
                        w_base=torch.from_numpy(q.w_base).cuda(), w_cond=torch.from_numpy(q.w_cond).cuda(),
                        in_dtype=B.CG_I8, out_dtype=B.CG_I32, gate_thr_i32=thr, tau_c=0.3)
    x = torch.from_numpy(q.x).cuda()
    for _ in range(2):
        y, bm, cnt = layer.forward(x, bitmap=False)
        torch.cuda.synchronize()
        assert bm is None
        assert np.array_equal(cnt.cpu().numpy().view(np.uint32), ref["counts"])
        assert np.array_equal(y.cpu().numpy(), ref["y"])
    layer.close()


SMALL_MAPS = [
    W.LayerShape("cg_cifar_512@4", 11, 4, 4, 512, 512),                      # 16 pixels per feature map
    W.LayerShape("cg_fc_256>512_n70", 70, 1, 1, 256, 512, pad=0, k=1),       # one pixel per map: a fully connected layer
    W.LayerShape("cg_pw_128>96@3", 9, 3, 3, 128, 96 + 32, pad=0, k=1),
]


@pytest.mark.parametrize("shape", SMALL_MAPS, ids=[s.name for s in SMALL_MAPS])
def test_counts_and_channel_gate_on_maps_of_a_few_pixels(shape):
    """Fired counts and the channel-wise gate where a feature map has at most 16 pixels (the counting
    kernel then walks a map per thread)."""
    q = W.quantize_int8(W.make_inputs(shape, 7300 + shape.c_out, kind="iid", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    for tau in (0.0, 0.3, 0.6, 1.0):
        rep = _say(P.run_int8(q, thr, tau_c=tau, name="%s int8 tau_c=%.2f" % (shape.name, tau)))
        assert rep.variant in (B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE)
    inp = W.make_inputs(shape, 7400 + shape.c_out, kind="iid", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    for tau in (0.0, 0.5):
        _say(P.run_float(inp, gate, tau_c=tau, name="%s bf16 tau_c=%.2f" % (shape.name, tau)))
