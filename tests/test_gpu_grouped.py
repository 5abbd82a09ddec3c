"""GPU parity of the channel-grouped layer (output group i takes input group i as its base path,
the other groups as its conditional path; optional channel-shuffled store) against the CPU oracle,
through the C ABI: the plain kernel on any shape and the row-tiled matrix-core kernel, both where a
64-channel block lies inside one group and where it covers several."""
import numpy as np
import pytest

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


GROUPED = [
    # 64 output channels per group or more: a block inside one group
    W.LayerShape("g_256@14", 3, 14, 14, 256, 256),
    W.LayerShape("g_512@7", 5, 7, 7, 512, 512),
    W.LayerShape("g_128>256@28s2", 2, 28, 28, 128, 256, stride=2),
    W.LayerShape("g_g2_64>128", 2, 14, 14, 64, 128, groups=2),
    # fewer: a block covers 2 or 4 groups
    W.LayerShape("g_128@28", 3, 28, 28, 128, 128),
    W.LayerShape("g_64@56", 2, 56, 56, 64, 64),
    W.LayerShape("g_64>128@56s2", 2, 56, 56, 64, 128, stride=2),
    W.LayerShape("g_g8_256>128", 2, 14, 14, 256, 128, groups=8),
    W.LayerShape("g_ragged_19x23", 2, 19, 23, 64, 64, groups=2),
]


@pytest.mark.parametrize("shape", GROUPED, ids=[s.name for s in GROUPED])
def test_rows_grouped_bf16(shape):
    inp = W.make_inputs(shape, 3000 + shape.c_out + shape.h, kind="coherent", rho=0.3, round_bf16=True, grouped=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_F32, name=shape.name + " bf16 grouped"))
    assert rep.variant == B.CG_VARIANT_MFMA_ROWS
    assert 0.1 < rep.fired_frac < 0.6
    _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_BF16, name=shape.name + " bf16 out"))


@pytest.mark.parametrize("shape", GROUPED, ids=[s.name for s in GROUPED])
def test_rows_grouped_int8_bit_exact(shape):
    if shape.c_base % 16:
        pytest.skip("int8 matrix-core path needs 16-channel groups")
    q = W.quantize_int8(W.make_inputs(shape, 4000 + shape.c_out + shape.h, kind="coherent", rho=0.35, grouped=True))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    rep = _say(P.run_int8(q, thr, name=shape.name + " int8 grouped"))
    assert rep.variant in (B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_NAIVE)
    assert 0.1 < rep.fired_frac < 0.6


@pytest.mark.parametrize("variant", [B.CG_VARIANT_NAIVE, B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE],
                         ids=["plain", "rows", "tile"])
@pytest.mark.parametrize("shape", [GROUPED[0], GROUPED[4]], ids=["one_group_per_block", "two_groups_per_block"])
def test_grouped_shuffle_and_epilogues(shape, variant):
    rng = np.random.default_rng(91)
    c = shape.c_out
    inp = W.make_inputs(shape, 5000 + c, kind="coherent", rho=0.3, round_bf16=True, grouped=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    aff = dict(scale0=rng.uniform(0.5, 1.5, c), shift0=rng.normal(0, 0.1, c),
               scale1=rng.uniform(0.5, 1.5, c), shift1=rng.normal(0, 0.1, c))
    res = rng.standard_normal((shape.n, shape.ho, shape.wo, c)).astype(np.float32)
    full = B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL
    for out_dtype in (B.CG_F32, B.CG_BF16):
        for shuffle in (False, True):
            rep = _say(P.run_float(inp, gate, out_dtype=out_dtype, variant=variant, affine=aff, residual=res,
                                   epilogue=full, shuffle=shuffle,
                                   name="%s out=%d shuffle=%d" % (shape.name, out_dtype, shuffle)))
            assert rep.variant == variant
    q = W.quantize_int8(W.make_inputs(shape, 5100 + c, kind="coherent", rho=0.35, grouped=True))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    rq = W.requant_params(q, rng)
    res8 = rng.integers(-128, 128, (shape.n, shape.ho, shape.wo, c)).astype(np.int8)
    for shuffle in (False, True):
        _say(P.run_int8(q, thr, out_i8=True, rq=rq, residual=res8, rq_res_mult=1 << 14, variant=variant,
                        epilogue=B.CG_EPI_RESIDUAL | B.CG_EPI_RELU, shuffle=shuffle,
                        name="%s int8 requant shuffle=%d" % (shape.name, shuffle)))
        _say(P.run_int8(q, thr, variant=variant, shuffle=shuffle, name="%s int32 shuffle=%d" % (shape.name, shuffle)))


ODD_GROUPED = [
    W.LayerShape("go_3x3_c12_40", 3, 9, 7, 12, 40, groups=4),
    W.LayerShape("go_3x3_s2", 2, 11, 8, 8, 34, stride=2, groups=2),
    W.LayerShape("go_1x1", 2, 5, 6, 24, 72, pad=0, groups=4, k=1),
]


@pytest.mark.parametrize("shape", ODD_GROUPED, ids=[s.name for s in ODD_GROUPED])
def test_plain_grouped_odd_shapes(shape):
    """fp32 / bf16 / int8 on shapes only the plain kernel covers."""
    for in_dtype in (B.CG_F32, B.CG_BF16):
        inp = W.make_inputs(shape, 6000 + shape.c_out, kind="iid", round_bf16=(in_dtype == B.CG_BF16), grouped=True)
        gate = W.calibrate_gate(inp, 0.4, sample_images=None)
        for shuffle in (False, True):
            rep = _say(P.run_float(inp, gate, in_dtype=in_dtype, shuffle=shuffle,
                                   name="%s in=%d shuffle=%d" % (shape.name, in_dtype, shuffle)))
            assert rep.variant == B.CG_VARIANT_NAIVE
    q = W.quantize_int8(W.make_inputs(shape, 6100 + shape.c_out, kind="iid", grouped=True))
    thr = W.calibrate_gate_int8(q, 0.4, sample_images=None)
    _say(P.run_int8(q, thr, shuffle=True, name=shape.name + " int8"))


@pytest.mark.parametrize("delta,frac", [(-np.inf, 1.0), (np.inf, 0.0)])
def test_grouped_delta_infinite(delta, frac):
    for shape in (GROUPED[0], GROUPED[4]):
        inp = W.make_inputs(shape, 41, kind="iid", round_bf16=True, grouped=True)
        gate = W.calibrate_gate(inp, 0.3, sample_images=None)
        gate.delta[:] = delta
        rep = _say(P.run_float(inp, gate, name="%s grouped delta=%s" % (shape.name, delta)))
        assert rep.fired_frac == frac and rep.flips == 0


def test_grouped_kernels_agree_bit_for_bit_int8():
    """Plain, row-tiled and large-tile kernels on the same grouped int8 layer: identical outputs, decisions, counts."""
    import torch
    for shape in (GROUPED[0], GROUPED[4]):
        q = W.quantize_int8(W.make_inputs(shape, 81, kind="coherent", rho=0.35, grouped=True))
        thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
        outs = []
        for variant in (B.CG_VARIANT_NAIVE, B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE):
            layer = B.GatedConv(n_max=shape.n, h=shape.h, w=shape.w, c_in=shape.c_in, c_out=shape.c_out,
                                c_base=shape.c_base, stride=shape.stride, pad=shape.pad,
                                w_base=torch.from_numpy(q.w_base).cuda(), w_cond=torch.from_numpy(q.w_cond).cuda(),
                                in_dtype=B.CG_I8, out_dtype=B.CG_I32, gate_thr_i32=thr, variant=variant,
                                groups=shape.groups, shuffle=True)
            assert layer.variant == variant
            outs.append([t.cpu() for t in layer.forward(torch.from_numpy(q.x).cuda())])
            torch.cuda.synchronize()
            layer.close()
        for other in outs[1:]:
            for u, v in zip(outs[0], other):
                assert torch.equal(u, v)
