"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Run on the GPU machine with ``-m gpu``."""
import numpy as np
import pytest
import torch

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


# ---------------------------------------------------------------------------
# config 1: single gated 3x3 conv, fp32, 16 -> 16 channels, 32x32, G = 4, ~30 % firing
# ---------------------------------------------------------------------------
def test_config1_fp32():
    shape = W.config1_shape()
    inp = W.make_inputs(shape, W.seed_for(1, 0), kind="iid")
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_F32, out_dtype=B.CG_F32, name="config1"))
    assert abs(rep.fired_frac - 0.30) < 0.01
    assert rep.variant == B.CG_VARIANT_NAIVE


@pytest.mark.parametrize("delta,frac", [(-np.inf, 1.0), (np.inf, 0.0)])
def test_config1_delta_infinite(delta, frac):
    shape = W.config1_shape()
    inp = W.make_inputs(shape, W.seed_for(1, 1), kind="iid")
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    gate.delta[:] = delta
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_F32, name="config1 delta=%s" % delta))
    assert rep.fired_frac == frac and rep.flips == 0


# ---------------------------------------------------------------------------
# the plain kernel on odd shapes, every dtype (ragged channel counts, 1x1, stride 2, pad 0)
# ---------------------------------------------------------------------------
ODD = [
    W.LayerShape("odd_3x3_c12_40", 3, 9, 7, 12, 40, stride=1, pad=1, groups=4),
    W.LayerShape("odd_3x3_s2", 2, 11, 8, 8, 33, stride=2, pad=1, groups=2),
    W.LayerShape("odd_3x3_p0", 2, 6, 10, 16, 16, stride=1, pad=0, groups=8),
    W.LayerShape("odd_1x1", 2, 5, 6, 24, 70, stride=1, pad=0, groups=4, k=1),
    W.LayerShape("odd_dense", 2, 7, 7, 8, 20, stride=1, pad=1, groups=1),
]


@pytest.mark.parametrize("shape", ODD, ids=[s.name for s in ODD])
@pytest.mark.parametrize("in_dtype", [B.CG_F32, B.CG_BF16])
def test_naive_float_odd_shapes(shape, in_dtype):
    inp = W.make_inputs(shape, 77 + shape.c_out, kind="iid", round_bf16=(in_dtype == B.CG_BF16))
    gate = W.calibrate_gate(inp, 0.4, sample_images=None) if shape.groups > 1 else None
    rng = np.random.default_rng(shape.c_out)
    aff = dict(scale0=rng.uniform(0.5, 1.5, shape.c_out), shift0=rng.normal(0, 0.1, shape.c_out),
               scale1=rng.uniform(0.5, 1.5, shape.c_out), shift1=rng.normal(0, 0.1, shape.c_out))
    res = rng.standard_normal((shape.n, shape.ho, shape.wo, shape.c_out)).astype(np.float32)
    for out_dtype in (B.CG_F32, B.CG_BF16):
        _say(P.run_float(inp, gate, in_dtype=in_dtype, out_dtype=out_dtype, variant=B.CG_VARIANT_NAIVE,
                         epilogue=B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL, affine=aff, residual=res,
                         name="%s in=%d out=%d" % (shape.name, in_dtype, out_dtype)))


@pytest.mark.parametrize("shape", ODD, ids=[s.name for s in ODD])
def test_naive_int8_odd_shapes(shape):
    inp = W.make_inputs(shape, 99 + shape.c_out, kind="iid")
    q = W.quantize_int8(inp)
    thr = W.calibrate_gate_int8(q, 0.4, sample_images=None)
    rng = np.random.default_rng(shape.c_out + 1)
    rq = W.requant_params(q, rng)
    res = rng.integers(-128, 128, (shape.n, shape.ho, shape.wo, shape.c_out)).astype(np.int8)
    _say(P.run_int8(q, thr, variant=B.CG_VARIANT_NAIVE, name=shape.name + " i32"))
    _say(P.run_int8(q, thr, out_i8=True, rq=rq, residual=res, rq_res_mult=1 << 14, variant=B.CG_VARIANT_NAIVE,
                    epilogue=B.CG_EPI_RESIDUAL, name=shape.name + " i8 requant"))
    _say(P.run_int8(q, thr, out_i8=True, rq=rq, variant=B.CG_VARIANT_NAIVE, epilogue=B.CG_EPI_RELU,
                    name=shape.name + " i8 relu"))


def test_two_sided_gate_naive():
    shape = W.LayerShape("two_sided", 2, 8, 8, 16, 32, groups=4)
    inp = W.make_inputs(shape, 5, kind="iid", round_bf16=True)
    gate = W.calibrate_gate(inp, 0.6, sample_images=None)
    hi = gate.delta + 1.0
    rep = _say(P.run_float(inp, gate, delta_hi=hi, variant=B.CG_VARIANT_NAIVE, name="two-sided"))
    assert 0.05 < rep.fired_frac < 0.6


def test_partial_batch_and_empty_batch():
    shape = W.LayerShape("partial", 4, 6, 6, 8, 32, groups=4)
    inp = W.make_inputs(shape, 6, kind="iid", round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    _say(P.run_float(inp, gate, n_run=3, name="n=3 of n_max=4"))
    # n = 0 is a no-op that succeeds
    x = torch.zeros((0, 6, 6, 8), dtype=torch.bfloat16, device="cuda")
    wb = torch.zeros((32, 3, 3, 2), dtype=torch.bfloat16, device="cuda")
    wc = torch.zeros((32, 3, 3, 6), dtype=torch.bfloat16, device="cuda")
    layer = B.GatedConv(n_max=4, h=6, w=6, c_in=8, c_out=32, c_base=2, w_base=wb, w_cond=wc,
                        in_dtype=B.CG_BF16, out_dtype=B.CG_F32, gate_mean=0.0, gate_var=1.0, delta=0.0)
    y, bm, cnt = layer.forward(x)
    torch.cuda.synchronize()
    assert y.shape == (0, 6, 6, 32)
    with pytest.raises(B.CGError) as e:
        layer.forward(torch.zeros((5, 6, 6, 8), dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == B.CG_EINVAL
    layer.close()


def test_determinism_naive():
    shape = W.LayerShape("det", 2, 12, 12, 16, 64, groups=4)
    inp = W.make_inputs(shape, 9, kind="iid", round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    x = torch.from_numpy(inp.x).cuda().to(torch.bfloat16)
    wb = torch.from_numpy(inp.w_base).cuda().to(torch.bfloat16)
    wc = torch.from_numpy(inp.w_cond).cuda().to(torch.bfloat16)
    layer = B.GatedConv(n_max=2, h=12, w=12, c_in=16, c_out=64, c_base=4, w_base=wb, w_cond=wc,
                        in_dtype=B.CG_BF16, out_dtype=B.CG_F32, gate_mean=gate.mean, gate_var=gate.var,
                        delta=gate.delta)
    a = [t.clone() for t in layer.forward(x)]
    b = layer.forward(x)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    layer.close()
