"""GPU parity of the matrix-core kernels (bf16 and int8) against the CPU oracle, through
the C ABI.  Sizes span several tiles, ragged tails, multi-image tiles, both strides."""
import numpy as np
import pytest

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


VARIANTS = [B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE]
VNAMES = ["rows", "tile"]


def _supported(shape, variant, int8=False):
    if variant == B.CG_VARIANT_MFMA_ROWS:      # 3x3, K stages of two 16-byte channel chunks (a one-chunk base group is padded)
        two_chunks = 32 if int8 else 16
        whole = shape.c_base % two_chunks == 0 and (shape.c_in - shape.c_base) % two_chunks == 0
        padded = shape.c_base % (two_chunks // 2) == 0 and shape.c_in % two_chunks == 0 and shape.c_base < shape.c_in
        return shape.k == 3 and (whole or padded)
    return True


SMALL = [
    # name, n, h, w, c_in, c_out, stride, groups
    W.LayerShape("m_64@56", 2, 56, 56, 64, 64),
    W.LayerShape("m_128@28", 3, 28, 28, 128, 128),
    W.LayerShape("m_256@14", 3, 14, 14, 256, 256),
    W.LayerShape("m_512@7", 5, 7, 7, 512, 512),            # 2 images per tile, odd batch
    W.LayerShape("m_64>128@56s2", 2, 56, 56, 64, 128, stride=2),
    W.LayerShape("m_128>256@28s2", 2, 28, 28, 128, 256, stride=2),
    W.LayerShape("m_256>512@14s2", 3, 14, 14, 256, 512, stride=2),
    W.LayerShape("m_cifar_64@32", 2, 32, 32, 64, 64),
    W.LayerShape("m_cifar_128@16", 2, 16, 16, 128, 128),
    W.LayerShape("m_cifar_256@8", 3, 8, 8, 256, 256),
    W.LayerShape("m_cifar_512@4", 11, 4, 4, 512, 512),     # 8 images per tile, ragged last tile
    W.LayerShape("m_ragged_19x23", 2, 19, 23, 64, 64),     # odd sizes: partial row bands
    W.LayerShape("m_g8", 2, 14, 14, 128, 64, groups=8),
    W.LayerShape("m_g2", 2, 14, 14, 64, 128, groups=2),
    W.LayerShape("m_pad0", 2, 16, 16, 64, 64, pad=0),
    W.LayerShape("m_1x1", 2, 14, 14, 128, 128, pad=0, k=1),
]


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
@pytest.mark.parametrize("shape", SMALL, ids=[s.name for s in SMALL])
def test_mfma_bf16_matches_oracle(shape, variant):
    if not _supported(shape, variant):
        pytest.skip("the row-tiled kernel takes 3x3 layers with 32-byte channel groups; the tile kernel covers the rest")
    inp = W.make_inputs(shape, 1000 + shape.c_out + shape.h, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=None)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_F32, variant=variant,
                           name=shape.name + " bf16"))
    assert rep.variant == variant
    assert 0.1 < rep.fired_frac < 0.6


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
@pytest.mark.parametrize("shape", SMALL, ids=[s.name for s in SMALL])
def test_mfma_int8_bit_exact(shape, variant):
    if not _supported(shape, variant, int8=True):
        pytest.skip("the row-tiled kernel takes 3x3 layers with 32-byte channel groups; the tile kernel covers the rest")
    if shape.c_base % 16:
        pytest.skip("int8 matrix-core path needs 16-channel groups")
    inp = W.make_inputs(shape, 2000 + shape.c_out + shape.h, kind="coherent", rho=0.35)
    q = W.quantize_int8(inp)
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    rep = _say(P.run_int8(q, thr, variant=variant, name=shape.name + " int8"))
    assert rep.variant == variant
    assert 0.1 < rep.fired_frac < 0.6


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
@pytest.mark.parametrize("kind", ["iid", "literal"])
def test_mfma_bf16_unclustered_maps(kind, variant):
    shape = W.LayerShape("m_lit", 2, 28, 28, 128, 128)
    inp = W.make_inputs(shape, 31, kind=kind, rho=0.35, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.35, sample_images=None)
    _say(P.run_float(inp, gate, variant=variant, name="unclustered " + kind))


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
@pytest.mark.parametrize("delta,frac", [(-np.inf, 1.0), (np.inf, 0.0)])
def test_mfma_delta_infinite(delta, frac, variant):
    shape = W.LayerShape("m_inf", 2, 14, 14, 64, 64)
    inp = W.make_inputs(shape, 41, kind="iid", round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    gate.delta[:] = delta
    rep = _say(P.run_float(inp, gate, variant=variant, name="delta=%s" % delta))
    assert rep.fired_frac == frac and rep.flips == 0
    if not _supported(shape, variant, int8=True):
        return
    q = W.quantize_int8(W.make_inputs(shape, 42, kind="iid"))
    thr = np.full(64, np.iinfo(np.int32).min if delta < 0 else np.iinfo(np.int32).max, np.int32)
    rep = _say(P.run_int8(q, thr, variant=variant, name="int8 delta=%s" % delta))
    assert rep.fired_frac == frac


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
def test_mfma_dense_comparator(variant):
    shape = W.LayerShape("m_dense", 2, 28, 28, 64, 128, groups=1)
    inp = W.make_inputs(shape, 51, kind="iid", round_bf16=True)
    rep = _say(P.run_float(inp, None, variant=variant, name="dense bf16"))
    assert rep.fired_frac == 0.0
    q = W.quantize_int8(W.make_inputs(shape, 52, kind="iid"))
    _say(P.run_int8(q, None, variant=variant, name="dense int8"))


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
def test_mfma_epilogues_bf16(variant):
    shape = W.LayerShape("m_epi", 3, 14, 14, 128, 128)
    inp = W.make_inputs(shape, 61, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    rng = np.random.default_rng(61)
    aff = dict(scale0=rng.uniform(0.5, 1.5, 128), shift0=rng.normal(0, 0.1, 128),
               scale1=rng.uniform(0.5, 1.5, 128), shift1=rng.normal(0, 0.1, 128))
    res = rng.standard_normal((3, 14, 14, 128)).astype(np.float32)
    for out_dtype in (B.CG_F32, B.CG_BF16):
        _say(P.run_float(inp, gate, out_dtype=out_dtype, variant=variant, affine=aff, residual=res,
                         epilogue=B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL,
                         name="epilogue out=%d" % out_dtype))
    _say(P.run_float(inp, gate, out_dtype=B.CG_BF16, variant=variant, epilogue=0, name="no epilogue bf16 out"))
    _say(P.run_float(inp, gate, variant=variant, delta_hi=gate.delta + 0.8, name="two-sided mfma"))


@pytest.mark.parametrize("variant", VARIANTS, ids=VNAMES)
def test_mfma_epilogues_int8(variant):
    shape = W.LayerShape("m_epi8", 3, 14, 14, 128, 128)
    q = W.quantize_int8(W.make_inputs(shape, 71, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    rng = np.random.default_rng(71)
    rq = W.requant_params(q, rng)
    res = rng.integers(-128, 128, (3, 14, 14, 128)).astype(np.int8)
    _say(P.run_int8(q, thr, out_i8=True, rq=rq, residual=res, rq_res_mult=1 << 14, variant=variant,
                    epilogue=B.CG_EPI_RESIDUAL | B.CG_EPI_RELU, name="int8 requant+res+relu"))
    _say(P.run_int8(q, thr, out_i8=True, rq=rq, variant=variant, epilogue=0, name="int8 requant"))
    _say(P.run_int8(q, thr, residual=res, rq_res_mult=5, variant=variant, epilogue=B.CG_EPI_RESIDUAL,
                    name="int32 + residual"))


def test_mfma_matches_naive_kernel_decisions():
    """Two independent GPU kernels, same inputs: int8 results must be identical."""
    import torch
    shape = W.LayerShape("m_x", 2, 28, 28, 128, 128)
    q = W.quantize_int8(W.make_inputs(shape, 81, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    outs = []
    for variant in (B.CG_VARIANT_NAIVE, B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE):
        x = torch.from_numpy(q.x).cuda()
        layer = B.GatedConv(n_max=2, h=28, w=28, c_in=128, c_out=128, c_base=32,
                            w_base=torch.from_numpy(q.w_base).cuda(), w_cond=torch.from_numpy(q.w_cond).cuda(),
                            in_dtype=B.CG_I8, out_dtype=B.CG_I32, gate_thr_i32=thr, variant=variant)
        a = layer.forward(x)
        b = layer.forward(x)          # run twice: results must not depend on the previous call
        torch.cuda.synchronize()
        for u, v in zip(a, b):
            assert torch.equal(u, v)
        outs.append([t.cpu() for t in b])
        layer.close()
    for other in outs[1:]:
        for u, v in zip(outs[0], other):
            assert torch.equal(u, v)
