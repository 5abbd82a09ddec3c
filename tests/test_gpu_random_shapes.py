"""GPU parity on seeded random layer shapes: odd image sizes, channel counts that are not powers of
two, both strides, with and without padding, 3x3 and 1x1, G in {2, 4, 8}, partial batches - whatever
kernel family the library picks, and the large-tile kernel forced where it takes the shape.  Every
case is checked element by element against the CPU oracle (bf16 within tolerance, int8 bit for bit)."""
import os
import zlib

import numpy as np
import pytest

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _say(rep):
    print("\n  " + str(rep), flush=True)
    return rep


def _shapes(seed, count, large=False):
    rng = np.random.default_rng(seed)
    top, nmax, budget = (65, 17, 2.5e10) if large else (34, 7, 6e9)
    out = []
    while len(out) < count:
        k = int(rng.choice([3, 3, 3, 1]))
        stride = int(rng.choice([1, 1, 2]))
        pad = int(rng.choice([1, 1, 0])) if k == 3 else 0
        g = int(rng.choice([2, 4, 4, 8]))
        c_in = int(rng.choice([32, 64, 96, 128, 160, 192, 256, 384, 512]))
        c_out = int(rng.choice([64, 128, 192, 256, 320, 512]))
        h = int(rng.integers(1 if k == 1 else 3, top))
        w = int(rng.integers(1 if k == 1 else 3, top))
        n = int(rng.integers(1, nmax))
        if c_in % g or (c_in // g) % 8:
            continue                                   # base groups of whole 16-byte bf16 chunks
        if (h + 2 * pad - k) // stride + 1 < 1 or (w + 2 * pad - k) // stride + 1 < 1:
            continue
        if n * h * w * c_in * c_out * k * k > budget:  # keep the oracle to a second or two
            continue
        out.append(W.LayerShape("r%d_%dx%dx%d_%d>%d_k%ds%dp%dg%d" % (len(out), n, h, w, c_in, c_out, k, stride, pad, g),
                                n, h, w, c_in, c_out, stride=stride, pad=pad, k=k, groups=g))
    return out


# CG_RANDOM_SHAPES="seed,count[,large]" runs another set (a longer soak by hand; `large`: images up to
# 64x64, batches up to 16); the default set is fixed
_ENV = os.environ.get("CG_RANDOM_SHAPES", "1805,36").split(",")
RANDOM = _shapes(int(_ENV[0]), int(_ENV[1]), large=len(_ENV) > 2)
# shapes that once failed: a tile height chosen for balance made the tiles straddle images, and the
# straddling tiles' patch no longer fitted its LDS buffer
RANDOM += [W.LayerShape("fixed_6x32x31_384>128_k3s1p1g4", 6, 32, 31, 384, 128, stride=1, pad=1, k=3, groups=4)]
# a wide stride-2 image with many channels: its patch fits only with two-chunk super-stages or a
# part-filled tile (once left to the plain kernel)
RANDOM += [W.LayerShape("fixed_1x37x64_384>512_k3s2p1g4", 1, 37, 64, 384, 512, stride=2, pad=1, k=3, groups=4)]


@pytest.mark.parametrize("shape", RANDOM, ids=[s.name for s in RANDOM])
def test_random_shape_bf16_and_int8(shape):
    rng = np.random.default_rng(zlib.crc32(shape.name.encode()))
    rho = float(rng.choice([0.1, 0.3, 0.5, 0.8]))
    kind = "coherent" if min(shape.h, shape.w) >= 8 else "iid"
    inp = W.make_inputs(shape, 9000 + len(shape.name) + shape.h * 31 + shape.w, kind=kind, rho=rho, round_bf16=True)
    gate = W.calibrate_gate(inp, rho, sample_images=None)
    c = shape.c_out
    aff = dict(scale0=rng.uniform(0.5, 1.5, c), shift0=rng.normal(0, 0.1, c),
               scale1=rng.uniform(0.5, 1.5, c), shift1=rng.normal(0, 0.1, c))
    res = rng.standard_normal((shape.n, shape.ho, shape.wo, c)).astype(np.float32)
    full = B.CG_EPI_RELU | B.CG_EPI_AFFINE | B.CG_EPI_RESIDUAL
    n_run = int(rng.integers(1, shape.n + 1))
    variants = [B.CG_VARIANT_AUTO]
    picked = _say(P.run_float(inp, gate, out_dtype=B.CG_BF16, affine=aff, residual=res, epilogue=full, n_run=n_run,
                              name=shape.name + " bf16 auto"))
    # on the matrix cores, except 1x1 layers whose base or conditional group is an odd number of 16-byte
    # chunks (a K step of the 1x1 kernel takes two chunks of one pixel): those run on the plain kernel
    odd_1x1 = shape.k == 1 and ((shape.c_base // 8) % 2 or ((shape.c_in - shape.c_base) // 8) % 2)
    if odd_1x1:
        assert picked.variant == B.CG_VARIANT_NAIVE
        return
    assert picked.variant in (B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE)
    if picked.variant != B.CG_VARIANT_TILE:
        try:
            _say(P.run_float(inp, gate, out_dtype=B.CG_F32, variant=B.CG_VARIANT_TILE, affine=aff, residual=res,
                             epilogue=full, n_run=n_run, name=shape.name + " bf16 tile"))
            variants.append(B.CG_VARIANT_TILE)
        except B.CGError as e:
            assert e.code == B.CG_EUNSUPPORTED       # (wide images whose patch rows do not fit its stage buffers)
    # the large-tile kernel with a forced tile shape (wavefront fragments, channel split, stage width)
    hint = int(rng.choice([1, 2, 4])) | (int(rng.choice([1, 2])) << 4) | (int(rng.choice([0, 0, 1, 2, 4, 8])) << 8)
    try:
        _say(P.run_float(inp, gate, out_dtype=B.CG_BF16, variant=B.CG_VARIANT_TILE, tile_hint=hint, n_run=n_run,
                         name="%s bf16 tile hint %#x" % (shape.name, hint)))
        if shape.c_base % 16 == 0:
            q8 = W.quantize_int8(W.make_inputs(shape, 9300 + shape.h * 31 + shape.w, kind=kind, rho=rho))
            _say(P.run_int8(q8, W.calibrate_gate_int8(q8, rho, sample_images=None), variant=B.CG_VARIANT_TILE, tile_hint=hint,
                            n_run=n_run, name="%s int8 tile hint %#x" % (shape.name, hint)))
    except B.CGError as e:
        assert e.code == B.CG_EUNSUPPORTED           # a tile shape this layer cannot take
    if shape.c_out % shape.groups == 0 and rng.random() < 0.4:
        # the same shape with channel grouping (output group i takes input group i as its base), shuffled store
        ginp = W.make_inputs(shape, 9200 + shape.h * 31 + shape.w, kind=kind, rho=rho, round_bf16=True, grouped=True)
        ggate = W.calibrate_gate(ginp, rho, sample_images=None)
        _say(P.run_float(ginp, ggate, out_dtype=B.CG_BF16, affine=aff, residual=res, epilogue=full, n_run=n_run,
                         shuffle=bool(rng.integers(0, 2)), name=shape.name + " bf16 grouped"))
    if rng.random() < 0.3:
        _say(P.run_float(inp, gate, tau_c=float(rng.choice([0.2, 0.5])), n_run=n_run, name=shape.name + " bf16 channel-wise gate"))
    if shape.c_base % 16 == 0:
        q = W.quantize_int8(W.make_inputs(shape, 9100 + len(shape.name) + shape.h * 31 + shape.w, kind=kind, rho=rho))
        thr = W.calibrate_gate_int8(q, rho, sample_images=None)
        rq = W.requant_params(q, rng)
        res8 = rng.integers(-128, 128, (shape.n, shape.ho, shape.wo, c)).astype(np.int8)
        for v in variants:
            if rng.random() < 0.5:
                _say(P.run_int8(q, thr, variant=v, n_run=n_run, name="%s int8 variant %d" % (shape.name, v)))
            else:
                _say(P.run_int8(q, thr, out_i8=True, rq=rq, residual=res8, rq_res_mult=1 << 14, variant=v, n_run=n_run,
                                epilogue=B.CG_EPI_RESIDUAL | B.CG_EPI_RELU, name="%s int8 requantised variant %d" % (shape.name, v)))
