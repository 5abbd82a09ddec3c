"""Full-size GPU parity: every layer of the benchmark workload (ImageNet-shaped ResNet-18 gated
3x3 convs, batch 64, bf16) and of the CIFAR and int8 configurations, element by element against
the CPU oracle, in the launch configuration bench.py times (kernel family AUTO, bf16 output,
ReLU, bitmap on).  The oracle runs a whole layer in about a second on the machine's cores."""
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


IMAGENET = W.imagenet_shapes(n=64)


@pytest.mark.parametrize("li", range(len(IMAGENET)), ids=[s.name for s in IMAGENET])
def test_imagenet_bf16_batch64(li):
    shape = IMAGENET[li]
    inp = W.make_inputs(shape, W.seed_for(3, li), kind="coherent", rho=0.30, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=8)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_BF16, name=shape.name + " N=64 bf16"))
    assert rep.variant == B.CG_VARIANT_MFMA_ROWS
    assert 0.15 < rep.fired_frac < 0.5
    # (flips are allowed only inside the margin, which the comparison enforces; their count is printed)


@pytest.mark.parametrize("li", range(len(IMAGENET)), ids=[s.name for s in IMAGENET])
def test_imagenet_grouped_bf16_batch64(li):
    """The same layers with channel grouping, as `bench.py --grouped` launches them."""
    shape = IMAGENET[li]
    inp = W.make_inputs(shape, W.seed_for(3, li), kind="coherent", rho=0.30, round_bf16=True, grouped=True)
    gate = W.calibrate_gate(inp, 0.30, sample_images=8)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_BF16, name=shape.name + " N=64 grouped"))
    assert rep.variant == B.CG_VARIANT_MFMA_ROWS
    assert 0.15 < rep.fired_frac < 0.5
    # (flips are allowed only inside the margin, which the comparison enforces; their count is printed)


def test_imagenet_literal_maps_fp32_out():
    shape = IMAGENET[1]
    inp = W.make_inputs(shape, W.seed_for(3, 11), kind="literal", rho=0.35, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.35, sample_images=8)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_F32, name=shape.name + " literal"))
    assert abs(rep.fired_frac - 0.35) < 0.05


CIFAR = W.cifar_shapes(n=128)


@pytest.mark.parametrize("li", range(len(CIFAR)), ids=[s.name for s in CIFAR])
def test_cifar_bf16_batch128(li):
    shape = CIFAR[li]
    inp = W.make_inputs(shape, W.seed_for(2, li), kind="iid", round_bf16=True)
    gate = W.calibrate_gate(inp, 0.25, sample_images=16)
    rep = _say(P.run_float(inp, gate, in_dtype=B.CG_BF16, out_dtype=B.CG_F32, name=shape.name + " N=128"))
    assert abs(rep.fired_frac - 0.25) < 0.05


@pytest.mark.parametrize("n", [1, 32])
@pytest.mark.parametrize("li", range(len(IMAGENET)), ids=[s.name for s in IMAGENET])
def test_imagenet_int8_bit_exact(li, n):
    shape = IMAGENET[li].with_batch(n)
    inp = W.make_inputs(shape, W.seed_for(4, li), kind="coherent", rho=0.35)
    q = W.quantize_int8(inp)
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=8)
    rep = _say(P.run_int8(q, thr, name="%s N=%d int8" % (shape.name, n)))
    assert rep.variant in (B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE)
    rng = np.random.default_rng(li)
    rq = W.requant_params(q, rng)
    _say(P.run_int8(q, thr, out_i8=True, rq=rq, name="%s N=%d int8 requant" % (shape.name, n)))


def test_counts_off_and_graph_replay_match_eager():
    """The benchmark passes no counts buffer and replays a HIP graph; both must give the eager result,
    on every replay (the counts path clears its buffer with a fill kernel, not a memset node)."""
    shape = W.LayerShape("g_128@28", 8, 28, 28, 128, 128)
    inp = W.make_inputs(shape, 17, kind="coherent", rho=0.3, round_bf16=True)
    gate = W.calibrate_gate(inp, 0.3, sample_images=None)
    x = torch.from_numpy(inp.x).cuda().to(torch.bfloat16)
    wb = torch.from_numpy(inp.w_base).cuda().to(torch.bfloat16)
    wc = torch.from_numpy(inp.w_cond).cuda().to(torch.bfloat16)
    layer = B.GatedConv(n_max=8, h=28, w=28, c_in=128, c_out=128, c_base=32, w_base=wb, w_cond=wc,
                        in_dtype=B.CG_BF16, out_dtype=B.CG_BF16, gate_mean=gate.mean, gate_var=gate.var,
                        delta=gate.delta)
    y0, bm0, c0 = [t.clone() for t in layer.forward(x)]
    y1, bm1, _ = layer.forward(x, counts=False)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(bm0, bm1)
    y = torch.empty_like(y0)
    bm = torch.empty_like(bm0)
    cnt = torch.empty_like(c0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.forward(x, y=y, bitmap=bm, counts=cnt)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            layer.forward(x, y=y, bitmap=bm, counts=cnt)
    torch.cuda.synchronize()
    for rep in range(3):
        y.zero_()
        bm.zero_()
        cnt.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y0) and torch.equal(bm, bm0) and torch.equal(cnt, c0), "replay %d differs" % rep
        layer.forward(x, counts=False)          # eager work between replays
        torch.cuda.synchronize()
    layer.close()
