"""The assembled channel-gated ResNet-18: every layer of one forward pass, fed with the tensors the
GPU pass itself produced, against the CPU oracle (layer by layer, so a decision that flips within the
margin in one layer cannot mask or fake an error in the next)."""
import numpy as np
import pytest
import torch

from oracle import cg_oracle as O
from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import resnet18 as R
from paper_1805_12549_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


def _host(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("grouped", [False, True], ids=["fixed_base", "grouped"])
def test_every_layer_of_a_forward_pass(grouped):
    n, size = 2, 96
    net = R.GatedResNet18(n, size, classes=40, rho=0.3, grouped=grouped, calib_images=2)
    x = R._t(net.calib_input[:n])
    tr = {}
    logits = net.forward(x, trace=tr)
    fused = net.forward(x)                  # the pass without a trace fuses the input layer with the pooling
    torch.cuda.synchronize()
    assert torch.equal(fused, logits)
    f32 = lambda a: np.asarray(a, np.float32).astype(np.float64)

    # input layer and pooling
    t = tr["input"]
    ref = O.dense_conv(_host(t["x"]), _host(net.w_in), stride=2, pad=3, scale=_host(net.scale_in), shift=_host(net.shift_in),
                       relu=True)
    got = _host(t["y"])
    assert (np.abs(got - ref) <= P.ATOL + P.RTOL * np.abs(ref) + P.bf16_ulp(ref)).all()
    assert np.array_equal(_host(t["pooled"]), O.maxpool3x3s2(got))

    fired = []
    for spec in net.specs:
        rec, t = net.records[spec.name], tr[spec.name]
        c_base = spec.c_in // net.groups
        wb, wc = W.split_weights(rec["wfull"], c_base, grouped)
        g = rec["gate"]
        epi = O.AFFINE | O.RELU | (O.RESIDUAL if spec.residual else 0)
        ref = O.forward_float(_host(t["x"]), wb, wc, stride=spec.stride, pad=1, gate_mean=f32(g.mean), gate_var=f32(g.var),
                              delta=f32(g.delta), scale0=f32(rec["scale"]), shift0=f32(rec["shift"]),
                              scale1=f32(rec["scale"]), shift1=f32(rec["shift"]),
                              residual=_host(t["residual"]) if spec.residual else None, epilogue=epi,
                              want_partials=False, groups=net.groups if grouped else 1)
        rep = P.compare_float(spec.name, _host(t["y"]), t["bitmap"].cpu().numpy().view(np.uint32),
                              t["counts"].cpu().numpy().view(np.uint32), ref, spec.c_out, B.CG_BF16, 0)
        fired.append(rep.fired_frac)
        if spec.name + ".sc" in tr:       # the block's 1x1 stride-2 shortcut
            s = tr[spec.name + ".sc"]
            srec = net.records[spec.name + ".sc"]
            ref = O.dense_conv(_host(s["x"]), srec["w"], stride=2, pad=0, scale=f32(srec["scale"]), shift=f32(srec["shift"]))
            got = _host(s["y"])
            assert (np.abs(got - ref) <= P.ATOL + P.RTOL * np.abs(ref) + P.bf16_ulp(ref)).all()
    # the gates do fire at roughly the calibrated rate in every layer
    assert all(0.1 < f < 0.6 for f in fired), fired

    t = tr["fc"]
    ref = O.avgpool_fc(_host(t["x"]), _host(net.w_fc), _host(net.b_fc))
    np.testing.assert_allclose(logits.cpu().numpy(), ref, rtol=P.RTOL, atol=P.ATOL)
    assert np.isfinite(ref).all() and ref.std() > 0
    net.close()


def test_dense_network_builds_and_runs():
    net = R.GatedResNet18(2, 64, classes=10, rho=0.0, calib_images=2)
    out = net.forward(R._t(net.calib_input[:2]))
    torch.cuda.synchronize()
    assert out.shape == (2, 10) and torch.isfinite(out).all()
    net.close()
