"""Pins for the CPU oracle: everything here checks ``oracle/`` against something
other than itself -- brute force in exact arithmetic, a library convolution,
closed forms, hand-built gate maps and a hand-computed fixture.  No GPU."""
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest
import torch

from oracle import cg_oracle as O
from tests.brute import gated_conv_brute

GOLDEN = Path(__file__).parent / "golden"


def lib_conv(x, w, stride, pad):
    """torch CPU fp64 convolution on NHWC / [CO,KH,KW,C] arrays."""
    xt = torch.from_numpy(np.asarray(x, np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.asarray(w, np.float64)).permute(0, 3, 1, 2)
    return torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()


def rand_problem(rng, n, h, w, c_in, c_out, g, k=3, ints=False):
    c_base = c_in // g
    if ints:
        x = rng.integers(0, 6, (n, h, w, c_in)).astype(np.float64)
        wt = rng.integers(-3, 4, (c_out, k, k, c_in)).astype(np.float64)
    else:
        x = np.maximum(rng.standard_normal((n, h, w, c_in)), 0)
        wt = rng.standard_normal((c_out, k, k, c_in)) * 0.3
    return x, np.ascontiguousarray(wt[..., :c_base]), np.ascontiguousarray(wt[..., c_base:])


# ---------------------------------------------------------------------------
# P1: brute force in exact rational arithmetic on tiny shapes
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0), (2, 0)])
@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_brute_force_float(stride, pad, g):
    rng = np.random.default_rng(100 * stride + 10 * pad + g)
    n, h, w, c_in, c_out = 2, 6, 5, 8, 4
    x, wb, wc = rand_problem(rng, n, h, w, c_in, c_out, g)
    mean = rng.standard_normal(c_out) * 0.1
    var = rng.uniform(0.5, 2.0, c_out)
    delta = rng.standard_normal(c_out) * 0.5
    out = O.forward_float(x, wb, wc, stride=stride, pad=pad, gate_mean=mean, gate_var=var, delta=delta,
                          epilogue=0)
    thr = [Fraction(float(mean[c] + delta[c] * np.sqrt(var[c]))) for c in range(c_out)]
    P, R, D, S = gated_conv_brute(x.tolist(), wb.tolist(), wc.tolist() if g > 1 else None, stride, pad, thr)
    P = np.array(P, dtype=np.float64)
    R = np.array(R, dtype=np.float64)
    S = np.array(S, dtype=np.float64)
    D = np.array(D, dtype=np.uint8)
    assert out["P"].shape == P.shape
    np.testing.assert_allclose(out["P"], P, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["R"], R, rtol=0, atol=1e-12)
    # decisions: equal except where the exact sum sits within rounding of the threshold
    thr_f = np.array([float(t) for t in thr])
    safe = np.abs(P - thr_f) > 1e-9
    assert np.array_equal(out["d"][safe], D[safe])
    assert safe.mean() > 0.99
    agree = out["d"] == D
    np.testing.assert_allclose(out["y"][agree], S[agree], rtol=0, atol=1e-12)


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
@pytest.mark.parametrize("g", [1, 2, 4])
def test_brute_force_int8_exact(stride, pad, g):
    rng = np.random.default_rng(7 + 100 * stride + 10 * pad + g)
    n, h, w, c_in, c_out = 2, 5, 6, 8, 4
    x = rng.integers(0, 128, (n, h, w, c_in)).astype(np.int8)
    wt = rng.integers(-127, 128, (c_out, 3, 3, c_in)).astype(np.int8)
    cb = c_in // g
    wb, wc = np.ascontiguousarray(wt[..., :cb]), np.ascontiguousarray(wt[..., cb:])
    thr = rng.integers(-3000, 3000, c_out).astype(np.int32)
    out = O.forward_int8(x, wb, wc, thr, stride=stride, pad=pad, epilogue=0)
    P, R, D, S = gated_conv_brute(x.tolist(), wb.tolist(), wc.tolist() if g > 1 else None, stride, pad,
                                  thr.tolist(), exact=False)
    assert np.array_equal(out["P"], np.array(P, dtype=np.int64))
    assert np.array_equal(out["R"], np.array(R, dtype=np.int64))
    assert np.array_equal(out["d"], np.array(D, dtype=np.uint8))
    assert np.array_equal(out["y"], np.array(S, dtype=np.int64))


# ---------------------------------------------------------------------------
# P2 / P3: Delta = -inf is the dense convolution, Delta = +inf the base path alone
# (the split identity W*x = W_p*x_p + W_r*x_r and the d = 0 branch of Eq. 1)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("stride,pad,h,w", [(1, 1, 9, 7), (2, 1, 9, 7), (2, 1, 8, 8), (1, 0, 6, 10), (2, 0, 7, 5)])
@pytest.mark.parametrize("k", [3, 1])
def test_delta_infinite_matches_library_conv(stride, pad, h, w, k):
    rng = np.random.default_rng(stride * 1000 + h * 10 + w + k)
    n, c_in, c_out, g = 3, 12, 40, 4
    x, wb, wc = rand_problem(rng, n, h, w, c_in, c_out, g, k=k)
    pad = pad if k == 3 else 0
    mean, var = rng.standard_normal(c_out), rng.uniform(0.1, 2, c_out)
    full = lib_conv(x, np.concatenate([wb, wc], axis=-1), stride, pad)
    base = lib_conv(x[..., : c_in // g], wb, stride, pad)
    lo = O.forward_float(x, wb, wc, stride=stride, pad=pad, gate_mean=mean, gate_var=var,
                         delta=np.full(c_out, -np.inf), epilogue=0)
    hi = O.forward_float(x, wb, wc, stride=stride, pad=pad, gate_mean=mean, gate_var=var,
                         delta=np.full(c_out, np.inf), epilogue=0)
    assert lo["y"].shape == full.shape
    np.testing.assert_allclose(lo["y"], full, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(hi["y"], base, rtol=1e-12, atol=1e-12)
    m = full.shape[0] * full.shape[1] * full.shape[2]
    assert lo["d"].all() and not hi["d"].any()
    assert lo["fired"] == m * c_out and hi["fired"] == 0
    # bitmap: c_out = 40 -> two words per pixel, upper 24 bits of the second word unused and zero
    assert lo["bitmap"].shape == (m, 2)
    assert (lo["bitmap"][:, 0] == 0xFFFFFFFF).all() and (lo["bitmap"][:, 1] == 0xFF).all()
    assert not hi["bitmap"].any()
    assert (lo["counts"][2:] == full.shape[1] * full.shape[2]).all()
    # executed multiply-adds: every in-range tap of every channel (dense), base channels only (never fires)
    ones = lib_conv(np.ones((1, h, w, 1)), np.ones((1, k, k, 1)), stride, pad)  # in-range taps per output
    taps = int(round(ones.sum())) * n
    assert lo["macs"] == taps * c_out * c_in
    assert hi["macs"] == taps * c_out * (c_in // g)


def test_dense_layer_has_no_gate():
    rng = np.random.default_rng(5)
    x, wb, _ = rand_problem(rng, 2, 5, 5, 8, 6, 1)
    out = O.forward_float(x, wb, None, stride=1, pad=1, epilogue=O.RELU)
    np.testing.assert_allclose(out["y"], np.maximum(lib_conv(x, wb, 1, 1), 0), rtol=1e-12, atol=1e-12)
    assert out["fired"] == 0 and not out["bitmap"].any() and not out["d"].any()


# ---------------------------------------------------------------------------
# gate formula and executed-work identity on integer-valued data (exact in fp64)
# ---------------------------------------------------------------------------
def test_gate_rule_matches_normalised_form_and_mac_identity():
    rng = np.random.default_rng(11)
    n, h, w, c_in, c_out, g = 2, 8, 8, 8, 8, 4
    x, wb, wc = rand_problem(rng, n, h, w, c_in, c_out, g, ints=True)
    P = lib_conv(x[..., :2], wb, 1, 1)
    R = lib_conv(x[..., 2:], wc, 1, 1)
    mean = np.round(P.reshape(-1, c_out).mean(0))
    var = np.full(c_out, 4.0)           # sigma = 2 exactly
    delta = np.array([0.5, -0.5, 1.0, 0.0, 2.0, -1.5, 0.25, 3.0])
    out = O.forward_float(x, wb, wc, gate_mean=mean, gate_var=var, delta=delta, epilogue=0)
    z = (P - mean) / 2.0
    d = (z >= delta).astype(np.uint8)                       # normalise, then compare with Delta
    assert np.array_equal(out["d"], d)
    np.testing.assert_array_equal(out["margin"], np.abs(z - delta))
    np.testing.assert_array_equal(out["y"], P + d * R)
    np.testing.assert_array_equal(out["y_other"], P + (1 - d) * R)
    assert out["fired"] == int(d.sum())
    assert np.array_equal(out["counts"][2:].reshape(n, c_out), d.sum(axis=(1, 2)))
    taps = lib_conv(np.ones((1, h, w, 1)), np.ones((1, 3, 3, 1)), 1, 1)[0, :, :, 0]
    want = int((taps[None, :, :, None] * (2 + 6 * d)).sum())
    assert out["macs"] == want
    # interior-only formula: M*C_out*K_p + fired*K_r when no tap is cut by the border
    out0 = O.forward_float(x, wb, wc, pad=0, gate_mean=mean, gate_var=var, delta=delta, epilogue=0)
    m0 = n * 6 * 6
    assert out0["macs"] == m0 * c_out * 9 * 2 + out0["fired"] * 9 * 6


def test_tie_fires():
    # integer data, threshold hit exactly: theta(0) = 1
    x = np.ones((1, 3, 3, 2))
    wb = np.ones((1, 3, 3, 1))
    wc = np.ones((1, 3, 3, 1))
    out = O.forward_float(x, wb, wc, gate_mean=[1.0], gate_var=[4.0], delta=[2.5], epilogue=0)  # t = 6
    assert out["d"].reshape(3, 3).tolist() == [[0, 1, 0], [1, 1, 1], [0, 1, 0]]
    assert out["margin"].reshape(3, 3)[0, 1] == 0.0
    out = O.forward_float(x, wb, wc, gate_mean=[1.0], gate_var=[4.0], delta=[2.5 + 1e-9], epilogue=0)
    assert out["d"].reshape(3, 3).tolist() == [[0, 0, 0], [0, 1, 0], [0, 0, 0]]
    # eps enters under the square root: Var + eps = 4
    out = O.forward_float(x, wb, wc, gate_mean=[1.0], gate_var=[3.0], gate_eps=1.0, delta=[2.5], epilogue=0)
    assert out["d"].sum() == 5


# ---------------------------------------------------------------------------
# hand-computed fixture
# ---------------------------------------------------------------------------
def test_closed_form_fixture():
    rows = {}
    for line in (GOLDEN / "closed_form_3x3.txt").read_text().splitlines():
        if line and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = [int(t) for t in v]
    x = np.ones((1, 3, 3, 2))
    out = O.forward_float(x, np.ones((1, 3, 3, 1)), np.ones((1, 3, 3, 1)), gate_mean=[0.0], gate_var=[1.0],
                          delta=[5.0], epilogue=O.RELU)
    assert out["P"].reshape(-1).tolist() == rows["P"]
    assert out["d"].reshape(-1).tolist() == rows["d"]
    assert out["y"].reshape(-1).tolist() == rows["y"]
    assert out["bitmap"].reshape(-1).tolist() == rows["bitmap"]
    assert out["fired"] == rows["fired"][0]
    assert out["counts"].tolist() == [5, 0, 5]
    # same numbers through the int8 path, threshold 5
    oi = O.forward_int8(x.astype(np.int8), np.ones((1, 3, 3, 1), np.int8), np.ones((1, 3, 3, 1), np.int8),
                        np.array([5], np.int32), epilogue=O.RELU)
    assert oi["y"].reshape(-1).tolist() == rows["y"] and oi["bitmap"].reshape(-1).tolist() == rows["bitmap"]


# ---------------------------------------------------------------------------
# P4: painted gate maps.  A one-hot base weight copies a shifted input channel into P,
# so the decision map is a known picture; pins tap orientation, stride, pad, bit order.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("r,s", [(0, 0), (0, 2), (1, 1), (2, 0), (2, 1)])
@pytest.mark.parametrize("stride", [1, 2])
def test_one_hot_tap_paints_shifted_image(r, s, stride):
    rng = np.random.default_rng(r * 3 + s)
    n, h, w, c_in, c_out, cb = 2, 7, 9, 6, 35, 2
    x = rng.integers(0, 10, (n, h, w, c_in)).astype(np.float64)
    wb = np.zeros((c_out, 3, 3, cb))
    src = rng.integers(0, cb, c_out)
    wb[np.arange(c_out), r, s, src] = 1.0
    wc = rng.integers(-2, 3, (c_out, 3, 3, c_in - cb)).astype(np.float64)
    thr = rng.integers(1, 9, c_out).astype(np.float64)
    out = O.forward_float(x, wb, wc, stride=stride, pad=1, gate_mean=np.zeros(c_out), gate_var=np.ones(c_out),
                          delta=thr, epilogue=0)
    ho, wo = out["y"].shape[1:3]
    xp = np.zeros((n, h + 2, w + 2, c_in))
    xp[:, 1:-1, 1:-1] = x
    want_p = np.empty((n, ho, wo, c_out))
    for a in range(ho):
        for b in range(wo):
            want_p[:, a, b, :] = xp[:, a * stride + r, b * stride + s, :][:, src]
    np.testing.assert_array_equal(out["P"], want_p)
    d = want_p >= thr
    assert np.array_equal(out["d"], d.astype(np.uint8))
    # bitmap layout: row m = (n*Ho + ho)*Wo + wo, word co>>5, bit co&31
    flat = d.reshape(-1, c_out)
    for m in (0, 1, wo, flat.shape[0] - 1):
        for co in (0, 1, 31, 32, 34):
            bit = (int(out["bitmap"][m, co >> 5]) >> (co & 31)) & 1
            assert bit == int(flat[m, co])
    assert (out["bitmap"][:, 1] >> 3 == 0).all()
    assert sum(bin(int(v)).count("1") for v in out["bitmap"].reshape(-1)) == out["fired"] == int(d.sum())


def test_zero_base_region_never_fires_with_positive_threshold():
    rng = np.random.default_rng(3)
    x = np.maximum(rng.standard_normal((1, 10, 10, 8)), 0)
    x[:, :, :5, :2] = 0.0                      # base channels are zero on the left half
    wb = rng.standard_normal((4, 3, 3, 2))
    wc = rng.standard_normal((4, 3, 3, 6))
    out = O.forward_float(x, wb, wc, gate_mean=np.zeros(4), gate_var=np.ones(4), delta=np.full(4, 0.01), epilogue=0)
    assert not out["d"][:, :, :4].any()        # columns 0..3 see only zero base inputs
    np.testing.assert_array_equal(out["y"][:, :, :4], 0.0)


# ---------------------------------------------------------------------------
# P6: nesting in Delta, count consistency
# ---------------------------------------------------------------------------
def test_fired_sets_nest_as_delta_grows():
    rng = np.random.default_rng(21)
    x, wb, wc = rand_problem(rng, 2, 9, 9, 8, 16, 4)
    mean, var = rng.standard_normal(16) * 0.1, rng.uniform(0.5, 1.5, 16)
    prev = None
    fired = []
    for dl in (-2.0, -0.5, 0.0, 0.7, 1.5, 4.0):
        out = O.forward_float(x, wb, wc, gate_mean=mean, gate_var=var, delta=np.full(16, dl), epilogue=0)
        if prev is not None:
            assert not (out["d"] & ~prev).any()
        prev = out["d"]
        fired.append(out["fired"])
        assert out["fired"] == int(out["d"].sum()) == int(out["counts"][2:].sum())
    assert fired == sorted(fired, reverse=True) and fired[0] > fired[-1]


def test_two_sided_gate():
    # theta(Delta_h - z) * theta(z - Delta_l): both ends inclusive
    x = np.ones((1, 3, 3, 2))
    wb = np.ones((1, 3, 3, 1))
    wc = np.ones((1, 3, 3, 1))
    out = O.forward_float(x, wb, wc, gate_mean=[0.0], gate_var=[1.0], delta=[5.0], delta_hi=[6.0], epilogue=0)
    assert out["d"].reshape(3, 3).tolist() == [[0, 1, 0], [1, 0, 1], [0, 1, 0]]
    out = O.forward_float(x, wb, wc, gate_mean=[0.0], gate_var=[1.0], delta=[-np.inf], delta_hi=[4.0], epilogue=0)
    assert out["d"].reshape(3, 3).tolist() == [[1, 0, 1], [0, 0, 0], [1, 0, 1]]
    out = O.forward_float(x, wb, wc, gate_mean=[0.0], gate_var=[1.0], delta=[5.0], delta_hi=[np.inf], epilogue=0)
    assert out["d"].sum() == 5


# ---------------------------------------------------------------------------
# epilogue: branch-specific scale/shift, residual, ReLU
# ---------------------------------------------------------------------------
def test_float_epilogue_against_library_conv():
    rng = np.random.default_rng(33)
    n, h, w, c_in, c_out, g = 2, 6, 6, 8, 5, 2
    x, wb, wc = rand_problem(rng, n, h, w, c_in, c_out, g, ints=True)
    P = lib_conv(x[..., :4], wb, 1, 1)
    R = lib_conv(x[..., 4:], wc, 1, 1)
    sc0, sh0 = rng.uniform(0.5, 1.5, c_out), rng.standard_normal(c_out)
    sc1, sh1 = rng.uniform(0.5, 1.5, c_out), rng.standard_normal(c_out)
    res = rng.standard_normal(P.shape)
    mean = np.round(P.reshape(-1, c_out).mean(0))
    out = O.forward_float(x, wb, wc, gate_mean=mean, gate_var=np.ones(c_out), delta=np.full(c_out, 0.5),
                          scale0=sc0, shift0=sh0, scale1=sc1, shift1=sh1, residual=res,
                          epilogue=O.RELU | O.AFFINE | O.RESIDUAL)
    d = (P - mean) >= 0.5
    want = np.where(d, sc1 * (P + R) + sh1, sc0 * P + sh0) + res
    np.testing.assert_allclose(out["y"], np.maximum(want, 0), rtol=1e-14, atol=1e-12)
    oth = np.where(~d, sc1 * (P + R) + sh1, sc0 * P + sh0) + res
    np.testing.assert_allclose(out["y_other"], np.maximum(oth, 0), rtol=1e-14, atol=1e-12)
    assert (out["y"] >= 0).all() and (out["y"] == 0).any()
    # flags off: the same call returns the bare sum
    bare = O.forward_float(x, wb, wc, gate_mean=mean, gate_var=np.ones(c_out), delta=np.full(c_out, 0.5),
                           scale0=sc0, shift0=sh0, scale1=sc1, shift1=sh1, residual=res, epilogue=0)
    np.testing.assert_array_equal(bare["y"], P + d * R)


@pytest.mark.parametrize("acc,mult,bias,shift,relu,want", [
    (3, 1, 0, 1, False, 2),        # 1.5 rounds half up
    (-3, 1, 0, 1, False, -1),      # -1.5 rounds half up (towards +inf)
    (-5, 1, 0, 1, False, -2),      # -2.5 -> -2
    (5, 3, 0, 2, False, 4),        # 15/4 = 3.75 -> 4
    (5, 3, 1, 2, False, 5),        # bias is added in output units
    (100, 5, 0, 1, False, 127),    # clamp high
    (-100, 5, 0, 1, False, -128),  # clamp low
    (-100, 5, 0, 1, True, 0),      # ReLU clamps at zero instead
    (7, 9, -2, 0, False, 61),      # shift 0: no rounding term
])
def test_int8_requant_closed_forms(acc, mult, bias, shift, relu, want):
    # 1x1 layer, one pixel: the base sum is x*w = acc exactly; gate never fires (branch 0)
    sign = 1 if acc >= 0 else -1
    x = np.array([[[[abs(acc) if abs(acc) <= 127 else 100, 1]]]], np.int8)
    wv = sign if abs(acc) <= 127 else sign * (abs(acc) // 100)
    wb = np.array([[[[wv]]]], np.int8)
    wc = np.array([[[[50]]]], np.int8)
    out = O.forward_int8(x, wb, wc, np.array([2 ** 31 - 1], np.int32), pad=0, out_i8=True,
                         rq_mult0=np.array([mult], np.int32), rq_mult1=np.array([1], np.int32),
                         rq_bias=np.array([bias], np.int32), rq_shift=shift,
                         epilogue=O.RELU if relu else 0)
    assert int(out["P"].reshape(-1)[0]) == acc
    assert int(out["y"].reshape(-1)[0]) == want


def test_int8_requant_branches_and_residual():
    rng = np.random.default_rng(8)
    n, h, w, c_in, c_out, cb = 1, 5, 5, 8, 6, 2
    x = rng.integers(0, 128, (n, h, w, c_in)).astype(np.int8)
    wb = rng.integers(-127, 128, (c_out, 3, 3, cb)).astype(np.int8)
    wc = rng.integers(-127, 128, (c_out, 3, 3, c_in - cb)).astype(np.int8)
    P = np.rint(lib_conv(x[..., :cb], wb, 1, 1)).astype(np.int64)
    R = np.rint(lib_conv(x[..., cb:], wc, 1, 1)).astype(np.int64)
    thr = np.median(P.reshape(-1, c_out), axis=0).astype(np.int32)
    m0 = rng.integers(1, 400, c_out).astype(np.int32)
    m1 = rng.integers(1, 400, c_out).astype(np.int32)
    bias = rng.integers(-20, 20, c_out).astype(np.int32)
    res = rng.integers(-128, 128, P.shape).astype(np.int8)
    shift, rmul = 14, 9000
    out = O.forward_int8(x, wb, wc, thr, out_i8=True, rq_mult0=m0, rq_mult1=m1, rq_bias=bias, rq_shift=shift,
                         residual=res, rq_res_mult=rmul, epilogue=O.RESIDUAL)
    d = P >= thr
    t = np.where(d, (P + R) * m1, P * m0) + bias.astype(np.int64) * (1 << shift) + res.astype(np.int64) * rmul
    want = np.clip(np.floor_divide(t + (1 << (shift - 1)), 1 << shift), -128, 127)
    assert np.array_equal(out["y"], want)
    assert np.array_equal(out["d"], d.astype(np.uint8))
    assert 0 < d.mean() < 1 and (want == 127).any() and (want > -128).any()
    # raw int32 output: S (+ residual*mult) with optional ReLU
    raw = O.forward_int8(x, wb, wc, thr, residual=res, rq_res_mult=3, epilogue=O.RESIDUAL | O.RELU)
    assert np.array_equal(raw["y"], np.maximum(P + d * R + 3 * res.astype(np.int64), 0))


def test_rejects_bad_problems():
    x = np.ones((1, 3, 3, 2))
    with pytest.raises(ValueError):
        O.forward_float(x, np.ones((1, 3, 3, 1)), np.ones((1, 3, 3, 1)))   # gated but no statistics


# ---------------------------------------------------------------------------
# Channel grouping (Sec. 3.3): output group i takes input group i as the base path
# and the remaining input groups as the conditional path
# ---------------------------------------------------------------------------
def split_grouped(wfull, g):
    """[CO,K,K,C] weights in input-channel order -> (w_base, w_cond) of the grouped layer, built
    with numpy slicing/deletion only."""
    c_out, c_in = wfull.shape[0], wfull.shape[-1]
    cp, cpg = c_in // g, c_out // g
    wb, wc = [], []
    for co in range(c_out):
        own = np.s_[(co // cpg) * cp:(co // cpg + 1) * cp]
        wb.append(wfull[co][..., own])
        wc.append(np.delete(wfull[co], own, axis=-1))
    return np.ascontiguousarray(np.stack(wb)), np.ascontiguousarray(np.stack(wc))


def lib_grouped_conv(x, w_base, g, stride, pad):
    """torch's grouped convolution: output group i reads input group i only."""
    xt = torch.from_numpy(np.asarray(x, np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.asarray(w_base, np.float64)).permute(0, 3, 1, 2)
    return torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad, groups=g).permute(0, 2, 3, 1).numpy()


def shuffle_channels(y, g):
    """channel j of group i -> position j*g + i (reshape [g, c/g], transpose, flatten)."""
    s = y.shape
    return np.ascontiguousarray(y.reshape(s[:-1] + (g, s[-1] // g)).swapaxes(-1, -2)).reshape(s)


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
@pytest.mark.parametrize("g,c_out", [(2, 4), (4, 4), (4, 8)])
def test_grouped_brute_force(stride, pad, g, c_out):
    rng = np.random.default_rng(900 + 100 * stride + 10 * pad + g + c_out)
    n, h, w, c_in = 2, 5, 6, 8
    x = np.maximum(rng.standard_normal((n, h, w, c_in)), 0)
    wb, wc = split_grouped(rng.standard_normal((c_out, 3, 3, c_in)) * 0.3, g)
    mean = rng.standard_normal(c_out) * 0.1
    var = rng.uniform(0.5, 2.0, c_out)
    delta = rng.standard_normal(c_out) * 0.5
    out = O.forward_float(x, wb, wc, stride=stride, pad=pad, gate_mean=mean, gate_var=var, delta=delta,
                          epilogue=0, groups=g)
    thr = [Fraction(float(mean[c] + delta[c] * np.sqrt(var[c]))) for c in range(c_out)]
    P, R, D, S = gated_conv_brute(x.tolist(), wb.tolist(), wc.tolist(), stride, pad, thr, groups=g)
    P, R, S = (np.array(a, dtype=np.float64) for a in (P, R, S))
    D = np.array(D, dtype=np.uint8)
    np.testing.assert_allclose(out["P"], P, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["R"], R, rtol=0, atol=1e-12)
    safe = np.abs(P - np.array([float(t) for t in thr])) > 1e-9
    assert np.array_equal(out["d"][safe], D[safe]) and safe.mean() > 0.99
    agree = out["d"] == D
    np.testing.assert_allclose(out["y"][agree], S[agree], rtol=0, atol=1e-12)
    # integer path, exact
    xi = rng.integers(0, 128, (n, h, w, c_in)).astype(np.int8)
    wbi, wci = split_grouped(rng.integers(-127, 128, (c_out, 3, 3, c_in)).astype(np.int8), g)
    thr_i = rng.integers(-3000, 3000, c_out).astype(np.int32)
    oi = O.forward_int8(xi, wbi, wci, thr_i, stride=stride, pad=pad, epilogue=0, groups=g)
    P, R, D, S = gated_conv_brute(xi.tolist(), wbi.tolist(), wci.tolist(), stride, pad, thr_i.tolist(),
                                  exact=False, groups=g)
    assert np.array_equal(oi["P"], np.array(P)) and np.array_equal(oi["R"], np.array(R))
    assert np.array_equal(oi["d"], np.array(D, dtype=np.uint8)) and np.array_equal(oi["y"], np.array(S))


@pytest.mark.parametrize("stride,pad,h,w", [(1, 1, 9, 7), (2, 1, 8, 8), (1, 0, 6, 10)])
@pytest.mark.parametrize("g", [2, 4])
def test_grouped_extremes_match_library_convs(stride, pad, h, w, g):
    """Never firing leaves the base path, an ordinary grouped convolution; always firing gives the
    dense convolution with every weight back at its own input channel."""
    rng = np.random.default_rng(77 + stride * 1000 + h * 10 + w + g)
    n, c_in, c_out = 3, 12, 8
    x = np.maximum(rng.standard_normal((n, h, w, c_in)), 0)
    wfull = rng.standard_normal((c_out, 3, 3, c_in)) * 0.3
    wb, wc = split_grouped(wfull, g)
    mean, var = rng.standard_normal(c_out), rng.uniform(0.1, 2, c_out)
    kw = dict(stride=stride, pad=pad, gate_mean=mean, gate_var=var, epilogue=0, groups=g)
    hi = O.forward_float(x, wb, wc, delta=np.full(c_out, np.inf), **kw)
    lo = O.forward_float(x, wb, wc, delta=np.full(c_out, -np.inf), **kw)
    np.testing.assert_allclose(hi["y"], lib_grouped_conv(x, wb, g, stride, pad), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lo["y"], lib_conv(x, wfull, stride, pad), rtol=1e-12, atol=1e-12)
    assert lo["d"].all() and not hi["d"].any()
    # a finite threshold: P is the grouped convolution, R the rest of the dense one
    mid = O.forward_float(x, wb, wc, delta=np.zeros(c_out), **kw)
    np.testing.assert_allclose(mid["P"], lib_grouped_conv(x, wb, g, stride, pad), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(mid["P"] + mid["R"], lib_conv(x, wfull, stride, pad), rtol=1e-12, atol=1e-12)


def test_grouped_cyclic_symmetry():
    """Rotating the input groups and the output groups together rotates the output groups."""
    rng = np.random.default_rng(31)
    n, h, w, c_in, c_out, g = 2, 6, 6, 8, 12, 4
    cp, cpg = c_in // g, c_out // g
    x = np.maximum(rng.standard_normal((n, h, w, c_in)), 0)
    wfull = rng.standard_normal((c_out, 3, 3, c_in)) * 0.3
    mean, var, delta = rng.standard_normal(c_out) * 0.1, rng.uniform(0.5, 2, c_out), rng.standard_normal(c_out) * 0.3
    a = O.forward_float(x, *split_grouped(wfull, g), gate_mean=mean, gate_var=var, delta=delta, groups=g)
    x2 = np.roll(x, cp, axis=-1)
    w2 = np.roll(np.roll(wfull, cp, axis=-1), cpg, axis=0)
    b = O.forward_float(x2, *split_grouped(w2, g), gate_mean=np.roll(mean, cpg), gate_var=np.roll(var, cpg),
                        delta=np.roll(delta, cpg), groups=g)
    np.testing.assert_allclose(b["y"], np.roll(a["y"], cpg, axis=-1), rtol=1e-12, atol=1e-12)
    assert np.array_equal(b["d"], np.roll(a["d"], cpg, axis=-1))
    assert 0.1 < a["d"].mean() < 0.9


def test_grouped_shuffle_is_a_transposed_store():
    rng = np.random.default_rng(32)
    n, h, w, c_in, c_out, g = 2, 5, 4, 8, 12, 4
    x = np.maximum(rng.standard_normal((n, h, w, c_in)), 0)
    wb, wc = split_grouped(rng.standard_normal((c_out, 3, 3, c_in)) * 0.3, g)
    mean, var, delta = rng.standard_normal(c_out) * 0.1, rng.uniform(0.5, 2, c_out), rng.standard_normal(c_out) * 0.3
    sc = rng.uniform(0.5, 1.5, c_out)
    res = rng.standard_normal((n, h, w, c_out))          # in the stored (shuffled) channel order
    kw = dict(gate_mean=mean, gate_var=var, delta=delta, scale0=sc, scale1=sc * 1.1, groups=g,
              epilogue=O.AFFINE | O.RESIDUAL | O.RELU)
    plain = O.forward_float(x, wb, wc, residual=np.zeros_like(res), **kw)
    pre = O.forward_float(x, wb, wc, residual=np.zeros_like(res), **dict(kw, epilogue=O.AFFINE | O.RESIDUAL))
    shuf = O.forward_float(x, wb, wc, residual=res, shuffle=True, **kw)
    # position j*g + i holds channel (i, j); the residual is added where the value is stored
    np.testing.assert_allclose(shuf["y"], np.maximum(shuffle_channels(pre["y"], g) + res, 0), rtol=1e-12, atol=1e-12)
    # decisions, bitmap and counts keep the natural channel order
    assert np.array_equal(shuf["d"], plain["d"]) and np.array_equal(shuf["bitmap"], plain["bitmap"])
    assert np.array_equal(shuf["counts"], plain["counts"])
    # a known position: channel 1 of group 2 (natural index 2*3 + 1 = 7) is stored at 1*4 + 2 = 6
    none = O.forward_float(x, wb, wc, shuffle=True, **dict(kw, epilogue=O.AFFINE))
    nat = O.forward_float(x, wb, wc, **dict(kw, epilogue=O.AFFINE))
    np.testing.assert_array_equal(none["y"][..., 6], nat["y"][..., 7])


def test_grouped_rejects_bad_problems():
    x = np.ones((1, 3, 3, 6))
    st = dict(gate_mean=np.zeros(4), gate_var=np.ones(4), delta=np.zeros(4))
    with pytest.raises(ValueError):   # c_base * groups != c_in
        O.forward_float(x, np.ones((4, 3, 3, 2)), np.ones((4, 3, 3, 4)), groups=2, **st)
    with pytest.raises(ValueError):   # c_out not a multiple of groups
        O.forward_float(x, np.ones((4, 3, 3, 2)), np.ones((4, 3, 3, 4)), groups=3, **st)
    with pytest.raises(ValueError):   # shuffle without grouping
        O.forward_float(x, np.ones((4, 3, 3, 2)), np.ones((4, 3, 3, 4)), shuffle=True, **st)


# ---------------------------------------------------------------------------
# Channel-wise gate (Sec. 3.2): an output channel of an image keeps its conditional path only if
# at least a fraction tau_c of its activations fired
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("tau", [Fraction(1, 10), Fraction(3, 10), Fraction(1, 2), Fraction(9, 10)])
@pytest.mark.parametrize("g,stride", [(1, 1), (2, 2)])
def test_channel_gate_brute_force(tau, g, stride):
    rng = np.random.default_rng(1200 + g + tau.numerator)
    n, h, w, c_in, c_out = 3, 6, 5, 8, 6
    x = rng.integers(0, 6, (n, h, w, c_in)).astype(np.float64)
    wfull = rng.integers(-3, 4, (c_out, 3, 3, c_in)).astype(np.float64)
    if g > 1:
        wb, wc = split_grouped(wfull, g)
    else:
        wb, wc = np.ascontiguousarray(wfull[..., :2]), np.ascontiguousarray(wfull[..., 2:])
    thr = rng.integers(-4, 12, c_out).astype(np.float64)
    out = O.forward_float(x, wb, wc, stride=stride, pad=1, gate_mean=np.zeros(c_out), gate_var=np.ones(c_out),
                          delta=thr, epilogue=0, groups=g, tau_c=float(tau))
    P, R, D, S = gated_conv_brute(x.tolist(), wb.tolist(), wc.tolist(), stride, 1, [Fraction(int(t)) for t in thr],
                                  groups=g, tau_c=tau)
    D = np.array(D, dtype=np.uint8)
    assert np.array_equal(out["d"], D)
    np.testing.assert_array_equal(out["y"], np.array(S, dtype=np.float64))
    # the test means something only if the gate removed some channels and kept others
    pre = out["pre_counts"].reshape(n, c_out)
    post = out["counts"][2:].reshape(n, c_out)
    assert np.array_equal(post, D.sum(axis=(1, 2)))
    if tau >= Fraction(3, 10):
        assert ((post == 0) & (pre > 0)).any()
    if tau <= Fraction(1, 2):
        assert (post > 0).any()
    assert out["fired"] == int(D.sum()) == sum(bin(int(v)).count("1") for v in out["bitmap"].reshape(-1))
    # integer path on the same numbers
    oi = O.forward_int8(x.astype(np.int8), wb.astype(np.int8), wc.astype(np.int8), thr.astype(np.int32),
                        stride=stride, pad=1, epilogue=0, groups=g, tau_c=float(tau))
    assert np.array_equal(oi["d"], D) and np.array_equal(oi["y"], np.array(S, dtype=np.int64))


def test_channel_gate_painted_counts_and_tie():
    """A one-hot centre tap makes P a copy of an input channel, so the fired count of each output
    channel is painted by hand: channel 0 fires on 12 of 30 pixels, channel 1 on 29, channel 2 on 30."""
    h, w = 5, 6
    x = np.zeros((2, h, w, 4))
    x[0, :2, :, 0] = 5.0          # image 0, channel 0: the first two rows (12 pixels)
    x[0, :, :, 1] = 5.0
    x[0, 0, 0, 1] = 0.0           # channel 1: everything but one pixel (29)
    x[:, :, :, 2] = 5.0           # channel 2: everywhere, both images
    x[1, 2, 3, 0] = 5.0           # image 1, channel 0: a single pixel
    x[..., 3] = 1.0               # the conditional channel
    wb = np.zeros((3, 3, 3, 3))
    wb[np.arange(3), 1, 1, np.arange(3)] = 1.0
    wc = np.zeros((3, 3, 3, 1))
    wc[:, 1, 1, 0] = 100.0        # R = 100 wherever computed
    kw = dict(gate_mean=np.zeros(3), gate_var=np.ones(3), delta=np.full(3, 1.0), epilogue=0)
    base = O.forward_float(x, wb, wc, **kw)
    assert base["counts"][2:].tolist() == [12, 29, 30, 1, 0, 30]
    tie = O.forward_float(x, wb, wc, tau_c=0.4, **kw)          # 0.4 * 30 = 12: equality keeps the channel
    assert tie["counts"][2:].tolist() == [12, 29, 30, 0, 0, 30]
    assert tie["pre_counts"].tolist() == [12, 29, 30, 1, 0, 30]
    over = O.forward_float(x, wb, wc, tau_c=0.41, **kw)
    assert over["counts"][2:].tolist() == [0, 29, 30, 0, 0, 30]
    np.testing.assert_array_equal(over["y"][0, :, :, 0], x[0, :, :, 0])          # base path only: y = P
    np.testing.assert_array_equal(over["y"][0, :, :, 1], x[0, :, :, 1] + 100.0 * (x[0, :, :, 1] >= 1))
    full = O.forward_float(x, wb, wc, tau_c=1.0, **kw)          # only all-firing channels survive
    assert full["counts"][2:].tolist() == [0, 0, 30, 0, 0, 30]
    assert full["fired"] == 60 and full["macs"] < over["macs"] < tie["macs"] < base["macs"]
    none = O.forward_float(x, wb, wc, tau_c=1.01, **kw)
    assert none["fired"] == 0 and not none["bitmap"].any()
    np.testing.assert_array_equal(none["y"], base["P"])


def test_channel_gate_extremes_and_nesting():
    rng = np.random.default_rng(55)
    n, c_in, c_out, g = 3, 12, 8, 4
    x, wb, wc = rand_problem(rng, n, 9, 7, c_in, c_out, g)
    mean, var = np.zeros(c_out), np.ones(c_out)
    kw = dict(stride=1, pad=1, gate_mean=mean, gate_var=var, delta=rng.uniform(0.2, 1.5, c_out), epilogue=O.RELU)
    off = O.forward_float(x, wb, wc, **kw)
    zero = O.forward_float(x, wb, wc, tau_c=0.0, **kw)
    np.testing.assert_array_equal(off["y"], zero["y"])
    assert np.array_equal(off["d"], zero["d"]) and off["macs"] == zero["macs"]
    never = O.forward_float(x, wb, wc, tau_c=2.0, **kw)
    np.testing.assert_allclose(never["y"], np.maximum(lib_conv(x[..., : c_in // g], wb, 1, 1), 0), rtol=1e-12, atol=1e-12)
    prev = off["d"]
    sums = []
    for tau in (0.1, 0.2, 0.3, 0.5, 0.8):
        cur = O.forward_float(x, wb, wc, tau_c=tau, **kw)
        assert not (cur["d"] & ~prev).any()                         # decisions only ever drop out
        pre = cur["pre_counts"].reshape(n, c_out)
        keep = pre >= tau * 9 * 7
        assert np.array_equal(cur["d"], off["d"] * keep[:, None, None, :])
        prev = cur["d"]
        sums.append(int(prev.sum()))
    assert any(0 < v < int(off["d"].sum()) for v in sums)


# ---------------------------------------------------------------------------
# Dense pieces of a ResNet around the gated layers: library routines and hand values
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("k,stride,pad,c_in", [(7, 2, 3, 3), (3, 1, 1, 4), (5, 2, 2, 1), (1, 2, 0, 8)])
def test_dense_conv_matches_library(k, stride, pad, c_in):
    rng = np.random.default_rng(k * 10 + stride)
    x = rng.standard_normal((2, 13, 11, c_in))
    w = rng.standard_normal((6, k, k, c_in)) * 0.2
    sc, sh = rng.uniform(0.5, 1.5, 6), rng.standard_normal(6) * 0.1
    got = O.dense_conv(x, w, stride=stride, pad=pad, scale=sc, shift=sh, relu=True)
    want = np.maximum(lib_conv(x, w, stride, pad) * sc + sh, 0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.dense_conv(x, w, stride=stride, pad=pad), lib_conv(x, w, stride, pad), rtol=1e-12, atol=1e-12)


def test_maxpool_matches_library_and_ignores_padding():
    rng = np.random.default_rng(8)
    for h, w in ((8, 8), (7, 9), (5, 4), (1, 1)):
        x = rng.standard_normal((2, h, w, 5)) - 3.0          # all negative: zero padding would win if it counted
        want = torch.nn.functional.max_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).numpy()
        got = O.maxpool3x3s2(x)
        assert got.shape == want.shape == (2, (h - 1) // 2 + 1, (w - 1) // 2 + 1, 5)
        np.testing.assert_array_equal(got, want)
    # by hand: 4x4 ramp, output (0,0) sees rows/cols {0,1}, output (1,1) sees rows/cols {1,2,3}
    x = np.arange(16, dtype=np.float64).reshape(1, 4, 4, 1)
    np.testing.assert_array_equal(O.maxpool3x3s2(x)[0, :, :, 0], [[5, 7], [13, 15]])


def test_avgpool_fc_matches_library():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 7, 7, 10))
    w, b = rng.standard_normal((4, 10)), rng.standard_normal(4)
    want = x.mean(axis=(1, 2)) @ w.T + b
    np.testing.assert_allclose(O.avgpool_fc(x, w, b), want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.avgpool_fc(x.reshape(3, 49, 10), w), want - b, rtol=1e-12, atol=1e-12)
    # by hand: constant maps, identity weights
    np.testing.assert_allclose(O.avgpool_fc(np.full((1, 4, 2), 3.0), np.eye(2)), [[3.0, 3.0]])


# ---------------------------------------------------------------------------
# The layer as Eq. 1 executes it (conditional sum only where the gate fired): brute force, the
# library convolutions at the two extremes, the executed-MAC count in closed form, and the build
# the benchmark times
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
@pytest.mark.parametrize("g", [2, 4])
def test_skip_where_closed_brute_force(stride, pad, g):
    rng = np.random.default_rng(900 + 100 * stride + 10 * pad + g)
    n, h, w, c_in, c_out = 2, 6, 5, 8, 4
    # integers: every sum is exact in any accumulator, so the rational brute force must be met exactly
    x, wb, wc = rand_problem(rng, n, h, w, c_in, c_out, g, ints=True)
    thr = rng.integers(-4, 12, c_out).astype(np.float64)
    P, R, D, S = gated_conv_brute(x.tolist(), wb.tolist(), wc.tolist(), stride, pad, [Fraction(float(t)) for t in thr])
    D, S = np.array(D, np.uint8), np.array(S, np.float64)
    for timed in (False, True):
        out = O.forward_skip(x, wb, wc, stride=stride, pad=pad, gate_mean=thr, gate_var=np.ones(c_out),
                             delta=np.zeros(c_out), epilogue=0, timed_build=timed)
        assert np.array_equal(out["d"], D)
        assert np.array_equal(out["y"], S)
        assert out["fired"] == int(D.sum())
        bits = np.unpackbits(out["bitmap"].view(np.uint8), bitorder="little").reshape(-1, 32)[:, :c_out]
        assert np.array_equal(bits.reshape(D.shape), D)
    # int8 path against the same brute force
    xi = rng.integers(0, 128, (n, h, w, c_in)).astype(np.int8)
    wt = rng.integers(-127, 128, (c_out, 3, 3, c_in)).astype(np.int8)
    cb = c_in // g
    wbi, wci = np.ascontiguousarray(wt[..., :cb]), np.ascontiguousarray(wt[..., cb:])
    ti = rng.integers(-3000, 3000, c_out).astype(np.int32)
    _, _, Di, Si = gated_conv_brute(xi.tolist(), wbi.tolist(), wci.tolist(), stride, pad, ti.tolist(), exact=False)
    for timed in (False, True):
        out = O.forward_skip(xi, wbi, wci, thr=ti, stride=stride, pad=pad, epilogue=0, timed_build=timed)
        assert np.array_equal(out["d"], np.array(Di, np.uint8))
        assert np.array_equal(out["y"], np.array(Si, np.int64))


def test_skip_where_closed_extremes_and_mac_count():
    rng = np.random.default_rng(77)
    n, h, w, c_in, c_out, g = 2, 7, 6, 8, 6, 4
    x, wb, wc = rand_problem(rng, n, h, w, c_in, c_out, g)
    wfull = np.concatenate([wb, wc], axis=-1)
    one, zero = np.ones(c_out), np.zeros(c_out)
    # every gate open: the dense convolution of all channels; every gate closed: the base channels alone
    op = O.forward_skip(x, wb, wc, pad=0, gate_mean=zero, gate_var=one, delta=np.full(c_out, -np.inf), epilogue=0)
    np.testing.assert_allclose(op["y"], lib_conv(x, wfull, 1, 0), rtol=0, atol=1e-12)
    cl = O.forward_skip(x, wb, wc, pad=0, gate_mean=zero, gate_var=one, delta=np.full(c_out, np.inf), epilogue=0)
    np.testing.assert_allclose(cl["y"], lib_conv(x[..., :2], wb, 1, 0), rtol=0, atol=1e-12)
    # no padding: every output sees all nine taps, so the executed multiply-adds have a closed form
    m = n * (h - 2) * (w - 2)
    assert op["macs"] == m * c_out * 9 * c_in and cl["macs"] == m * c_out * 9 * 2
    mid = O.forward_skip(x, wb, wc, pad=0, gate_mean=zero, gate_var=one, delta=np.full(c_out, 0.2), epilogue=0)
    assert 0 < mid["fired"] < m * c_out
    assert mid["macs"] == m * c_out * 9 * 2 + mid["fired"] * 9 * 6
    # and the same decisions, outputs and counts as the both-branches oracle
    ref = O.forward_float(x, wb, wc, pad=0, gate_mean=zero, gate_var=one, delta=np.full(c_out, 0.2), epilogue=0)
    assert np.array_equal(mid["d"], ref["d"]) and np.array_equal(mid["bitmap"], ref["bitmap"])
    assert np.array_equal(mid["counts"], ref["counts"]) and mid["macs"] == ref["macs"]
    np.testing.assert_array_equal(mid["y"], ref["y"])


def test_timed_build_differs_only_by_single_precision_rounding():
    rng = np.random.default_rng(78)
    x, wb, wc = rand_problem(rng, 2, 9, 8, 16, 8, 4)
    kw = dict(gate_mean=np.zeros(8), gate_var=np.ones(8), delta=np.full(8, 0.3), epilogue=O.RELU)
    a = O.forward_skip(x, wb, wc, **kw)
    b = O.forward_skip(x, wb, wc, timed_build=True, **kw)
    same = a["d"] == b["d"]
    assert same.mean() > 0.99                                   # a sum on the threshold may round either way
    np.testing.assert_allclose(b["y"][same], a["y"][same], rtol=1e-5, atol=1e-5)
