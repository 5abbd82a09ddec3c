"""cg_conv_forward_noalloc (the entry point for callers that cannot allocate or pass a workspace)
against cg_conv_forward, through the C ABI: same outputs bit for bit, on two calls in a row, the
second with a smaller batch; and the refusal of a call whose scratch does not fit the library's array."""
import numpy as np
import pytest
import torch

from paper_1805_12549_amd import binding as B
from paper_1805_12549_amd import workloads as W

pytestmark = pytest.mark.gpu


def _layer(shape, q, thr, variant, tau_c=0.0):
    return B.GatedConv(n_max=shape.n, h=shape.h, w=shape.w, c_in=shape.c_in, c_out=shape.c_out, c_base=shape.c_base,
                       stride=shape.stride, pad=shape.pad, w_base=torch.from_numpy(q.w_base).cuda(),
                       w_cond=torch.from_numpy(q.w_cond).cuda(), in_dtype=B.CG_I8, out_dtype=B.CG_I32,
                       gate_thr_i32=thr, variant=variant, tau_c=tau_c)


def _call(layer, x, n, noalloc, want_bitmap):
    dev = x.device
    y = torch.full((n, layer.ho, layer.wo, layer.c_out), -7, dtype=torch.int32, device=dev)
    cnt = torch.full((2 + n * layer.c_out,), -7, dtype=torch.int32, device=dev)
    bm = torch.full((n * layer.ho * layer.wo, layer.words), -7, dtype=torch.int32, device=dev) if want_bitmap else None
    s = torch.cuda.current_stream().cuda_stream
    if noalloc:
        B.cg_conv_forward_noalloc(layer.handle, n, x.data_ptr(), 0, y.data_ptr(), bm.data_ptr() if want_bitmap else 0,
                                  cnt.data_ptr(), s)
    else:
        need = B.cg_conv_workspace_bytes(layer.handle, n)
        ws = torch.empty(need + 256, dtype=torch.uint8, device=dev)
        B.cg_conv_forward(layer.handle, n, x.data_ptr(), 0, y.data_ptr(), bm.data_ptr() if want_bitmap else 0,
                          cnt.data_ptr(), (ws.data_ptr() + 255) & ~255, need, s)
    torch.cuda.synchronize()
    return y, cnt, bm


@pytest.mark.parametrize("variant", [B.CG_VARIANT_MFMA_ROWS, B.CG_VARIANT_TILE], ids=["rows", "tile"])
@pytest.mark.parametrize("tau_c", [0.0, 0.3], ids=["plain_gate", "channel_gate"])
def test_noalloc_matches_forward_on_two_calls(variant, tau_c):
    shape = W.LayerShape("na_128@28", 6, 28, 28, 128, 128)
    q = W.quantize_int8(W.make_inputs(shape, 9100, kind="coherent", rho=0.35))
    thr = W.calibrate_gate_int8(q, 0.35, sample_images=None)
    layer = _layer(shape, q, thr, variant, tau_c)
    assert layer.variant == variant
    x = torch.from_numpy(q.x).cuda()
    # counts without a bitmap: the decisions of the batch go through the scratch
    assert B.cg_conv_workspace_bytes(layer.handle, shape.n) > 0
    for n in (shape.n, 2):                          # the second call is smaller and sees the first one's leftovers
        for want_bitmap in (False, True):
            ref = _call(layer, x[:n], n, False, want_bitmap)
            got = _call(layer, x[:n], n, True, want_bitmap)
            for u, v in zip(ref, got):
                if u is not None:
                    assert torch.equal(u, v)
            assert int(ref[1][0]) > 0               # something fired
    layer.close()


def test_noalloc_refuses_what_does_not_fit():
    # a batch whose decision bitmap alone (48 * 112 * 112 pixels of 8 words) is larger than the 16 MiB array
    n_max = 48
    w = torch.zeros((256, 3, 3, 16), dtype=torch.int8, device="cuda")
    wc = torch.zeros((256, 3, 3, 48), dtype=torch.int8, device="cuda")
    layer = B.GatedConv(n_max=n_max, h=112, w=112, c_in=64, c_out=256, c_base=16, w_base=w, w_cond=wc,
                        in_dtype=B.CG_I8, out_dtype=B.CG_I32, gate_thr_i32=np.zeros(256, np.int32))
    assert B.cg_conv_workspace_bytes(layer.handle, n_max) > (16 << 20)
    # buffers for two images only: the refused call must not touch them, the small one fits
    x = torch.zeros((2, 112, 112, 64), dtype=torch.int8, device="cuda")
    y = torch.zeros((2, 112, 112, 256), dtype=torch.int32, device="cuda")
    cnt = torch.full((2 + n_max * 256,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(B.CGError) as e:
        B.cg_conv_forward_noalloc(layer.handle, n_max, x.data_ptr(), 0, y.data_ptr(), 0, cnt.data_ptr(), 0)
    assert e.value.code == B.CG_EUNSUPPORTED and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert int((cnt != -7).sum()) == 0              # nothing was enqueued
    B.cg_conv_forward_noalloc(layer.handle, 2, x.data_ptr(), 0, y.data_ptr(), 0, cnt.data_ptr(), 0)
    torch.cuda.synchronize()
    # zero weights and zero thresholds: every gate fires (0 >= 0)
    assert int(cnt[0]) == 2 * 112 * 112 * 256
    layer.close()
