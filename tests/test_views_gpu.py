"""GPU-vs-oracle parity of the channel-range entry points of the 2x2x2 stride-2 layers (conv3d_fwd_view,
conv3d_dgrad_view, conv3d_wgrad_view) and of the weight-gradient kernel of those layers.  The oracle side slices
the wide tensor with numpy and runs the plain fp64 passes."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from paper_1812_07816_amd import conv3d as mc
from paper_1812_07816_amd._lib import Mi3dError
from tests import parity

pytestmark = pytest.mark.gpu

CASES = [
    # N, D, H, W (big volume), Cin (big side), Cout (small side), pitch, offset
    (1, 8, 8, 16, 32, 64, 64, 0),
    (1, 8, 8, 16, 32, 64, 64, 32),
    (2, 6, 10, 14, 64, 128, 128, 0),
    (1, 4, 6, 6, 256, 320, 512, 256),
    (1, 6, 22, 26, 32, 64, 96, 40),     # ragged tile tails, an offset that is no multiple of 32
]


@pytest.mark.parametrize("case", CASES)
def test_view_passes_match_oracle_on_the_sliced_tensor(device, case):
    N, D, H, W, Cin, Cout, pitch, off = case
    x, w, dy = si.conv_case(94, 10 * CASES.index(case), N, D, H, W, Cin, Cout, 2, 2, 0, True)
    wide = si.normal(94, 10 * CASES.index(case) + 5, (N, D, H, W, pitch), bf16=True)
    wide[..., off:off + Cin] = x
    g = oc.shape(N, D, H, W, Cin, Cout, 2, 2, 0)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, 2, 2, 0, torch.bfloat16)
    for p in range(3):
        assert mc.kernel_name(desc, p) == "mfma_k2s2_panel_gemm"
    wd, dyd, wided = parity.to_device(w, True), parity.to_device(dy, True), parity.to_device(wide, True)
    tol = parity.TOL["bf16"]

    y = parity.to_host(mc.conv3d_fwd_view(desc, wided, off, wd))
    e_f = oc.rel_err(y, oc.fwd(g, x, w))
    dw = parity.to_host(mc.conv3d_wgrad_view(desc, wided, off, dyd))
    e_w = oc.rel_err(dw, oc.wgrad(g, x, dy))
    # dense calls give the same bits as views onto the same data
    xd = parity.to_device(x, True)
    assert torch.equal(mc.conv3d_fwd(desc, xd, wd), mc.conv3d_fwd_view(desc, wided, off, wd))
    assert torch.equal(mc.conv3d_wgrad(desc, xd, dyd), mc.conv3d_wgrad_view(desc, wided, off, dyd))

    out = wided.clone()
    mc.conv3d_dgrad_view(desc, dyd, wd, out, off)
    o = parity.to_host(out)
    e_d = oc.rel_err(o[..., off:off + Cin], oc.dgrad(g, dy, w))
    keep = np.ones(pitch, dtype=bool)
    keep[off:off + Cin] = False
    assert np.array_equal(o[..., keep], wide[..., keep].astype(np.float32))      # the other channels are untouched
    print(case, f"fwd {e_f:.2e} dgrad {e_d:.2e} wgrad {e_w:.2e}", flush=True)
    assert e_f <= tol and e_d <= tol and e_w <= tol


def test_k2_weight_gradient_is_bit_reproducible(device):
    N, D, H, W, Cin, Cout = 2, 12, 20, 36, 64, 128
    x, _, dy = si.conv_case(94, 90, N, D, H, W, Cin, Cout, 2, 2, 0, True)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, 2, 2, 0, torch.bfloat16)
    xd, dyd = parity.to_device(x, True), parity.to_device(dy, True)
    dw = torch.full((Cout, 2, 2, 2, Cin), 7.0, device="cuda")
    a = mc.conv3d_wgrad(desc, xd, dyd, dw=dw).clone()
    b = mc.conv3d_wgrad(desc, xd, dyd, dw=dw).clone()
    assert torch.equal(a, b)
    assert oc.rel_err(a.cpu().numpy(), oc.wgrad(oc.shape(N, D, H, W, Cin, Cout, 2, 2, 0), x, dy)) <= 1e-2


def test_views_are_refused_where_no_kernel_takes_them(device):
    desc = mc.make_desc(1, 4, 4, 4, 32, 32, 3, 1, 1, torch.bfloat16)
    wide = torch.zeros((1, 4, 4, 4, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((32, 3, 3, 3, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(Mi3dError):
        mc.conv3d_fwd_view(desc, wide, 0, w)
    d2 = mc.make_desc(1, 4, 4, 4, 32, 64, 2, 2, 0, torch.bfloat16)
    w2 = torch.zeros((64, 2, 2, 2, 32), dtype=torch.bfloat16, device="cuda")
    from paper_1812_07816_amd._lib import View, lib
    import ctypes
    y = torch.zeros((1, 2, 2, 2, 64), dtype=torch.bfloat16, device="cuda")
    for pitch, off in ((64, 36), (60, 0), (64, 40)):      # offset not a multiple of 8 / pitch too small / range past the end
        v = View(pitch, off)
        st = lib().mi3d_conv3d_fwd_view(ctypes.byref(d2), wide.data_ptr(), ctypes.byref(v), w2.data_ptr(), y.data_ptr(), None, 0, None)
        assert st == -1, (pitch, off, st)
