"""GPU-vs-oracle parity of the convolution entry points with the LeakyReLU epilogue:
conv3d_fwd_lrelu (y = lrelu(conv(x, w))) and conv3d_dgrad_lrelu (dx = dgrad(dy, w) * lrelu'(a_in)).
The oracle side is the fp64 convolution followed by the network's LeakyReLU (Section 4.1) written out with
numpy; tolerance as for the plain bf16 passes.  The geometries cover every kernel that applies the epilogue
itself (stride-1 plane streaming with 1, 2 and more input-channel chunks, the chunked variants, the stride-2
forward kernels, the 4-channel first layer) and ones that fall back to a separate elementwise pass."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from oracle import unet as ou
from paper_1812_07816_amd import conv3d as mc
from tests import parity

pytestmark = pytest.mark.gpu

CASES = [
    # N, D, H, W, Cin, Cout, k, s, p
    (1, 10, 20, 40, 32, 32, 3, 1, 1),     # plane streaming, one chunk
    (1, 8, 16, 32, 64, 32, 3, 1, 1),      # two chunks (forward) / one chunk, two cout tiles (data gradient)
    (1, 65, 65, 66, 128, 32, 3, 1, 1),    # streamed weights (enough units to fill the chip without chunking); sampled
    (1, 6, 6, 12, 128, 64, 3, 1, 1),      # chunked variant, forward
    (1, 4, 6, 12, 64, 128, 3, 1, 1),      # chunked variant, data gradient
    (1, 4, 4, 6, 320, 320, 3, 1, 1),
    (2, 12, 20, 36, 4, 32, 3, 1, 1),      # first layer
    (1, 12, 14, 34, 32, 64, 3, 2, 1),     # stride 2, one chunk
    (1, 12, 12, 12, 64, 128, 3, 2, 1),    # stride 2, chunked forward and chunked data gradient
    (1, 9, 21, 37, 32, 32, 3, 2, 1),
    (1, 8, 8, 16, 32, 64, 2, 2, 0),       # up-sampling geometry: separate elementwise pass
    (2, 9, 10, 37, 8, 8, 3, 1, 1),        # operand embedding: separate elementwise pass
]


@pytest.mark.parametrize("case", CASES)
def test_fwd_lrelu_and_dgrad_lrelu(device, case):
    N, D, H, W, Cin, Cout, k, s, p = case
    x, w, dy = si.conv_case(92, 10 * CASES.index(case), N, D, H, W, Cin, Cout, k, s, p, True)
    g = oc.shape(N, D, H, W, Cin, Cout, k, s, p)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16)
    xd, wd, dyd = parity.to_device(x, True), parity.to_device(w, True), parity.to_device(dy, True)
    tol = parity.TOL["bf16"]

    full = N * D * H * W * Cin * Cout * 27 < 4e9
    y = parity.to_host(mc.conv3d_fwd_lrelu(desc, xd, wd, ou.SLOPE))
    if full:
        ref = ou._lrelu(oc.fwd(g, x, w))
    else:
        idx = parity.structured_and_random(y.shape, 20000, 1)
        y, ref = y.ravel()[idx], ou._lrelu(oc.fwd_at(g, x, w, idx))
    e_f = oc.rel_err(y, ref)
    # the activation must have been applied: negative outputs are scaled, not clipped and not left alone
    neg = ref < 0
    assert neg.any() and (~neg).any()
    e_neg = oc.rel_err(y[neg], ref[neg])

    # x doubles as the activated input of the layer (mixed signs)
    dxd = mc.conv3d_dgrad_lrelu(desc, dyd, wd, xd, ou.SLOPE)
    dx = parity.to_host(dxd)
    if full:
        ref_d = ou._lrelu_grad(x.astype(np.float64), oc.dgrad(g, dy, w))
        e_d = oc.rel_err(dx, ref_d)
    else:
        idx = parity.structured_and_random(dx.shape, 20000, 2)
        ref_d = ou._lrelu_grad(x.astype(np.float64).ravel()[idx], oc.dgrad_at(g, dy, w, idx))
        e_d = oc.rel_err(dx.ravel()[idx], ref_d)
    print(case, f"fwd {e_f:.2e} (negative part {e_neg:.2e}) dgrad {e_d:.2e}", flush=True)
    assert e_f <= tol and e_neg <= tol and e_d <= tol


SKIP_CASES = [
    # N, D, H, W, Cin, Cout, k, s, p
    (1, 12, 14, 34, 32, 64, 3, 2, 1),     # stride-2 data gradient, sum and factor in the store path; ragged patch tails
    (1, 11, 13, 35, 32, 64, 3, 2, 1),     # odd extents: the last plane, row and column pair are half outside
    (1, 8, 10, 12, 32, 64, 3, 2, 0),      # no padding
    (1, 12, 12, 12, 64, 128, 3, 2, 1),    # chunked data gradient: sum and factor while the chunks are added
    (1, 4, 6, 6, 256, 320, 3, 2, 1),
    (1, 9, 21, 37, 32, 32, 3, 2, 1),      # Cout 32: two passes
    (1, 8, 16, 32, 32, 32, 3, 1, 1),      # stride 1: two passes
    (2, 6, 10, 70, 64, 64, 3, 2, 1),      # two samples, two tiles of input channels, two patch columns
]


@pytest.mark.parametrize("case", SKIP_CASES)
@pytest.mark.parametrize("slope", [ou.SLOPE, 1.0])
def test_dgrad_skip_is_the_data_gradient_plus_the_skip_gradient_through_the_activation(device, case, slope):
    from paper_1812_07816_amd import glue
    N, D, H, W, Cin, Cout, k, s, p = case
    x, w, dy = si.conv_case(96, 10 * SKIP_CASES.index(case), N, D, H, W, Cin, Cout, k, s, p, True)
    add = si.normal(96, 10 * SKIP_CASES.index(case) + 5, x.shape, bf16=True)
    g = oc.shape(N, D, H, W, Cin, Cout, k, s, p)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16)
    xd, wd, dyd, addd = (parity.to_device(t, True) for t in (x, w, dy, add))
    # x doubles as the activated skip tensor (mixed signs)
    out = torch.full_like(xd, 7.0)
    mc.conv3d_dgrad_skip(desc, dyd, wd, addd, xd, slope, out)
    # the bits of the two separate passes
    two = mc.conv3d_dgrad(desc, dyd, wd)
    glue.skip_grad(two, addd, 0, xd, slope)
    assert torch.equal(out, two)
    total = oc.dgrad(g, dy, w) + add.astype(np.float64)
    ref = np.where(x > 0, total, slope * total)
    e = oc.rel_err(parity.to_host(out), ref)
    print(case, slope, f"{e:.2e}", flush=True)
    # Two roundings: the data gradient is rounded to bf16 before the second gradient is added, so the first error
    # (2^-9 of the data gradient) is measured against the sum, which can be several times smaller; the second is the
    # usual 2^-9.  Twice the tolerance of a plain pass covers both; the elementwise pass itself is pinned bit for bit
    # against numpy in the glue tests.
    assert e <= 2 * parity.TOL["bf16"]


@pytest.mark.parametrize("case", [c for c in SKIP_CASES if c[5] == 64 and c[7] == 2])
def test_dgrad_with_the_skip_gradient_and_the_sums_of_the_normalisation_backward_pass(device, case):
    """conv3d_dgrad_insums with an added gradient: dx is the sum alone (the bits of conv3d_dgrad_skip with slope 1), and
    the two means are those of the stored sum against the skip tensor (fp64 on the host)."""
    N, D, H, W, Cin, Cout, k, s, p = case
    x, w, dy = si.conv_case(96, 10 * SKIP_CASES.index(case), N, D, H, W, Cin, Cout, k, s, p, True)
    add = si.normal(96, 10 * SKIP_CASES.index(case) + 5, x.shape, bf16=True)
    a = si.bf16_round((x * np.linspace(0.2, 3.0, Cin)).astype(np.float32))     # the activated skip tensor (mixed signs)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16)
    assert mc.dgrad_insums_supported(desc, with_add=True)
    ad, wd, dyd, addd = (parity.to_device(t, True) for t in (a, w, dy, add))
    sums = torch.full((N, Cin, 2), 7.0, device="cuda")
    dx = mc.conv3d_dgrad_insums(desc, dyd, wd, ad, ou.SLOPE, sums, add=addd)
    ref = torch.empty_like(dx)
    mc.conv3d_dgrad_skip(desc, dyd, wd, addd, ad, 1.0, ref)
    assert torch.equal(dx, ref)
    again = torch.zeros_like(sums)
    mc.conv3d_dgrad_insums(desc, dyd, wd, ad, ou.SLOPE, again, add=addd)
    assert torch.equal(sums, again)                               # fixed summation order
    dxh = parity.to_host(dx).astype(np.float64)
    xhat = ou.lrelu_inverse(a.astype(np.float64))
    g = np.where(xhat > 0, dxh, ou.SLOPE * dxh)
    m1, m2 = g.mean(axis=(1, 2, 3)), (g * xhat).mean(axis=(1, 2, 3))
    got = sums.cpu().numpy().astype(np.float64)
    s1, s2 = g.std(axis=(1, 2, 3)), (g * xhat).std(axis=(1, 2, 3))
    e1, e2 = (np.abs(got[..., 0] - m1) / s1).max(), (np.abs(got[..., 1] - m2) / s2).max()
    print(case, f"mean g {e1:.2e} mean g xhat {e2:.2e}", flush=True)
    assert e1 <= 1e-6 and e2 <= 1e-6


def test_epilogue_argument_checks(device):
    desc = mc.make_desc(1, 4, 4, 4, 32, 32, 3, 1, 1, torch.bfloat16)
    x = torch.zeros((1, 4, 4, 4, 32), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((32, 3, 3, 3, 32), dtype=torch.bfloat16, device="cuda")
    for bad in (1.0, 1.5, -0.1):
        with pytest.raises(RuntimeError):
            mc.conv3d_fwd_lrelu(desc, x, w, bad)
    # an fp32 geometry no tiled kernel takes (5 taps per axis runs through the plain kernels) has no epilogue
    d32 = mc.make_desc(1, 6, 6, 6, 4, 4, 5, 1, 2, torch.float32)
    assert mc.kernel_name(d32, 0) == "direct"
    with pytest.raises(RuntimeError):
        mc.conv3d_fwd_lrelu(d32, torch.zeros((1, 6, 6, 6, 4), device="cuda"), torch.zeros((4, 5, 5, 5, 4), device="cuda"), 0.01)


def test_dgrad_skip_argument_checks(device):
    import ctypes
    from paper_1812_07816_amd._lib import lib
    bf = torch.bfloat16
    desc = mc.make_desc(1, 8, 8, 8, 32, 64, 3, 2, 1, bf)
    dy = torch.zeros((1, 4, 4, 4, 64), dtype=bf, device="cuda")
    w = torch.zeros((64, 3, 3, 3, 32), dtype=bf, device="cuda")
    t = torch.zeros((1, 8, 8, 8, 32), dtype=bf, device="cuda")
    ws = torch.empty(mc.workspace_bytes(desc, 1) + 16, dtype=torch.uint8, device="cuda")

    def call(add, a_in, slope, ws_bytes=ws.numel(), d=desc):
        return lib().mi3d_conv3d_dgrad_skip(ctypes.byref(d), dy.data_ptr(), w.data_ptr(), add, a_in, ctypes.c_float(slope),
                                            t.data_ptr(), ws.data_ptr(), ws_bytes, None)

    other = torch.zeros_like(t)
    assert call(other.data_ptr(), other.data_ptr(), 0.01) == 0
    assert call(None, other.data_ptr(), 0.01) == -1                  # no second gradient
    assert call(other.data_ptr(), None, 0.01) == -1                  # no skip tensor
    assert call(other.data_ptr() + 2, other.data_ptr(), 0.01) == -1  # misaligned
    assert call(other.data_ptr(), other.data_ptr(), 1.5) == -1       # slope out of range
    assert call(other.data_ptr(), other.data_ptr(), 0.01, ws_bytes=16) == -3
    # fp32 geometries outside the tiled fp32 kernels are refused (5 taps per axis; same element counts as above,
    # so the buffers would be large enough for any kernel that ran)
    d32 = mc.make_desc(1, 4, 4, 4, 16, 32, 5, 1, 2, torch.float32)
    assert mc.kernel_name(d32, 1) == "direct"
    assert call(other.data_ptr(), other.data_ptr(), 0.01, d=d32) == -1
    torch.cuda.synchronize()
