"""GPU-vs-oracle parity of the virtual-concatenation entry points (conv3d_fwd_pair, conv3d_dgrad_pair,
conv3d_wgrad_pair): the decoder's first convolution of a level reads [up-sampled | skip] as two tensors.  The oracle
side concatenates with numpy and runs the plain fp64 passes; the plain GPU calls on the materialised concatenation
must give the same bits.  Also here: conv3d_fwd_stats, the forward pass that hands out the instance-normalisation
statistics of its output (plain and two-tensor input), and conv3d_dgrad_insums, the data gradient that hands out the
two means of the instance-normalisation backward pass of the layer below."""
import ctypes

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from paper_1812_07816_amd import conv3d as mc
from paper_1812_07816_amd._lib import Mi3dError, lib
from tests import parity

pytestmark = pytest.mark.gpu

CASES = [
    # N, D, H, W, Cin (both halves together), Cout, pad
    (1, 6, 20, 40, 64, 32, 1),      # two resident weight chunks forward; one-chunk data gradient, two cout tiles
    (2, 5, 18, 34, 128, 64, 1),     # streamed weights forward; ragged patch tails
    (1, 7, 16, 32, 64, 64, 1),
    (1, 12, 12, 12, 256, 128, 1),   # few units: chunked variants with fp32 partial sums in both passes
    (1, 6, 10, 12, 512, 256, 1),
    (1, 5, 17, 33, 64, 32, 0),      # no padding
]


@pytest.mark.parametrize("case", CASES)
def test_pair_passes_match_oracle_on_the_concatenated_tensor(device, case):
    N, D, H, W, Cin, Cout, p = case
    seed = 10 * CASES.index(case)
    x, w, dy = si.conv_case(95, seed, N, D, H, W, Cin, Cout, 3, 1, p, True)
    g = oc.shape(N, D, H, W, Cin, Cout, 3, 1, p)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, 3, 1, p, torch.bfloat16)
    for q in range(3):
        assert mc.pair_supported(desc, q)
    h = Cin // 2
    xd, wd, dyd = parity.to_device(x, True), parity.to_device(w, True), parity.to_device(dy, True)
    lo, hi = xd[..., :h].contiguous(), xd[..., h:].contiguous()
    tol = parity.TOL["bf16"]

    y = mc.conv3d_fwd_pair(desc, lo, hi, wd)
    e_f = oc.rel_err(parity.to_host(y), oc.fwd(g, x, w))
    assert torch.equal(y, mc.conv3d_fwd(desc, xd, wd))
    ya = mc.conv3d_fwd_pair(desc, lo, hi, wd, slope=0.01)
    assert torch.equal(ya, mc.conv3d_fwd_lrelu(desc, xd, wd, 0.01))

    dw = mc.conv3d_wgrad_pair(desc, lo, hi, dyd)
    e_w = oc.rel_err(parity.to_host(dw), oc.wgrad(g, x, dy))
    assert torch.equal(dw, mc.conv3d_wgrad(desc, xd, dyd))

    dlo = torch.full_like(lo, 7.0)
    dhi = torch.full_like(hi, 7.0)
    mc.conv3d_dgrad_pair(desc, dyd, wd, dlo, dhi)
    dx = torch.cat([dlo, dhi], dim=-1)
    e_d = oc.rel_err(parity.to_host(dx), oc.dgrad(g, dy, w))
    assert torch.equal(dx, mc.conv3d_dgrad(desc, dyd, wd))
    print(case, f"fwd {e_f:.2e} dgrad {e_d:.2e} wgrad {e_w:.2e}", flush=True)
    assert e_f <= tol and e_d <= tol and e_w <= tol


def test_pairs_are_refused_where_no_kernel_takes_them(device):
    bf = torch.bfloat16
    for args in ((1, 8, 8, 8, 96, 32, 3, 1, 1),       # halves of 48 channels
                 (1, 8, 8, 8, 64, 32, 3, 2, 1),       # stride 2
                 (1, 8, 8, 8, 64, 64, 2, 2, 0),       # up-sampling layer
                 (1, 8, 8, 8, 64, 3, 1, 1, 0)):       # head
        d = mc.make_desc(*args, bf)
        assert not any(mc.pair_supported(d, q) for q in range(3)), args
        N, D, H, W, Cin, Cout, k = args[:7]
        lo = torch.zeros((N, D, H, W, Cin // 2), dtype=bf, device="cuda")
        w = torch.zeros((Cout, k, k, k, Cin), dtype=bf, device="cuda")
        with pytest.raises(Mi3dError):
            mc.conv3d_fwd_pair(d, lo, lo, w)
    # the fp32 kernels take halves of 32-channel multiples as well, and nothing narrower
    assert all(mc.pair_supported(mc.make_desc(1, 8, 8, 8, 64, 32, 3, 1, 1, torch.float32), q) for q in range(3))
    assert not any(mc.pair_supported(mc.make_desc(1, 8, 8, 8, 32, 32, 3, 1, 1, torch.float32), q) for q in range(3))
    # a missing or misaligned high half is an invalid argument
    d = mc.make_desc(1, 8, 8, 8, 64, 32, 3, 1, 1, bf)
    lo = torch.zeros((1, 8, 8, 8, 32), dtype=bf, device="cuda")
    w = torch.zeros((32, 3, 3, 3, 64), dtype=bf, device="cuda")
    y = torch.zeros((1, 8, 8, 8, 32), dtype=bf, device="cuda")
    ws = torch.empty(mc.workspace_bytes(d, 0) + 16, dtype=torch.uint8, device="cuda")
    for hi_ptr in (None, lo.data_ptr() + 2):
        st = lib().mi3d_conv3d_fwd_pair(ctypes.byref(d), lo.data_ptr(), hi_ptr, w.data_ptr(), y.data_ptr(), ctypes.c_float(1.0),
                                        ws.data_ptr(), ws.numel(), None)
        assert st == -1, st


STATS_CASES = [
    # N, D, H, W, Cin, Cout, pad, two-tensor input
    (2, 6, 20, 40, 32, 32, 1, False),    # one chunk; two samples
    (1, 9, 17, 33, 32, 64, 1, False),    # two cout tiles, ragged patches
    (2, 5, 18, 34, 64, 32, 1, True),     # two resident chunks, halves
    (2, 33, 33, 66, 128, 32, 1, True),   # streamed weights (enough units to stay unchunked), halves
    (3, 4, 9, 70, 64, 96, 2, False),     # three samples, pad 2, three cout tiles
    (2, 12, 20, 36, 4, 32, 1, False),    # first layer (4 input channels): one segment per workgroup
    (1, 5, 19, 45, 4, 32, 0, False),
    (1, 2, 384, 776, 4, 32, 1, False),   # more patch columns than workgroups: several segments per workgroup
]


@pytest.mark.parametrize("case", STATS_CASES)
def test_forward_statistics_match_the_separate_pass_and_the_oracle(device, case):
    from oracle import unet as ou
    from paper_1812_07816_amd import glue
    N, D, H, W, Cin, Cout, p, pair = case
    x, w, _ = si.conv_case(98, 10 * STATS_CASES.index(case), N, D, H, W, Cin, Cout, 3, 1, p, True)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, 3, 1, p, torch.bfloat16)
    assert mc.fwd_stats_supported(desc)
    xd, wd = parity.to_device(x, True), parity.to_device(w, True)
    stats = torch.full((N, Cout, 2), 7.0, device="cuda")
    if pair:
        h = Cin // 2
        y = mc.conv3d_fwd_stats(desc, xd[..., :h].contiguous(), wd, stats, x_hi=xd[..., h:].contiguous())
    else:
        y = mc.conv3d_fwd_stats(desc, xd, wd, stats)
    assert torch.equal(y, mc.conv3d_fwd(desc, xd, wd))           # the convolution itself is unchanged
    again = torch.zeros_like(stats)
    mc.conv3d_fwd_stats(desc, xd, wd, again) if not pair else mc.conv3d_fwd_stats(
        desc, xd[..., :Cin // 2].contiguous(), wd, again, x_hi=xd[..., Cin // 2:].contiguous())
    assert torch.equal(stats, again)                             # fixed summation order
    # the separate pass over the stored tensor
    ref = torch.zeros_like(stats)
    glue.instnorm_stats(y, ref, glue.instnorm_workspace(N, Cout))
    got, sep = stats.cpu().numpy().astype(np.float64), ref.cpu().numpy().astype(np.float64)
    # the oracle's statistics of the same stored values (fp64)
    yh = parity.to_host(y).astype(np.float64)
    mean = yh.mean(axis=(1, 2, 3))
    rstd = 1.0 / np.sqrt(yh.var(axis=(1, 2, 3)) + ou.IN_EPS)
    scale = np.sqrt(yh.var(axis=(1, 2, 3)))                      # a mean is as good as its size against the spread
    e_mean = np.abs(got[..., 0] - mean).max() / scale.max()
    e_rstd = np.abs(got[..., 1] / rstd - 1).max()
    e_sep = max(np.abs(got[..., 0] - sep[..., 0]).max() / scale.max(), np.abs(got[..., 1] / sep[..., 1] - 1).max())
    print(case, f"mean {e_mean:.2e} rstd {e_rstd:.2e} vs separate pass {e_sep:.2e}", flush=True)
    assert e_mean <= 1e-6 and e_rstd <= 1e-6 and e_sep <= 1e-6


def test_forward_statistics_are_refused_where_the_kernel_cannot_produce_them(device):
    bf = torch.bfloat16
    for args in ((1, 12, 12, 12, 320, 320, 3, 1, 1),   # chunked variant
                 (1, 8, 8, 8, 32, 64, 3, 2, 1),        # stride 2
                 (1, 8, 8, 8, 4, 64, 3, 1, 1)):        # first layer with more than one block of output channels
        d = mc.make_desc(*args, bf)
        assert not mc.fwd_stats_supported(d), args
        N, D, H, W, Cin, Cout, k = args[:7]
        x = torch.zeros((N, D, H, W, Cin), dtype=bf, device="cuda")
        w = torch.zeros((Cout, k, k, k, Cin), dtype=bf, device="cuda")
        with pytest.raises(Mi3dError):
            mc.conv3d_fwd_stats(d, x, w, torch.zeros((N, Cout, 2), device="cuda"))


BSUM_CASES = [
    # N, D, H, W, Cin, Cout, pad
    (2, 6, 20, 40, 32, 32, 1),     # one chunk; two samples
    (1, 9, 17, 33, 64, 32, 1),     # one chunk contracted, two tiles of output channels, ragged patches
    (2, 5, 18, 34, 64, 64, 1),     # two resident chunks
    (2, 33, 33, 66, 32, 128, 1),   # streamed weights (enough units to stay unchunked)
    (3, 4, 9, 70, 96, 64, 2),      # three samples, pad 2, three tiles of output channels
]


@pytest.mark.parametrize("case", BSUM_CASES)
def test_data_gradient_with_the_sums_of_the_normalisation_backward_pass(device, case):
    from oracle import unet as ou
    from paper_1812_07816_amd import glue
    N, D, H, W, Cin, Cout, p = case
    seed = 10 * BSUM_CASES.index(case)
    x, w, dy = si.conv_case(99, seed, N, D, H, W, Cin, Cout, 3, 1, p, True)
    # x doubles as the activated output of the layer below (mixed signs); channels of different spread
    a = si.bf16_round((x * np.linspace(0.2, 3.0, Cin)).astype(np.float32))
    desc = mc.make_desc(N, D, H, W, Cin, Cout, 3, 1, p, torch.bfloat16)
    assert mc.dgrad_insums_supported(desc)
    ad, wd, dyd = parity.to_device(a, True), parity.to_device(w, True), parity.to_device(dy, True)
    sums = torch.full((N, Cin, 2), 7.0, device="cuda")
    dx = mc.conv3d_dgrad_insums(desc, dyd, wd, ad, ou.SLOPE, sums)
    assert torch.equal(dx, mc.conv3d_dgrad(desc, dyd, wd))        # the data gradient itself is unchanged
    again = torch.zeros_like(sums)
    mc.conv3d_dgrad_insums(desc, dyd, wd, ad, ou.SLOPE, again)
    assert torch.equal(sums, again)                               # fixed summation order
    # the oracle's means of the same stored values (fp64)
    dxh = parity.to_host(dx).astype(np.float64)
    xhat = ou.lrelu_inverse(a.astype(np.float64))
    g = np.where(xhat > 0, dxh, ou.SLOPE * dxh)
    m1, m2 = g.mean(axis=(1, 2, 3)), (g * xhat).mean(axis=(1, 2, 3))
    got = sums.cpu().numpy().astype(np.float64)
    # a mean is as good as its size against the spread of what is averaged
    s1, s2 = g.std(axis=(1, 2, 3)), (g * xhat).std(axis=(1, 2, 3))
    e1, e2 = (np.abs(got[..., 0] - m1) / s1).max(), (np.abs(got[..., 1] - m2) / s2).max()
    print(case, f"mean g {e1:.2e} mean g xhat {e2:.2e}", flush=True)
    assert e1 <= 1e-6 and e2 <= 1e-6
    # the backward pass finished from these means against the one that takes its sums in a pass of its own
    stats = torch.zeros((N, Cin, 2), device="cuda")
    zst = torch.from_numpy(np.stack([np.zeros((N, Cin)), np.linspace(0.5, 2.0, Cin)[None].repeat(N, 0)], axis=-1).astype(np.float32)).cuda()
    stats.copy_(zst)
    d1, d2 = dx.clone(), dx.clone()
    glue.instnorm_lrelu_bwd_sums(d1, ad, stats, sums)
    glue.instnorm_lrelu_bwd(d2, ad, stats, glue.instnorm_workspace(N, Cin))
    ref = ou.instnorm_lrelu_bwd(xhat, zst[..., 1].cpu().numpy().astype(np.float64), dxh)
    e_f = np.max(np.abs(parity.to_host(d1) - ref), axis=(0, 1, 2, 3)) / np.max(np.abs(ref), axis=(0, 1, 2, 3))
    e_s = np.max(np.abs(parity.to_host(d2) - ref), axis=(0, 1, 2, 3)) / np.max(np.abs(ref), axis=(0, 1, 2, 3))
    print(case, f"dz: with the kernel's means {e_f.max():.2e}, with a pass of its own {e_s.max():.2e}", flush=True)
    assert e_f.max() <= 1e-2 and e_s.max() <= 1e-2


@pytest.mark.parametrize("shape", [(2, 9, 10, 37, 32, 3), (1, 5, 6, 7, 64, 4), (3, 4, 4, 4, 8, 1)])
def test_head_data_gradient_with_the_sums_of_the_normalisation_backward_pass(device, shape):
    from oracle import unet as ou
    N, D, H, W, Cin, Cout = shape
    x, w, dy = si.conv_case(99, 100 + Cin, N, D, H, W, Cin, Cout, 1, 1, 0, True)
    a = si.bf16_round((x * np.linspace(0.2, 3.0, Cin)).astype(np.float32))
    desc = mc.make_desc(N, D, H, W, Cin, Cout, 1, 1, 0, torch.bfloat16)
    assert mc.dgrad_insums_supported(desc) and mc.kernel_name(desc, 1) == "valu_pointwise_head"
    ad, wd, dyd = parity.to_device(a, True), parity.to_device(w, True), parity.to_device(dy, True)
    sums = torch.full((N, Cin, 2), 7.0, device="cuda")
    dx = mc.conv3d_dgrad_insums(desc, dyd, wd, ad, ou.SLOPE, sums)
    assert torch.equal(dx, mc.conv3d_dgrad(desc, dyd, wd))
    again = torch.zeros_like(sums)
    mc.conv3d_dgrad_insums(desc, dyd, wd, ad, ou.SLOPE, again)
    assert torch.equal(sums, again)
    dxh = parity.to_host(dx).astype(np.float64)
    xhat = ou.lrelu_inverse(a.astype(np.float64))
    g = np.where(xhat > 0, dxh, ou.SLOPE * dxh)
    m1, m2 = g.mean(axis=(1, 2, 3)), (g * xhat).mean(axis=(1, 2, 3))
    got = sums.cpu().numpy().astype(np.float64)
    s1, s2 = g.std(axis=(1, 2, 3)), (g * xhat).std(axis=(1, 2, 3))
    e1, e2 = (np.abs(got[..., 0] - m1) / s1).max(), (np.abs(got[..., 1] - m2) / s2).max()
    print(shape, f"mean g {e1:.2e} mean g xhat {e2:.2e}", flush=True)
    assert e1 <= 1e-6 and e2 <= 1e-6


def test_backward_sums_are_refused_where_the_kernel_cannot_produce_them(device):
    bf = torch.bfloat16
    for args in ((1, 12, 12, 12, 320, 320, 3, 1, 1),   # chunked variant
                 (1, 8, 8, 8, 32, 64, 3, 2, 1),        # stride 2
                 (1, 8, 8, 8, 4, 32, 3, 1, 1)):        # first layer
        d = mc.make_desc(*args, bf)
        assert not mc.dgrad_insums_supported(d), args
        N, D, H, W, Cin, Cout, k, s_ = args[:8]
        Do = (D + 2 - k) // s_ + 1
        dy = torch.zeros((N, Do, Do, Do, Cout), dtype=bf, device="cuda")
        w = torch.zeros((Cout, k, k, k, Cin), dtype=bf, device="cuda")
        a = torch.zeros((N, D, H, W, Cin), dtype=bf, device="cuda")
        with pytest.raises(Mi3dError):
            mc.conv3d_dgrad_insums(d, dy, w, a, 0.01, torch.zeros((N, Cin, 2), device="cuda"))
    d = mc.make_desc(1, 8, 16, 32, 32, 32, 3, 1, 1, bf)
    t = torch.zeros((1, 8, 16, 32, 32), dtype=bf, device="cuda")
    w = torch.zeros((32, 3, 3, 3, 32), dtype=bf, device="cuda")
    for bad in (0.0, 1.5, -0.1):                        # the inverse of the activation needs a positive slope
        with pytest.raises(Mi3dError):
            mc.conv3d_dgrad_insums(d, t, w, t.clone(), bad, torch.zeros((1, 32, 2), device="cuda"))
