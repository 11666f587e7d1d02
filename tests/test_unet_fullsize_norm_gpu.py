"""The headline step itself (192^3, N = 2, bf16, convolution -> instance normalisation -> LeakyReLU) against the fp64
oracle, teacher-forced: the step runs once with a trace of the tensors around a few normalised layers, and each step
of such a layer is compared with the oracle's definition of it applied to the tensors the step fed it.  What this
reaches and the reduced-volume tests do not: the statistics that come out of the convolution kernels' store paths and
the backward sums that come out of the data gradients (plane streaming, stride 2 with the skip gradient, the 1x1x1
head) with the unit ranges, segment counts and workgroup numbers of the full-size launches.  Statistics and sums are
compared on the whole tensor (fp64 means of the stored values), element-wise results on the tile seams plus a few
thousand random positions."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from oracle import unet as ou
from tests import parity

pytestmark = pytest.mark.gpu

CH = [32, 64, 128, 256, 320]
N, VOL = 2, 192
SLOPE = ou.SLOPE
TOL = 1e-2
N_SAMPLES = 8000

# name -> (input tensor, Cin, Cout, stride, level of the input volume, who delivers the backward sums)
LAYERS = {
    "enc0.conv1": ("input", 4, 32, 1, 0, "the data gradient of enc0.conv2"),
    "enc0.conv2": ("enc0.conv1", 32, 32, 1, 0, "the stride-2 data gradient of enc1.conv1, which also adds the skip gradient"),
    "dec0.conv1": ("dec0.cat", 64, 32, 1, 0, "the data gradient of dec0.conv2"),
    "dec0.conv2": ("dec0.conv1", 32, 32, 1, 0, "the data gradient of the head"),
    "enc1.conv2": ("enc1.conv1", 64, 64, 1, 1, "a reduction pass of its own"),
    "enc3.conv2": ("enc3.conv1", 256, 256, 1, 3, "a reduction pass of its own"),
}


class _Pick(dict):
    keep_fused = True

    def __init__(self, wanted):
        super().__init__()
        self.wanted = set(wanted)

    def __setitem__(self, k, v):
        if k in self.wanted:
            super().__setitem__(k, v)


_cache = {}


def _step(f32=False):
    if _cache.get("f32") != f32:
        _cache.clear()            # one traced step at a time (the fp32 one holds 40 GB of traced tensors)
        torch.cuda.empty_cache()
        from paper_1812_07816_amd import unet
        x = si.normal(5, 0, (N, VOL, VOL, VOL, 4), bf16=True)
        labels = si.ellipsoid_labels(5, 1, N, VOL)
        ws = si.unet_weights(5, CH)
        step = unet.UNetStep(N, VOL, CH, ws, parity.to_device(x, not f32), torch.from_numpy(labels).cuda(), swap=False, norm=True,
                             dtype=torch.float32 if f32 else torch.bfloat16)
        wanted = set()
        for name, (src, *_r) in LAYERS.items():
            wanted |= {src + ".a", name + ".z", name + ".stats", name + ".a", name + ".dout", name + ".dz"}
        tr = _Pick(wanted)
        step.run(update=False, trace=tr)
        torch.cuda.synchronize()
        names = [n for n, _ in si.unet_weight_shapes(CH)]
        sums = {op["name"]: op["bwd_sums"].clone() for op in step.ops if op["kind"] == "conv"}
        flags = {op["name"]: (bool(op.get("fused_stats")), bool(op.get("through_norm")), bool(op.get("skip_sums"))) for op in step.ops
                 if op["kind"] in ("conv", "head")}
        _cache.update(f32=f32, tr=tr, w=dict(zip(names, ws)), dw=dict(zip(names, step.dw)), sums=sums, flags=flags, step=step)
    return _cache


def _host(t):
    return t.float().cpu().numpy()


def _pick(t, idx):
    return t.reshape(-1)[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)


def _check(what, got, ref, tol):
    e = oc.rel_err(got, ref)
    print(f"{what}: {e:.2e}", flush=True)
    assert e <= tol, (what, e)


def _means(v):
    """fp64 mean over the voxels of each (sample, channel) of a float32 NDHWC array."""
    return np.mean(v, axis=(1, 2, 3), dtype=np.float64)


def test_which_kernels_deliver_statistics_and_sums(device):
    f = _step()["flags"]
    # statistics from the convolution's store path in every layer checked here; backward sums from the data gradient
    # of the layer above (plane streaming with 32 contracted channels), of the head, and of the stride-2 layer that
    # adds the skip gradient
    assert all(f[n][0] for n in ("enc0.conv1", "enc0.conv2", "dec0.conv1", "dec0.conv2", "enc1.conv2", "enc3.conv2")), f
    assert f["enc0.conv2"][1] and f["dec0.conv2"][1] and f["head"][1] and f["enc1.conv1"][2], f


@pytest.mark.parametrize("name", list(LAYERS))
@pytest.mark.parametrize("f32", [False, True])       # (the precision varies slowest: one traced step per precision)
def test_normalised_layer_of_the_headline_step(device, f32, name):
    """f32: the same step in fp32 (the bench's fp32 row with the normalisation), where statistics and sums come from
    passes of their own; element-wise tolerance 2e-4."""
    c = _step(f32)
    tol = 2e-4 if f32 else TOL
    tr, w = c["tr"], c["w"][name]
    src, cin, cout, s, level, sums_from = LAYERS[name]
    vin = VOL >> level
    g = oc.shape(N, vin, vin, vin, cin, cout, 3, s, 1)
    a_in = _host(tr[src + ".a"])
    z = _host(tr[name + ".z"])
    # 1. the convolution (raw output, before the normalisation)
    idx = parity.structured_and_random(z.shape, N_SAMPLES, 31)
    _check(f"{name} conv", z.reshape(-1)[idx].astype(np.float64), oc.fwd_at(g, a_in, w, idx), tol)
    # 2. statistics of the stored output against its fp64 mean and variance
    mean = _means(z)
    var = np.mean(z * z, axis=(1, 2, 3), dtype=np.float64) - mean * mean
    rstd = 1.0 / np.sqrt(var + ou.IN_EPS)
    st = tr[name + ".stats"].cpu().numpy().astype(np.float64)
    e_mean = np.abs(st[..., 0] - mean).max() / np.sqrt(var).max()
    e_rstd = np.abs(st[..., 1] / rstd - 1.0).max()
    print(f"{name} statistics: mean {e_mean:.2e} of the spread, rstd {e_rstd:.2e}", flush=True)
    assert e_mean <= 1e-5 and e_rstd <= 1e-5
    # 3. normalisation + LeakyReLU, from the stored z and the exact statistics
    C = cout
    ch = idx % C
    smp = idx // (vin * vin * vin * C)
    xh = (z.reshape(-1)[idx].astype(np.float64) - mean[smp, ch]) * rstd[smp, ch]
    _check(f"{name} norm fwd", _pick(tr[name + ".a"], idx), np.where(xh > 0, xh, SLOPE * xh), tol)
    del z
    # 4. backward sums (from: sums_from) against the fp64 means of g and g * xhat of the stored tensors
    a = _host(tr[name + ".a"])
    da = _host(tr[name + ".dout"])
    xhat = np.where(a > 0, a, a / np.float32(SLOPE))
    gg = np.where(a > 0, da, np.float32(SLOPE) * da)
    m1, m2 = _means(gg), np.mean(gg * xhat, axis=(1, 2, 3), dtype=np.float64)
    sd1 = np.sqrt(np.mean(gg * gg, axis=(1, 2, 3), dtype=np.float64))
    sd2 = np.sqrt(np.mean((gg * xhat) ** 2, axis=(1, 2, 3), dtype=np.float64))
    fused_sums = sums_from != "a reduction pass of its own" and not f32
    if fused_sums:
        got = c["sums"][name].cpu().numpy().astype(np.float64)
        e1, e2 = (np.abs(got[..., 0] - m1) / sd1).max(), (np.abs(got[..., 1] - m2) / sd2).max()
        print(f"{name} backward sums from {sums_from}: mean g {e1:.2e}, mean g xhat {e2:.2e} of the spread", flush=True)
        assert e1 <= 1e-5 and e2 <= 1e-5
    # 5. the normalisation's backward pass on sampled elements, with the exact means
    gs, xs = gg.reshape(-1)[idx].astype(np.float64), xhat.reshape(-1)[idx].astype(np.float64)
    dz_ref = rstd[smp, ch] * (gs - m1[smp, ch] - xs * m2[smp, ch])
    _check(f"{name} norm bwd", _pick(tr[name + ".dz"], idx), dz_ref, tol)
    del a, da, xhat, gg
    # 6. weight gradient from the saved input and the gradient the step fed it
    dz = _host(tr[name + ".dz"])
    dw = c["dw"][name]
    total = dw.numel()
    widx = np.unique(np.concatenate([[0, total - 1], np.random.default_rng(32).integers(0, total, size=16)]))
    # (fp32: an entry is a sum of 1.4e7 products accumulated in fp32, 1.4e4 of them one after the other in a workgroup's
    # accumulator and the 512 to 1024 partial sums in order.  Behind a normalisation the gradient dz sums to zero over
    # each channel, so the entries are what is left of heavy cancellation: measured 1e-6 to 2e-4 of the entries' size,
    # the same with the partial sums added in double)
    _check(f"{name} wgrad", _pick(dw, widx), oc.wgrad_at(g, a_in, dz, widx), 1e-3 if f32 else tol)


def test_release_the_traced_step(device):
    _cache.clear()
    torch.cuda.empty_cache()
