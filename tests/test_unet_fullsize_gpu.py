"""The whole training step at its own shapes (192^3 and 208^3, N = 2) against the fp64 oracle, teacher-forced and
sampled: the step runs once with a trace of the tensors around a set of ops, and every such op is compared with the
oracle's definition of it applied to the tensors the step itself fed it, on the tile seams plus a few thousand random
outputs (a full fp64 pass of these layers would take hours).  The ops are the ones whose kernel variant or unit
mapping differs from what the reduced-volume step tests reach: the level-0 layers at batch 2 (first layer, 32->32
with the LeakyReLU derivative in its store path, the virtual concatenation 64->32, the head), the stride-2 layer that
adds the skip gradient in its data gradient, an up-sampling layer, and the 24^3 / 12^3 layers, which at N = 2 run the
streamed-weight kernel (512->256 included)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from tests import parity

pytestmark = pytest.mark.gpu

CH = [32, 64, 128, 256, 320]
N = 2
SLOPE = 0.01
TOL = 1e-2
N_SAMPLES = 12000

# convolutions checked: name -> (input tensor, Cin, Cout, stride, level of its input volume)
CONVS = {
    "enc0.conv1": ("input", 4, 32, 1, 0),
    "enc0.conv2": ("enc0.conv1", 32, 32, 1, 0),
    "enc1.conv1": ("enc0.conv2", 32, 64, 2, 0),
    "enc3.conv2": ("enc3.conv1", 256, 256, 1, 3),
    "enc4.conv1": ("enc3.conv2", 256, 320, 2, 3),
    "enc4.conv2": ("enc4.conv1", 320, 320, 1, 4),
    "dec3.conv1": ("dec3.cat", 512, 256, 1, 3),
    "dec0.conv1": ("dec0.cat", 64, 32, 1, 0),
    "dec0.conv2": ("dec0.conv1", 32, 32, 1, 0),
}
# the second convolution of a level hands the gradient down with the LeakyReLU derivative of the first applied
THROUGH = {"enc0.conv2", "enc3.conv2", "enc4.conv2", "dec0.conv2"}
# the stride-2 convolutions that read a skip tensor add the decoder's gradient of it in their data-gradient call
SKIP_READERS = {"enc1.conv1", "enc4.conv1"}
EXPECTED_KERNELS_192 = {
    "enc3.conv2": "mfma_plane_stream", "dec3.conv1": "mfma_plane_stream", "enc4.conv2": "mfma_plane_stream",
}


class _Pick(dict):
    """Keeps only the wanted entries of the step's trace (the others are dropped as they come)."""
    keep_fused = True

    def __init__(self, wanted):
        super().__init__()
        self.wanted = set(wanted)

    def __setitem__(self, k, v):
        if k in self.wanted:
            super().__setitem__(k, v)


def _wanted():
    w = {"input.a", "head.a", "head.dout", "head.din", "loss.din", "dec0.up.a", "dec0.up.dout", "dec0.up.din", "dec1.conv2.a"}
    for name, (src, *_r) in CONVS.items():
        w |= {src + ".a", name + ".a", name + ".dz", name + ".din", name + ".skip_add"}
    return w


_cache = {}


def _step(vol):
    """One traced step per volume, kept for the tests of this module (about 15 GB of traced tensors per volume stay
    on the GPU until the last test of the module lets go of them)."""
    if vol not in _cache:
        from paper_1812_07816_amd import unet
        config = 5 if vol == 192 else 6
        x = si.normal(config, 0, (N, vol, vol, vol, 4), bf16=True)
        labels = si.ellipsoid_labels(config, 1, N, vol)
        ws = si.unet_weights(config, CH)
        xd = parity.to_device(x, True)
        step = unet.UNetStep(N, vol, CH, ws, xd, torch.from_numpy(labels).cuda(), swap=False)
        tr = _Pick(_wanted())
        step.run(update=False, trace=tr)
        torch.cuda.synchronize()
        names = [n for n, _ in si.unet_weight_shapes(CH)]
        _cache[vol] = dict(tr=tr, w=dict(zip(names, ws)), dw=dict(zip(names, step.dw)), loss=float(step.loss.item()),
                           labels=labels, step=step)
    return _cache[vol]


def _host(t):
    return t.float().cpu().numpy()


def _pick(t, idx):
    return t.reshape(-1)[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)


def _lrelu(v):
    return np.where(v > 0, v, SLOPE * v)


def _check(what, got, ref):
    e = oc.rel_err(got, ref)
    print(f"{what}: {e:.2e}", flush=True)
    assert e <= TOL, (what, e)


@pytest.mark.parametrize("name", list(CONVS))
@pytest.mark.parametrize("vol", [192, 208])       # (the volume varies slowest: one traced step per volume)
def test_convolution_ops_of_the_full_size_step(device, vol, name):
    from paper_1812_07816_amd import conv3d as mc
    c = _step(vol)
    tr, w = c["tr"], c["w"][name]
    src, cin, cout, s, level = CONVS[name]
    vin = vol >> level
    g = oc.shape(N, vin, vin, vin, cin, cout, 3, s, 1)
    if vol == 192 and name in EXPECTED_KERNELS_192:
        d = mc.make_desc(N, vin, vin, vin, cin, cout, 3, s, 1, torch.bfloat16)
        assert mc.kernel_name(d, 0) == mc.kernel_name(d, 1) == EXPECTED_KERNELS_192[name]
    a_in, a_out, dz = _host(tr[src + ".a"]), tr[name + ".a"], _host(tr[name + ".dz"])
    # forward: convolution + LeakyReLU
    idx = parity.structured_and_random(a_out.shape, N_SAMPLES, 11)
    _check(f"{vol} {name} fwd", _pick(a_out, idx), _lrelu(oc.fwd_at(g, a_in, w, idx)))
    # weight gradient from the saved input and the gradient the step fed it
    dw = c["dw"][name]
    total = dw.numel()
    widx = np.unique(np.concatenate([[0, total - 1], np.random.default_rng(12).integers(0, total, size=24)]))
    _check(f"{vol} {name} wgrad", _pick(dw, widx), oc.wgrad_at(g, a_in, dz, widx))
    if name == "enc0.conv1":
        assert name + ".din" not in tr       # the network input needs no gradient
        return
    din = tr[name + ".din"]
    idx = parity.structured_and_random(din.shape, N_SAMPLES, 13)
    ref = oc.dgrad_at(g, dz, w, idx)
    src_a = a_in.reshape(-1)[idx]
    if name in THROUGH:                      # times the LeakyReLU derivative of the layer below
        ref = ref * np.where(src_a > 0, 1.0, SLOPE)
    if name + ".skip_add" in tr:             # the skip connection's second gradient joins in the same call
        assert name in SKIP_READERS
        # (the call is defined as the stored, i.e. bf16-rounded, data gradient plus the second gradient, times the
        # derivative: the reference takes the same storage rounding of the intermediate)
        ref = si.bf16_round(ref.astype(np.float32)).astype(np.float64)
        ref = (ref + _pick(tr[name + ".skip_add"], idx)) * np.where(src_a > 0, 1.0, SLOPE)
    else:
        assert name not in SKIP_READERS
    _check(f"{vol} {name} dgrad", _pick(din, idx), ref)


@pytest.mark.parametrize("vol", [192, 208])
def test_head_loss_and_upsampling_of_the_full_size_step(device, vol):
    from oracle import unet as ou
    c = _step(vol)
    tr = c["tr"]
    # 1x1x1 head, all three passes
    gh = oc.shape(N, vol, vol, vol, 32, 3, 1, 1, 0)
    a = _host(tr["dec0.conv2.a"])
    idx = parity.structured_and_random(tr["head.a"].shape, N_SAMPLES, 21)
    _check(f"{vol} head fwd", _pick(tr["head.a"], idx), oc.fwd_at(gh, a, c["w"]["head"], idx))
    dlog = _host(tr["head.dout"])
    _check(f"{vol} head wgrad", _host(c["dw"]["head"]).ravel(), oc.wgrad_at(gh, a, dlog, np.arange(96)))
    idx = parity.structured_and_random(tr["head.din"].shape, N_SAMPLES, 22)
    _check(f"{vol} head dgrad", _pick(tr["head.din"], idx),
           oc.dgrad_at(gh, dlog, c["w"]["head"], idx) * np.where(a.reshape(-1)[idx] > 0, 1.0, SLOPE))
    # sigmoid + soft Dice on the step's own logits: loss and gradient (full; the loss is a global sum)
    loss_ref, dl_ref = ou.dice_loss(_host(tr["head.a"]).astype(np.float64), c["labels"])
    assert abs(c["loss"] - loss_ref) <= 1e-5
    idx = parity.structured_and_random(tr["loss.din"].shape, N_SAMPLES, 23)
    _check(f"{vol} loss grad", _pick(tr["loss.din"], idx), dl_ref.reshape(-1)[idx])
    del dl_ref
    # up-sampling 64 -> 32 into the level-0 volume: transposed convolution = data gradient of the k2/s2 convolution
    gu = oc.shape(N, vol, vol, vol, 32, 64, 2, 2, 0)
    z, wu = _host(tr["dec1.conv2.a"]), c["w"]["dec0.up"]
    idx = parity.structured_and_random(tr["dec0.up.a"].shape, N_SAMPLES, 24)
    _check(f"{vol} dec0.up fwd", _pick(tr["dec0.up.a"], idx), oc.dgrad_at(gu, z, wu, idx))
    du = _host(tr["dec0.up.dout"])
    widx = np.unique(np.concatenate([[0, wu.size - 1], np.random.default_rng(25).integers(0, wu.size, size=24)]))
    _check(f"{vol} dec0.up wgrad", _pick(c["dw"]["dec0.up"], widx), oc.wgrad_at(gu, du, z, widx))
    idx = parity.structured_and_random(tr["dec0.up.din"].shape, N_SAMPLES, 26)
    _check(f"{vol} dec0.up dgrad", _pick(tr["dec0.up.din"], idx), oc.fwd_at(gu, du, wu, idx))


def test_release_the_traced_steps(device):
    _cache.clear()
    torch.cuda.empty_cache()
