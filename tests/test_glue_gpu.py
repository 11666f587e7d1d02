"""GPU parity of the elementwise / loss / optimiser entry points against the
fp64 oracle's formulas (oracle/unet.py) on seeded inputs."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import unet as ou

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def glue():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1812_07816_amd import glue as g
    return g


def dev(a):
    return torch.from_numpy(si.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16).reshape(a.shape)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def test_leaky_relu_fwd_bwd(glue):
    x = si.normal(50, 0, (3, 5, 7, 9, 16), bf16=True)
    da = si.normal(50, 1, x.shape, bf16=True)
    a = dev(x)
    glue.leaky_relu_fwd(a)
    ref = ou._lrelu(x.astype(np.float64))
    assert np.max(np.abs(host(a) - ref)) <= 2 ** -8 * np.max(np.abs(ref))
    g = dev(da)
    glue.leaky_relu_bwd(g, a)
    refg = ou._lrelu_grad(x.astype(np.float64), da.astype(np.float64))
    assert np.max(np.abs(host(g) - refg)) <= 2 ** -8 * np.max(np.abs(refg))


def test_concat_split_add(glue):
    a = si.normal(50, 2, (2, 3, 4, 5, 32), bf16=True)
    b = si.normal(50, 3, (2, 3, 4, 5, 64), bf16=True)
    out = torch.empty((2, 3, 4, 5, 96), dtype=torch.bfloat16, device="cuda")
    glue.concat_channels(dev(a), dev(b), out)
    assert np.array_equal(host(out), np.concatenate([a, b], axis=-1).astype(np.float64))
    a2, b2 = torch.empty_like(dev(a)), torch.empty_like(dev(b))
    glue.split_channels(out, a2, b2)
    assert np.array_equal(host(a2), a.astype(np.float64)) and np.array_equal(host(b2), b.astype(np.float64))
    c = si.normal(50, 4, a.shape, bf16=True)
    s = dev(a)
    glue.add_inplace(s, dev(c))
    ref = a.astype(np.float64) + c.astype(np.float64)
    assert np.max(np.abs(host(s) - ref)) <= 2 ** -8 * np.max(np.abs(ref))


def test_slice_and_skip_gradient(glue):
    shape = (2, 3, 5, 7)
    dcat = si.normal(50, 5, shape + (96,), bf16=True)
    for off, C in ((0, 32), (32, 64), (64, 32)):
        out = torch.empty(shape + (C,), dtype=torch.bfloat16, device="cuda")
        glue.slice_channels(dev(dcat), off, out)
        assert np.array_equal(host(out), dcat[..., off:off + C].astype(np.float64))
    # gradient of a skip tensor: (encoder-path gradient + its half of the concatenated gradient) * LeakyReLU'(a)
    da = si.normal(50, 6, shape + (64,), bf16=True)
    a = si.normal(50, 7, shape + (64,), bf16=True)
    a[0, 0, 0, 0, :4] = 0.0                       # zero counts as the negative branch
    g = dev(da)
    glue.skip_grad(g, dev(dcat), 32, dev(a))
    ref = ou._lrelu_grad(a.astype(np.float64), da.astype(np.float64) + dcat[..., 32:].astype(np.float64))
    assert np.max(np.abs(host(g) - ref)) <= 2 ** -8 * np.max(np.abs(ref))
    neg = a <= 0
    assert neg.any() and np.max(np.abs(host(g)[neg] - ref[neg])) <= 2 ** -8 * np.max(np.abs(ref[neg]))


@pytest.mark.parametrize("vol", [8, 24])
def test_dice_loss_and_gradient(glue, vol):
    N = 2
    logits = si.normal(50, 5, (N, vol, vol, vol, 3), std=2.0, bf16=True)
    labels = si.ellipsoid_labels(50, 6, N, vol)
    loss_ref, grad_ref = ou.dice_loss(logits.astype(np.float64), labels)
    lg, lb = dev(logits), torch.from_numpy(labels).cuda()
    ws = glue.dice_workspace()
    sums = torch.empty(9, dtype=torch.float32, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    glue.dice_loss(lg, lb, ws, sums, loss)
    assert abs(float(loss.item()) - loss_ref) <= 1e-5
    loss2 = torch.empty(1, dtype=torch.float32, device="cuda")
    glue.dice_loss(lg, lb, ws, sums, loss2)
    assert loss2.item() == loss.item()            # fixed reduction order
    d = torch.empty_like(lg)
    glue.dice_grad(lg, lb, sums, d)
    err = np.max(np.abs(host(d) - grad_ref)) / np.max(np.abs(grad_ref))
    assert err <= 1e-2, err


def test_sgd_update(glue):
    rng = np.random.default_rng(7)
    w = rng.standard_normal(1000).astype(np.float32)
    dw = rng.standard_normal(1000).astype(np.float32)
    w32, d32 = torch.from_numpy(w).cuda(), torch.from_numpy(dw).cuda()
    w16 = torch.empty(1000, dtype=torch.bfloat16, device="cuda")
    glue.sgd_update(w32, d32, w16, 0.125)
    ref = w - np.float32(0.125) * dw
    assert np.allclose(w32.cpu().numpy(), ref, rtol=1e-6, atol=1e-7)
    assert np.array_equal(w16.float().cpu().numpy(), si.bf16_round(w32.cpu().numpy()))


def test_adam_update_over_several_steps(glue):
    rng = np.random.default_rng(11)
    n = 4099
    w = rng.standard_normal(n).astype(np.float32)
    w32 = torch.from_numpy(w).cuda()
    m32, v32 = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    w16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    rw, rm, rv = w.astype(np.float64), np.zeros(n), np.zeros(n)
    # the C ABI takes the coefficients as floats: the oracle gets the same (float32-rounded) values
    b1, b2, eps, lr = (float(np.float32(c)) for c in (0.9, 0.999, 1e-8, 5e-4))
    mag = np.zeros(n)     # the first moment is a sum of signed terms: its fp32 error is relative to the terms' magnitudes
    for step in range(1, 6):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-4, 2, size=n)).astype(np.float32)    # gradients over six decades
        mag = b1 * mag + (1.0 - b1) * np.abs(g)
        glue.adam_update(w32, torch.from_numpy(g).cuda(), m32, v32, w16, 5e-4, step)
        rw, rm, rv = ou.adam_step(rw, g.astype(np.float64), rm, rv, lr, step, b1, b2, eps)
        assert np.allclose(w32.cpu().numpy(), rw, rtol=2e-6, atol=1e-7), step
        assert np.all(np.abs(m32.cpu().numpy() - rm) <= 1e-6 * mag) and np.allclose(v32.cpu().numpy(), rv, rtol=1e-5, atol=1e-20)
    assert np.array_equal(w16.float().cpu().numpy(), si.bf16_round(w32.cpu().numpy()))
    # the first step moves every weight by lr in the direction of its gradient's sign, whatever the gradient's size
    w1 = torch.from_numpy(w).cuda()
    g1 = torch.from_numpy(np.where(np.arange(n) % 2 == 0, 3e-3, -7.0).astype(np.float32)).cuda()
    glue.adam_update(w1, g1, torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda"), w16, 0.25, 1)
    assert np.allclose(w1.cpu().numpy() - w, np.where(np.arange(n) % 2 == 0, -0.25, 0.25), rtol=1e-4)


@pytest.mark.parametrize("shape", [(2, 5, 6, 7, 32), (1, 4, 4, 6, 320), (2, 3, 3, 3, 8), (1, 16, 16, 24, 64)])
def test_instance_norm_forward_and_backward(glue, shape):
    N, C = shape[0], shape[-1]
    idx = [(2, 5, 6, 7, 32), (1, 4, 4, 6, 320), (2, 3, 3, 3, 8), (1, 16, 16, 24, 64)].index(shape)
    scale = np.linspace(0.05, 20.0, C)                         # channels of very different spread and offset
    z = si.bf16_round((si.normal(51, 10 * idx, shape) * scale + np.linspace(-3, 3, C)).astype(np.float32))
    da = si.normal(51, 10 * idx + 1, shape, bf16=True)
    z64 = z.astype(np.float64)
    xhat, mean, rstd = ou.instnorm(z64)
    ws = glue.instnorm_workspace(N, C)
    stats = torch.zeros((N, C, 2), dtype=torch.float32, device="cuda")
    a = dev(z)
    glue.instnorm_stats(a, stats, ws)
    st = stats.cpu().numpy().astype(np.float64)
    assert np.allclose(st[..., 0], mean, rtol=1e-5, atol=1e-5 * np.abs(z64).max()) and np.allclose(st[..., 1], rstd, rtol=1e-4)
    glue.instnorm_lrelu_fwd(a, stats)
    ref = ou._lrelu(xhat)
    assert np.max(np.abs(host(a) - ref)) <= 2 ** -8 * np.max(np.abs(ref))
    # backward from the stored (bf16) activation: the oracle gets the normalised value back from the same tensor
    g = dev(da)
    glue.instnorm_lrelu_bwd(g, a, stats, ws)
    refd = ou.instnorm_lrelu_bwd(ou.lrelu_inverse(host(a)), rstd, da.astype(np.float64))
    err = np.max(np.abs(host(g) - refd), axis=(0, 1, 2, 3)) / np.max(np.abs(refd), axis=(0, 1, 2, 3))     # per channel: the scales differ by 400x
    assert err.max() <= 1e-2, err.max()
    # reductions in a fixed order: the same bits every time
    g2 = dev(da)
    glue.instnorm_lrelu_bwd(g2, a, stats, ws)
    assert torch.equal(g.view(torch.int16), g2.view(torch.int16))


@pytest.mark.parametrize("shape", [(2, 5, 6, 7, 32), (1, 4, 4, 6, 320), (2, 3, 3, 3, 8), (1, 16, 16, 24, 64)])
def test_instance_norm_fp32(glue, shape):
    """The fp32 entry points against the fp64 definition, at fp32 accuracy."""
    N, C = shape[0], shape[-1]
    scale = np.linspace(0.05, 20.0, C)
    z = (si.normal(52, C, shape) * scale + np.linspace(-3, 3, C)).astype(np.float32)
    da = si.normal(52, C + 1, shape).astype(np.float32)
    xhat, mean, rstd = ou.instnorm(z.astype(np.float64))
    ws = glue.instnorm_workspace(N, C)
    stats = torch.zeros((N, C, 2), dtype=torch.float32, device="cuda")
    a = torch.from_numpy(z).cuda()
    glue.instnorm_stats(a, stats, ws)
    st = stats.cpu().numpy().astype(np.float64)
    assert np.allclose(st[..., 0], mean, rtol=1e-5, atol=1e-6 * np.abs(z).max()) and np.allclose(st[..., 1], rstd, rtol=1e-4)
    glue.instnorm_lrelu_fwd(a, stats)
    ref = ou._lrelu(xhat)
    # (one-pass variance from fp32 block sums: a channel whose offset is 60 standard deviations loses 1e-4 of rstd)
    assert np.max(np.abs(a.cpu().numpy() - ref)) <= 2e-4 * np.max(np.abs(ref))
    g = torch.from_numpy(da).cuda()
    glue.instnorm_lrelu_bwd(g, a, stats, ws)
    refd = ou.instnorm_lrelu_bwd(ou.lrelu_inverse(a.cpu().numpy().astype(np.float64)), rstd, da.astype(np.float64))
    err = np.max(np.abs(g.cpu().numpy() - refd), axis=(0, 1, 2, 3)) / np.max(np.abs(refd), axis=(0, 1, 2, 3))
    assert err.max() <= 5e-4, err.max()
    g2 = torch.from_numpy(da).cuda()
    glue.instnorm_lrelu_bwd(g2, a, stats, ws)
    assert torch.equal(g, g2)
