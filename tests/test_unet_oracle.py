"""Pins of the whole-step oracle (oracle/unet.py): the loss against the Dice
coefficient of Section 4.3 on binary predictions, its gradient and the whole
backward pass against central finite differences of the forward pass."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import unet as ou


def test_soft_dice_reduces_to_dice_coefficient_on_binary_predictions():
    # logits +-40 give p in {0, 1} to fp64 precision; Dice = |P and T| / ((|P| + |T|) / 2)  (Section 4.3)
    rng = np.random.default_rng(1)
    t = (rng.random((2, 4, 5, 6, 3)) < 0.4)
    pred = (rng.random(t.shape) < 0.5)
    logits = np.where(pred, 40.0, -40.0)
    loss, _ = ou.dice_loss(logits, t.astype(np.uint8))
    dice = [(pred[..., c] & t[..., c]).sum() / ((pred[..., c].sum() + t[..., c].sum()) / 2) for c in range(3)]
    assert abs(loss - (1.0 - np.mean(dice))) < 1e-6


def test_dice_loss_of_perfect_and_of_disjoint_prediction():
    t = np.zeros((1, 4, 4, 4, 3), dtype=np.uint8)
    t[:, :2] = 1
    perfect = np.where(t > 0, 40.0, -40.0)
    assert ou.dice_loss(perfect, t)[0] < 1e-9
    assert abs(ou.dice_loss(-perfect, t)[0] - 1.0) < 1e-6


def test_dice_gradient_matches_finite_differences():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((2, 3, 4, 5, 3))
    t = (rng.random(logits.shape) < 0.3).astype(np.uint8)
    _, g = ou.dice_loss(logits, t)
    h = 1e-6
    for idx in [(0, 0, 0, 0, 0), (1, 2, 3, 4, 2), (0, 1, 2, 3, 1), (1, 0, 3, 0, 0)]:
        a, b = logits.copy(), logits.copy()
        a[idx] += h; b[idx] -= h
        fd = (ou.dice_loss(a, t)[0] - ou.dice_loss(b, t)[0]) / (2 * h)
        assert abs(fd - g[idx]) <= 1e-7 + 1e-5 * abs(g[idx])


@pytest.mark.parametrize("channels", [[2, 3], [2, 3, 4]])
def test_backward_matches_finite_differences_of_forward(channels):
    # tiny network: every kind of layer (strided conv, up-sampling, concatenation, head) is on the path
    V = 4 * 2 ** (len(channels) - 1) // 2
    V = max(V, 2 ** (len(channels) - 1) * 2)
    rng = np.random.default_rng(3)
    shapes = si.unet_weight_shapes(channels, in_ch=2, classes=3)
    ws = [rng.standard_normal(shp) * 0.4 for _, shp in shapes]
    x = rng.standard_normal((2, V, V, V, 2))
    t = (rng.random((2, V, V, V, 3)) < 0.4).astype(np.uint8)
    loss, grads, _ = ou.train_step(x, t, ws, channels, lr=0.0)

    def f(ws_):
        return ou.dice_loss(ou.forward(x, ws_, channels)[0], t)[0]

    h = 1e-5
    for k, (name, shp) in enumerate(shapes):
        for _ in range(2):
            idx = tuple(int(rng.integers(0, n)) for n in shp)
            wp = [w.copy() for w in ws]; wm = [w.copy() for w in ws]
            wp[k][idx] += h; wm[k][idx] -= h
            fd = (f(wp) - f(wm)) / (2 * h)
            assert abs(fd - grads[k][idx]) <= 1e-8 + 2e-4 * abs(fd), (name, idx, fd, grads[k][idx])


def test_sgd_update_and_weight_order():
    channels = [2, 3]
    rng = np.random.default_rng(4)
    shapes = si.unet_weight_shapes(channels, in_ch=2, classes=3)
    assert [n for n, _ in shapes] == ["enc0.conv1", "enc0.conv2", "enc1.conv1", "enc1.conv2", "dec0.up", "dec0.conv1", "dec0.conv2", "head"]
    ws = [rng.standard_normal(shp) * 0.3 for _, shp in shapes]
    x = rng.standard_normal((1, 4, 4, 4, 2))
    t = (rng.random((1, 4, 4, 4, 3)) < 0.5).astype(np.uint8)
    loss, grads, new = ou.train_step(x, t, ws, channels, lr=0.25)
    for w, g, n in zip(ws, grads, new):
        assert g.shape == w.shape
        assert np.allclose(n, w - 0.25 * g, rtol=0, atol=1e-15)


def test_label_generator_shape_and_determinism():
    a = si.ellipsoid_labels(5, 7, 2, 16)
    b = si.ellipsoid_labels(5, 7, 2, 16)
    assert a.dtype == np.uint8 and a.shape == (2, 16, 16, 16, 3)
    assert np.array_equal(a, b) and set(np.unique(a)) <= {0, 1} and a.any()


def test_bf16_rounding_helper():
    # ties to even on the 16th mantissa bit; exact values unchanged; matches the shared input rounding
    a = np.array([1.0, 1.00390625, 1.01171875, -3.0e-5, 123456.789, 0.0])
    r = ou.bf16(a)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625          # 1 + 2^-8 ties down, 1 + 3 * 2^-8 ties up
    assert np.array_equal(r.astype(np.float32), si.bf16_round(a.astype(np.float32)))
    assert np.all(np.abs(r - a) <= np.abs(a) * 2.0 ** -8)


def test_rounded_step_stays_close_to_exact_step():
    channels = [4, 8]
    rng = np.random.default_rng(5)
    ws = [si.bf16_round((rng.standard_normal(shp) * 0.3).astype(np.float32)) for _, shp in si.unet_weight_shapes(channels, in_ch=2)]
    x = si.bf16_round(rng.standard_normal((1, 8, 8, 8, 2)).astype(np.float32))
    t = (rng.random((1, 8, 8, 8, 3)) < 0.4).astype(np.uint8)
    l0, g0, _ = ou.train_step(x, t, ws, channels, 0.0)
    l1, g1, _ = ou.train_step(x, t, ws, channels, 0.0, q=ou.bf16)
    assert abs(l0 - l1) < 1e-2 * abs(l0)
    for a, b in zip(g0, g1):
        assert np.sum(a * b) / np.sqrt(np.sum(a * a) * np.sum(b * b)) > 0.98


def test_adam_step_against_closed_forms():
    """Pins of the Adam oracle (Section 4.1): the first step is -lr * sign(g) up to eps; with a constant gradient the
    bias-corrected moments equal g and g^2 at every step, so every step moves by lr * g / (|g| + eps)."""
    g = np.array([3e-3, -7.0, 0.5, -1e-6])
    w, m, v = np.zeros(4), np.zeros(4), np.zeros(4)
    w1, m1, v1 = ou.adam_step(w, g, m, v, 0.1, 1)
    assert np.allclose(w1, -0.1 * np.sign(g), rtol=1e-2) and np.allclose(m1, 0.1 * g) and np.allclose(v1, 1e-3 * g * g)
    for step in range(1, 8):
        w_new, m, v = ou.adam_step(w, g, m, v, 0.1, step)
        assert np.allclose(w_new - w, -0.1 * g / (np.abs(g) + 1e-8), rtol=1e-9)
        assert np.allclose(m / (1 - 0.9 ** step), g) and np.allclose(v / (1 - 0.999 ** step), g * g)
        w = w_new
    # hand-worked second step with a changing gradient: g1 = 1, g2 = -1, lr = 1, eps -> 0
    w, m, v = ou.adam_step(0.0, 1.0, 0.0, 0.0, 1.0, 1, eps=1e-12)
    w, m, v = ou.adam_step(w, -1.0, m, v, 1.0, 2, eps=1e-12)
    mhat = (0.9 * 0.1 - 0.1) / (1 - 0.81)
    vhat = (0.999 * 0.001 + 0.001) / (1 - 0.999 ** 2)
    assert abs(w - (-1.0 - mhat / np.sqrt(vhat))) < 1e-9


# ---- instance normalisation (Section 4.1) ------------------------------------------------------------------------
def test_instnorm_output_statistics_and_invariances():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((2, 3, 4, 5, 6)) * rng.uniform(0.1, 30.0, size=6) + rng.uniform(-5, 5, size=6)
    xhat, mean, rstd = ou.instnorm(z)
    ax = (1, 2, 3)
    assert np.allclose(xhat.mean(axis=ax), 0.0, atol=1e-12)
    var = z.var(axis=ax)
    assert np.allclose(xhat.var(axis=ax), var / (var + ou.IN_EPS), rtol=1e-12)
    assert np.allclose(mean, z.mean(axis=ax)) and np.allclose(rstd, 1.0 / np.sqrt(var + ou.IN_EPS))
    # a shift per (sample, channel) changes nothing; a scale changes nothing up to eps
    shift = rng.standard_normal((2, 1, 1, 1, 6)) * 100
    assert np.allclose(ou.instnorm(z + shift)[0], xhat, atol=1e-9)
    assert np.allclose(ou.instnorm(z * 1e3)[0], xhat, atol=1e-6)
    # a single sample and channel by hand: values 1, 2, 3, 6 -> mean 3, variance 3.5
    z1 = np.array([1.0, 2.0, 3.0, 6.0]).reshape(1, 1, 2, 2, 1)
    assert np.allclose(ou.instnorm(z1, eps=0.5)[0].ravel(), (np.array([1.0, 2.0, 3.0, 6.0]) - 3.0) / 2.0)


def test_instnorm_lrelu_backward_matches_finite_differences_and_is_orthogonal():
    rng = np.random.default_rng(6)
    z = rng.standard_normal((2, 3, 3, 4, 5)) * 2.0 + 0.7
    da = rng.standard_normal(z.shape)

    def f(z_):
        return float((ou._lrelu(ou.instnorm(z_)[0]) * da).sum())

    xhat, _, rstd = ou.instnorm(z)
    dz = ou.instnorm_lrelu_bwd(xhat, rstd, da)
    h = 1e-6
    for _ in range(12):
        idx = tuple(int(rng.integers(0, n)) for n in z.shape)
        zp, zm = z.copy(), z.copy()
        zp[idx] += h; zm[idx] -= h
        fd = (f(zp) - f(zm)) / (2 * h)
        assert abs(fd - dz[idx]) <= 1e-7 + 1e-5 * abs(fd), (idx, fd, dz[idx])
    # the output does not depend on the mean or (up to eps) the scale of z: the gradient has no component along 1,
    # and along xhat only the part eps / (var + eps) of rstd * sum(g xhat)
    ax = (1, 2, 3)
    assert np.allclose(dz.sum(axis=ax), 0.0, atol=1e-10)
    g = np.where(xhat > 0, da, ou.SLOPE * da)
    along = (dz * xhat).sum(axis=ax)
    assert np.allclose(along, rstd * (g * xhat).sum(axis=ax) * (1.0 - (xhat ** 2).mean(axis=ax)), rtol=1e-9, atol=1e-12)
    assert np.all(np.abs(along) < 1e-4)
    # the kept activation gives the normalised value back
    assert np.allclose(ou.lrelu_inverse(ou._lrelu(xhat)), xhat, rtol=1e-12)


def test_backward_with_instance_normalisation_matches_finite_differences():
    channels = [2, 3, 4]
    V = 8
    rng = np.random.default_rng(8)
    shapes = si.unet_weight_shapes(channels, in_ch=2, classes=3)
    ws = [rng.standard_normal(shp) * 0.4 for _, shp in shapes]
    x = rng.standard_normal((2, V, V, V, 2))
    t = (rng.random((2, V, V, V, 3)) < 0.4).astype(np.uint8)
    loss, grads, _ = ou.train_step(x, t, ws, channels, lr=0.0, norm=True)

    def f(ws_):
        return ou.dice_loss(ou.forward(x, ws_, channels, norm=True)[0], t)[0]

    h = 1e-5
    for k, (name, shp) in enumerate(shapes):
        for _ in range(2):
            idx = tuple(int(rng.integers(0, n)) for n in shp)
            wp = [w.copy() for w in ws]; wm = [w.copy() for w in ws]
            wp[k][idx] += h; wm[k][idx] -= h
            fd = (f(wp) - f(wm)) / (2 * h)
            assert abs(fd - grads[k][idx]) <= 1e-8 + 5e-4 * abs(fd), (name, idx, fd, grads[k][idx])
