"""fp64 oracle of the whole training step (test infrastructure only).

Network (the paper's 3D U-Net, Section 4.1, in the reading fixed for this
build): L encoder levels with two 3x3x3 pad-1 convolutions each, the first
one of every level but the top with stride 2; decoder levels with a 2x2x2
stride-2 transposed convolution, channel concatenation [upsampled, skip],
and two 3x3x3 convolutions; a 1x1x1 head; LeakyReLU (slope 0.01) after every
3x3x3 convolution; no bias, no normalisation; sigmoid per class and the soft
Dice loss built on the Dice coefficient of Section 4.3,
    D_c = (2 sum p t + eps) / (sum p + sum t + eps),  loss = 1 - mean_c D_c,
sums over samples and voxels; plain SGD.  Everything in float64; the
convolutions are the direct-loop oracle of conv3d.py, the rest is written out
with numpy elementwise operations and sums.
"""
import numpy as np

from . import conv3d as oc

SLOPE = 0.01
DICE_EPS = 1e-5


def exact(a):
    return a


def bf16(a):
    """Values rounded to the nearest bfloat16 (ties to even), returned as float64.
    Passed as `q` to forward/backward it puts the step's storage roundings where
    the bf16 pipeline has them (every activation and activation gradient that
    is written to memory), so that the sign decisions of the LeakyReLU are
    taken on the same numbers on both sides of a comparison; the sums inside a
    convolution, the loss and the weight gradients stay in float64."""
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def _lrelu(z):
    return np.where(z > 0, z, SLOPE * z)


def _lrelu_grad(z, da):
    return np.where(z > 0, da, SLOPE * da)


IN_EPS = 1e-5


def instnorm(z, eps=IN_EPS):
    """Instance normalisation without scale and shift (Section 4.1): per sample and channel, over the voxels,
    xhat = (z - mean) / sqrt(var + eps) with the biased variance.  Returns (xhat, mean, rstd), the last two [N, C]."""
    ax = (1, 2, 3)
    mean = z.mean(axis=ax)
    var = ((z - mean[:, None, None, None, :]) ** 2).mean(axis=ax)
    rstd = 1.0 / np.sqrt(var + eps)
    return (z - mean[:, None, None, None, :]) * rstd[:, None, None, None, :], mean, rstd


def lrelu_inverse(a):
    """The argument of the LeakyReLU that produced a (its slope is positive, so it is one to one)."""
    return np.where(a > 0, a, a / SLOPE)


def instnorm_lrelu_bwd(xhat, rstd, da):
    """Gradient with respect to z of a = lrelu(instnorm(z)), given da, xhat = instnorm(z) and rstd [N, C]:
    g = da * lrelu'(xhat);  dz = rstd * (g - mean_v(g) - xhat * mean_v(g * xhat))."""
    ax = (1, 2, 3)
    g = np.where(xhat > 0, da, SLOPE * da)
    m1 = g.mean(axis=ax)[:, None, None, None, :]
    m2 = (g * xhat).mean(axis=ax)[:, None, None, None, :]
    return rstd[:, None, None, None, :] * (g - m1 - xhat * m2)


def forward(x, weights, channels, q=exact, norm=False):
    """x [N, V, V, V, Cin] float64; weights in the order of
    synth_inputs.unet_weight_shapes; q: rounding applied to every tensor the
    step stores (exact = none); norm: instance normalisation between every
    3x3x3 convolution and its LeakyReLU.  Returns (logits, saved) where saved
    holds what the backward pass needs."""
    L = len(channels)
    N, V = x.shape[0], x.shape[1]
    it = iter(weights)
    saved = {"enc": [], "dec": {}, "skip": {}}
    a, vol = np.asarray(x, dtype=np.float64), V

    def conv(a, w, vol, s):
        cout, cin = w.shape[0], w.shape[4]
        g = oc.shape(N, vol, vol, vol, cin, cout, 3, s, 1)
        z = q(oc.fwd(g, a, w))
        if norm:
            xhat, _, rstd = instnorm(z)
            out = q(_lrelu(xhat))
            return out, (g, a, w, out, rstd)      # the activated tensor and the statistics are what is kept
        return q(_lrelu(z)), (g, a, w, z)

    for l in range(L):
        a, r1 = conv(a, next(it), vol, 1 if l == 0 else 2)
        if l > 0:
            vol //= 2
        a, r2 = conv(a, next(it), vol, 1)
        saved["enc"].append((r1, r2))
        if l < L - 1:
            saved["skip"][l] = a
    for l in range(L - 2, -1, -1):
        w_up = next(it)
        vol *= 2
        g = oc.shape(N, vol, vol, vol, channels[l], channels[l + 1], 2, 2, 0)
        u = q(oc.dgrad(g, a, w_up))         # transposed convolution = data gradient of the k2/s2 convolution
        rup = (g, a, w_up)
        a = np.concatenate([u, saved["skip"][l]], axis=-1)
        a, r1 = conv(a, next(it), vol, 1)
        a, r2 = conv(a, next(it), vol, 1)
        saved["dec"][l] = (rup, r1, r2)
    w_head = next(it)
    g = oc.shape(N, vol, vol, vol, channels[0], w_head.shape[0], 1, 1, 0)
    logits = q(oc.fwd(g, a, w_head))
    saved["head"] = (g, a, w_head)
    return logits, saved


def dice_loss(logits, labels):
    """(loss, dloss/dlogits) of the sigmoid + soft Dice loss."""
    e = np.exp(-np.abs(logits))
    p = np.where(logits >= 0, 1.0 / (1.0 + e), e / (1.0 + e))   # sigmoid without overflow
    t = np.asarray(labels, dtype=np.float64)
    axes = (0, 1, 2, 3)
    inter, sp, st = (p * t).sum(axes), p.sum(axes), t.sum(axes)
    den = sp + st + DICE_EPS
    dice = (2.0 * inter + DICE_EPS) / den
    loss = 1.0 - dice.mean()
    C = logits.shape[-1]
    # d dice_c / d p = (2 t den - (2 inter + eps)) / den^2
    dp = -(2.0 * t * den - (2.0 * inter + DICE_EPS)) / (den * den) / C
    return loss, dp * p * (1.0 - p)


def backward(saved, dlogits, channels, q=exact, trace=None):
    """Weight gradients in the order of the weights (the gradient with respect
    to the network input is not formed).  q as in forward."""
    L = len(channels)
    dw = {}

    def conv_bwd(rec, da, name, need_dx=True):
        if len(rec) == 5:       # with instance normalisation: (geometry, input, weights, activated output, rstd)
            g, a, w, out, rstd = rec
            dz = q(instnorm_lrelu_bwd(lrelu_inverse(out), rstd, da))
        else:
            g, a, w, z = rec
            dz = q(_lrelu_grad(z, da))
        if trace is not None:
            trace[name + ".dz"] = dz
        dw[name] = oc.wgrad(g, a, dz)
        return q(oc.dgrad(g, dz, w)) if need_dx else None

    g, a, w = saved["head"]
    dlogits = q(dlogits)
    if trace is not None:
        trace["dlogits"] = dlogits
    dw["head"] = oc.wgrad(g, a, dlogits)
    da = q(oc.dgrad(g, dlogits, w))
    dskip = {}
    for l in range(0, L - 1):
        rup, r1, r2 = saved["dec"][l]
        da = conv_bwd(r2, da, f"dec{l}.conv2")
        da = conv_bwd(r1, da, f"dec{l}.conv1")
        c = channels[l]
        d_up, dskip[l] = da[..., :c], da[..., c:]
        g, a_small, w_up = rup
        dw[f"dec{l}.up"] = oc.wgrad(g, d_up, a_small)   # roles: x := gradient of the upsampled map, dy := the small input
        da = q(oc.fwd(g, d_up, w_up))
    for l in range(L - 1, -1, -1):
        if l < L - 1:
            da = q(da + dskip[l])
        r1, r2 = saved["enc"][l]
        da = conv_bwd(r2, da, f"enc{l}.conv2")
        da = conv_bwd(r1, da, f"enc{l}.conv1", need_dx=l > 0)
    order = [f"enc{l}.conv{i}" for l in range(L) for i in (1, 2)]
    for l in range(L - 2, -1, -1):
        order += [f"dec{l}.up", f"dec{l}.conv1", f"dec{l}.conv2"]
    order.append("head")
    return [dw[k] for k in order]


def train_step(x, labels, weights, channels, lr, q=exact, norm=False):
    """One SGD step: (loss, weight gradients, updated weights)."""
    w64 = [np.asarray(w, dtype=np.float64) for w in weights]
    logits, saved = forward(x, w64, channels, q, norm)
    loss, dlogits = dice_loss(logits, labels)
    grads = backward(saved, dlogits, channels, q)
    return loss, grads, [w - lr * g for w, g in zip(w64, grads)]


def adam_step(w, g, m, v, lr, step, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (the optimiser of Section 4.1) in fp64: returns (w, m, v) after step `step` (counted from 1)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v
