"""Pins for the fp64 CPU oracle: everything here checks oracle/ against facts
fixed by mathematics or by a library routine, never against the HIP path."""
import itertools
import os

import numpy as np
import pytest

from oracle import conv3d as oc

HERE = os.path.dirname(os.path.abspath(__file__))

CASES = [
    # N, D, H, W, Cin, Cout, k, s, p
    (1, 4, 5, 6, 2, 3, 3, 1, 1),
    (2, 5, 4, 6, 3, 2, 3, 2, 1),
    (1, 6, 5, 4, 2, 2, 3, 2, 0),
    (1, 3, 4, 5, 3, 2, 1, 1, 0),
    (1, 4, 6, 4, 2, 3, 2, 2, 0),
    (1, 5, 5, 6, 1, 2, 2, 1, 1),
    (1, 4, 5, 7, 2, 2, (1, 2, 3), (1, 2, 1), (0, 1, 2)),
    (2, 6, 6, 5, 2, 2, 3, (2, 1, 2), (1, 0, 1)),
]


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _tensors(case, seed=0):
    g = oc.shape(*case)
    x = _rand((g.N, g.D, g.H, g.W, g.Cin), seed)
    w = _rand((g.Cout, g.kD, g.kH, g.kW, g.Cin), seed + 1)
    dy = _rand((g.N,) + oc.out_dims(g) + (g.Cout,), seed + 2)
    return g, x, w, dy


def _window_reference(g, x, w):
    """Independent statement of the forward pass: pad the volume with zeros,
    then for every tap take a strided slice of the padded volume and contract
    its channels with that tap's [Cout, Cin] matrix."""
    Do, Ho, Wo = oc.out_dims(g)
    xp = np.zeros((g.N, g.D + 2 * g.pD, g.H + 2 * g.pH, g.W + 2 * g.pW, g.Cin))
    xp[:, g.pD:g.pD + g.D, g.pH:g.pH + g.H, g.pW:g.pW + g.W, :] = x
    y = np.zeros((g.N, Do, Ho, Wo, g.Cout))
    for kd, kh, kw in itertools.product(range(g.kD), range(g.kH), range(g.kW)):
        sl = xp[:, kd:kd + (Do - 1) * g.sD + 1:g.sD, kh:kh + (Ho - 1) * g.sH + 1:g.sH,
                kw:kw + (Wo - 1) * g.sW + 1:g.sW, :]
        y += np.einsum("ndhwc,oc->ndhwo", sl, w[:, kd, kh, kw, :])
    return y


@pytest.mark.parametrize("case", CASES)
def test_fwd_matches_window_reference(case):
    g, x, w, _ = _tensors(case)
    np.testing.assert_allclose(oc.fwd(g, x, w), _window_reference(g, x, w), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_fwd_matches_torch_library(case):
    torch = pytest.importorskip("torch")
    g, x, w, _ = _tensors(case, 10)
    xt = torch.from_numpy(x).permute(0, 4, 1, 2, 3)
    wt = torch.from_numpy(w).permute(0, 4, 1, 2, 3)
    yt = torch.nn.functional.conv3d(xt, wt, stride=(g.sD, g.sH, g.sW), padding=(g.pD, g.pH, g.pW))
    np.testing.assert_allclose(oc.fwd(g, x, w), yt.permute(0, 2, 3, 4, 1).numpy(), rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("case", CASES)
def test_gradients_match_torch_autograd(case):
    torch = pytest.importorskip("torch")
    g, x, w, dy = _tensors(case, 20)
    xt = torch.from_numpy(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)
    wt = torch.from_numpy(w).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)
    yt = torch.nn.functional.conv3d(xt, wt, stride=(g.sD, g.sH, g.sW), padding=(g.pD, g.pH, g.pW))
    yt.backward(torch.from_numpy(dy).permute(0, 4, 1, 2, 3))
    np.testing.assert_allclose(oc.dgrad(g, dy, w), xt.grad.permute(0, 2, 3, 4, 1).numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(oc.wgrad(g, x, dy), wt.grad.permute(0, 2, 3, 4, 1).numpy(), rtol=1e-11, atol=1e-11)


def test_hand_worked_example():
    vals = {}
    with open(os.path.join(HERE, "golden", "conv3d_hand_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            vals[key] = np.array([float(v) for v in nums])
    g = oc.shape(1, 1, 2, 3, 1, 1, (1, 2, 2), 1, (0, 0, 1))
    x = np.arange(1.0, 7.0).reshape(1, 1, 2, 3, 1)
    w = np.array([1.0, 10.0, 100.0, 1000.0]).reshape(1, 1, 2, 2, 1)
    dy = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 1, 4, 1)
    assert np.array_equal(oc.fwd(g, x, w).ravel(), vals["y"])
    assert np.array_equal(oc.dgrad(g, dy, w).ravel(), vals["dx"])
    assert np.array_equal(oc.wgrad(g, x, dy).ravel(), vals["dw"])


def test_identity_kernel_returns_input():
    g = oc.shape(2, 5, 4, 6, 3, 3, 3, 1, 1)
    x = _rand((2, 5, 4, 6, 3), 3)
    w = np.zeros((3, 3, 3, 3, 3))
    for c in range(3):
        w[c, 1, 1, 1, c] = 1.0
    assert np.array_equal(oc.fwd(g, x, w), x)
    assert np.array_equal(oc.dgrad(g, x, w), x)


@pytest.mark.parametrize("tap", [(0, 0, 0), (2, 1, 0), (1, 2, 2), (0, 2, 1)])
def test_shift_kernel_translates(tap):
    D, H, W = 5, 6, 7
    g = oc.shape(1, D, H, W, 1, 1, 3, 1, 1)
    x = _rand((1, D, H, W, 1), 4)
    w = np.zeros((1, 3, 3, 3, 1))
    w[0, tap[0], tap[1], tap[2], 0] = 1.0
    y = oc.fwd(g, x, w)
    dx = oc.dgrad(g, x, w)
    exp = np.zeros_like(x)
    exp_adj = np.zeros_like(x)
    for d, h, ww in itertools.product(range(D), range(H), range(W)):
        sd, sh, sw = d + tap[0] - 1, h + tap[1] - 1, ww + tap[2] - 1
        if 0 <= sd < D and 0 <= sh < H and 0 <= sw < W:
            exp[0, d, h, ww, 0] = x[0, sd, sh, sw, 0]          # y(o) = x(o + t - p)
            exp_adj[0, sd, sh, sw, 0] = x[0, d, h, ww, 0]      # adjoint shifts back
    assert np.array_equal(y, exp)
    assert np.array_equal(dx, exp_adj)


def test_channel_roles_not_transposed():
    # w maps input channel 1 to output channel 0 only; Cin != Cout
    g = oc.shape(1, 3, 3, 3, 2, 3, 1, 1, 0)
    x = _rand((1, 3, 3, 3, 2), 5)
    w = np.zeros((3, 1, 1, 1, 2))
    w[0, 0, 0, 0, 1] = 2.0
    y = oc.fwd(g, x, w)
    assert np.array_equal(y[..., 0], 2.0 * x[..., 1])
    assert not y[..., 1:].any()


def test_ones_closed_form_counts_in_range_taps():
    Cin = 3
    g = oc.shape(1, 5, 6, 7, Cin, 2, 3, 1, 1)
    y = oc.fwd(g, np.ones((1, 5, 6, 7, Cin)), np.ones((2, 3, 3, 3, Cin)))
    assert y[0, 2, 2, 2, 0] == 27 * Cin       # interior
    assert y[0, 0, 2, 2, 1] == 18 * Cin       # face
    assert y[0, 0, 0, 3, 0] == 12 * Cin       # edge
    assert y[0, 0, 0, 0, 1] == 8 * Cin        # corner
    assert y[0, 4, 5, 6, 0] == 8 * Cin        # opposite corner
    cnt = lambda n: np.array([2] + [3] * (n - 2) + [2])
    exp = cnt(5)[:, None, None] * cnt(6)[None, :, None] * cnt(7)[None, None, :] * Cin
    assert np.array_equal(y[0, ..., 0], exp)


def test_pointwise_kernel_is_matrix_product():
    g = oc.shape(2, 3, 4, 5, 6, 4, 1, 1, 0)
    x = _rand((2, 3, 4, 5, 6), 6)
    w = _rand((4, 1, 1, 1, 6), 7)
    ref = (x.reshape(-1, 6) @ w.reshape(4, 6).T).reshape(2, 3, 4, 5, 4)
    np.testing.assert_allclose(oc.fwd(g, x, w), ref, rtol=1e-13, atol=1e-13)
    dy = _rand((2, 3, 4, 5, 4), 8)
    np.testing.assert_allclose(oc.dgrad(g, dy, w), (dy.reshape(-1, 4) @ w.reshape(4, 6)).reshape(x.shape), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oc.wgrad(g, x, dy).reshape(4, 6), dy.reshape(-1, 4).T @ x.reshape(-1, 6), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("case", CASES)
def test_linearity(case):
    g, x, w, dy = _tensors(case, 30)
    x2 = _rand(x.shape, 31)
    w2 = _rand(w.shape, 32)
    np.testing.assert_allclose(oc.fwd(g, 2 * x - 3 * x2, w), 2 * oc.fwd(g, x, w) - 3 * oc.fwd(g, x2, w), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(oc.fwd(g, x, w + 0.5 * w2), oc.fwd(g, x, w) + 0.5 * oc.fwd(g, x, w2), rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("case", CASES)
def test_dgrad_is_adjoint_of_fwd(case):
    g, x, w, dy = _tensors(case, 40)
    lhs = np.vdot(oc.fwd(g, x, w), dy)
    rhs = np.vdot(x, oc.dgrad(g, dy, w))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


@pytest.mark.parametrize("case", CASES)
def test_wgrad_bilinear_identity(case):
    g, x, w, dy = _tensors(case, 50)
    lhs = np.vdot(oc.fwd(g, x, w), dy)
    rhs = np.vdot(w, oc.wgrad(g, x, dy))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_wgrad_exact_finite_difference():
    # L(w) = <fwd(x; w), dy> is linear in w, so a unit step in one weight
    # changes it by exactly that weight's gradient.
    case = (1, 4, 5, 4, 2, 2, 3, 2, 1)
    g, x, w, dy = _tensors(case, 60)
    dw = oc.wgrad(g, x, dy)
    base = np.vdot(oc.fwd(g, x, w), dy)
    rng = np.random.default_rng(61)
    for _ in range(12):
        j = tuple(rng.integers(0, n) for n in w.shape)
        w2 = w.copy()
        w2[j] += 1.0
        fd = np.vdot(oc.fwd(g, x, w2), dy) - base
        assert abs(fd - dw[j]) <= 1e-10 * max(1.0, abs(dw[j]))


def test_dgrad_finite_difference():
    case = (1, 4, 5, 4, 2, 2, 3, 2, 1)
    g, x, w, dy = _tensors(case, 70)
    dx = oc.dgrad(g, dy, w)
    base = np.vdot(oc.fwd(g, x, w), dy)
    rng = np.random.default_rng(71)
    for _ in range(12):
        j = tuple(rng.integers(0, n) for n in x.shape)
        x2 = x.copy()
        x2[j] += 1.0
        fd = np.vdot(oc.fwd(g, x2, w), dy) - base
        assert abs(fd - dx[j]) <= 1e-10 * max(1.0, abs(dx[j]))


def test_stride2_positions_without_contribution_are_zero():
    # D=6,k=3,s=2,p=0 -> Do=2 reads input planes 0..4; plane 5 gets no gradient
    g = oc.shape(1, 6, 6, 6, 1, 1, 3, 2, 0)
    dx = oc.dgrad(g, np.ones((1, 2, 2, 2, 1)), np.ones((1, 3, 3, 3, 1)))
    assert not dx[0, 5].any() and not dx[0, :, 5].any() and not dx[0, :, :, 5].any()
    assert dx[0, 2, 2, 2, 0] == 8.0  # read by both outputs along each axis


@pytest.mark.parametrize("case", CASES)
def test_sampled_evaluations_agree_with_full(case):
    g, x, w, dy = _tensors(case, 80)
    x32, w32, dy32 = (a.astype(np.float32) for a in (x, w, dy))
    x64, w64, dy64 = (a.astype(np.float64) for a in (x32, w32, dy32))
    y = oc.fwd(g, x64, w64)
    dx = oc.dgrad(g, dy64, w64)
    dw = oc.wgrad(g, x64, dy64)
    np.testing.assert_allclose(oc.fwd_at(g, x32, w32, np.arange(y.size)), y.ravel(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oc.dgrad_at(g, dy32, w32, np.arange(dx.size)), dx.ravel(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oc.wgrad_at(g, x32, dy32, np.arange(dw.size)), dw.ravel(), rtol=1e-12, atol=1e-12)


def test_transposed_conv_brute_force_and_role_swap():
    N, Dz, Hz, Wz, Ci, Co = 1, 2, 3, 2, 3, 2
    z = _rand((N, Dz, Hz, Wz, Ci), 90)
    v = _rand((Ci, 2, 2, 2, Co), 91)
    u = oc.tconv_fwd(z, v)
    exp = np.zeros((N, 2 * Dz, 2 * Hz, 2 * Wz, Co))
    for jd, jh, jw, td, th, tw in itertools.product(range(Dz), range(Hz), range(Wz), range(2), range(2), range(2)):
        exp[0, 2 * jd + td, 2 * jh + th, 2 * jw + tw, :] = z[0, jd, jh, jw, :] @ v[:, td, th, tw, :]
    np.testing.assert_allclose(u, exp, rtol=1e-13, atol=1e-13)
    # the same map is the data-gradient of a k2/s2/p0 convolution whose input
    # channels are the upsampled side (Co) and output channels the coarse side (Ci)
    g = oc.shape(N, 2 * Dz, 2 * Hz, 2 * Wz, Co, Ci, 2, 2, 0)
    w = np.transpose(v, (0, 1, 2, 3, 4))  # [Ci][t][Co] == [Cout'][t][Cin']
    np.testing.assert_allclose(oc.dgrad(g, z, w), u, rtol=1e-13, atol=1e-13)


def test_out_dims_and_invalid_shapes():
    assert oc.out_dims(oc.shape(1, 192, 192, 192, 32, 64, 3, 2, 1)) == (96, 96, 96)
    assert oc.out_dims(oc.shape(1, 16, 16, 16, 4, 8, 3, 1, 1)) == (16, 16, 16)
    assert oc.out_dims(oc.shape(1, 7, 8, 9, 1, 1, 3, 2, 1)) == (4, 4, 5)
    with pytest.raises(ValueError):
        oc.out_dims(oc.shape(1, 1, 4, 4, 1, 1, 3, 1, 0))
    with pytest.raises(ValueError):
        oc.out_dims(oc.shape(1, 4, 4, 4, 0, 1, 3, 1, 1))


def test_rel_err_metric():
    ref = np.array([1.0, -2.0, 0.0, 4.0])
    got = ref + np.array([0.0, 0.02, 0.01, 0.0])
    rms = np.sqrt(np.mean(ref ** 2))
    assert oc.rel_err(got, ref) == pytest.approx(max(0.02 / max(2.0, rms), 0.01 / rms))
    assert oc.rel_err(ref, ref) == 0.0
