"""Thin binding of the convolution entry points: argument marshalling only.

Tensors are torch CUDA tensors used as plain device buffers (NDHWC
activations, [Cout][kD][kH][kW][Cin] weights); every arithmetic step runs in
libmi3d.so on the current torch stream.
"""
import ctypes

import torch

from ._lib import ConvDesc, check, lib

F32, BF16 = 0, 1
PASS_FWD, PASS_DGRAD, PASS_WGRAD = 0, 1, 2
_DT = {torch.float32: F32, torch.bfloat16: BF16}


def _t3(v):
    return (v, v, v) if isinstance(v, int) else tuple(int(a) for a in v)


def make_desc(N, D, H, W, Cin, Cout, k, s, p, dtype):
    k, s, p = _t3(k), _t3(s), _t3(p)
    dt = _DT[dtype] if isinstance(dtype, torch.dtype) else int(dtype)
    return ConvDesc(N, D, H, W, Cin, Cout, *k, *s, *p, dt)


def out_dims(desc):
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    check(lib().mi3d_conv3d_out_dims(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "conv3d_out_dims")
    return a.value, b.value, c.value


def workspace_bytes(desc, pass_):
    return int(lib().mi3d_conv3d_workspace_bytes(ctypes.byref(desc), pass_))


def kernel_name(desc, pass_):
    buf = ctypes.create_string_buffer(64)
    check(lib().mi3d_conv3d_kernel_name(ctypes.byref(desc), pass_, buf, 64), "conv3d_kernel_name")
    return buf.value.decode()


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _tdtype(desc):
    return torch.float32 if desc.dtype == F32 else torch.bfloat16


def _chk(t, shape, dtype, name):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: need contiguous CUDA {dtype} tensor of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)} on {t.device}")


def _ws(desc, pass_, ws):
    need = workspace_bytes(desc, pass_)
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    return ws, ws.data_ptr(), ws.numel() * ws.element_size()


def _shapes(desc):
    Do, Ho, Wo = out_dims(desc)
    return ((desc.N, desc.D, desc.H, desc.W, desc.Cin),
            (desc.Cout, desc.kD, desc.kH, desc.kW, desc.Cin),
            (desc.N, Do, Ho, Wo, desc.Cout))


def conv3d_fwd(desc, x, w, y=None, ws=None):
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x, xs, dt, "x"); _chk(w, wsh, dt, "w")
    if y is None:
        y = torch.empty(ys, dtype=dt, device=x.device)
    _chk(y, ys, dt, "y")
    ws, p, n = _ws(desc, PASS_FWD, ws)
    check(lib().mi3d_conv3d_fwd(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), y.data_ptr(), p, n, _stream()), "conv3d_fwd")
    return y


def conv3d_dgrad(desc, dy, w, dx=None, ws=None):
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(dy, ys, dt, "dy"); _chk(w, wsh, dt, "w")
    if dx is None:
        dx = torch.empty(xs, dtype=dt, device=dy.device)
    _chk(dx, xs, dt, "dx")
    ws, p, n = _ws(desc, PASS_DGRAD, ws)
    check(lib().mi3d_conv3d_dgrad(ctypes.byref(desc), dy.data_ptr(), w.data_ptr(), dx.data_ptr(), p, n, _stream()), "conv3d_dgrad")
    return dx


def _view(t, C, offset):
    """(View, shape check) for the `C` channels starting at `offset` of the channel-last tensor t."""
    from ._lib import View
    pitch = t.shape[-1]
    assert 0 <= offset and offset + C <= pitch
    return View(int(pitch), int(offset))


def conv3d_fwd_view(desc, x_wide, offset, w, y=None, ws=None):
    """conv3d_fwd whose x is channels [offset, offset + Cin) of x_wide (k2/s2 layers only)."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x_wide, xs[:-1] + (x_wide.shape[-1],), dt, "x"); _chk(w, wsh, dt, "w")
    if y is None:
        y = torch.empty(ys, dtype=dt, device=x_wide.device)
    _chk(y, ys, dt, "y")
    v = _view(x_wide, desc.Cin, offset)
    ws, p, n = _ws(desc, PASS_FWD, ws)
    check(lib().mi3d_conv3d_fwd_view(ctypes.byref(desc), x_wide.data_ptr(), ctypes.byref(v), w.data_ptr(), y.data_ptr(), p, n, _stream()), "conv3d_fwd_view")
    return y


def conv3d_dgrad_view(desc, dy, w, dx_wide, offset, ws=None):
    """conv3d_dgrad that writes dx into channels [offset, offset + Cin) of dx_wide (k2/s2 layers only)."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(dy, ys, dt, "dy"); _chk(w, wsh, dt, "w"); _chk(dx_wide, xs[:-1] + (dx_wide.shape[-1],), dt, "dx")
    v = _view(dx_wide, desc.Cin, offset)
    ws, p, n = _ws(desc, PASS_DGRAD, ws)
    check(lib().mi3d_conv3d_dgrad_view(ctypes.byref(desc), dy.data_ptr(), w.data_ptr(), dx_wide.data_ptr(), ctypes.byref(v), p, n, _stream()), "conv3d_dgrad_view")
    return dx_wide


def conv3d_wgrad_view(desc, x_wide, offset, dy, dw=None, ws=None):
    """conv3d_wgrad whose x is channels [offset, offset + Cin) of x_wide (k2/s2 layers only)."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x_wide, xs[:-1] + (x_wide.shape[-1],), dt, "x"); _chk(dy, ys, dt, "dy")
    if dw is None:
        dw = torch.empty(wsh, dtype=torch.float32, device=dy.device)
    _chk(dw, wsh, torch.float32, "dw")
    v = _view(x_wide, desc.Cin, offset)
    ws, p, n = _ws(desc, PASS_WGRAD, ws)
    check(lib().mi3d_conv3d_wgrad_view(ctypes.byref(desc), x_wide.data_ptr(), ctypes.byref(v), dy.data_ptr(), dw.data_ptr(), p, n, _stream()), "conv3d_wgrad_view")
    return dw


def conv3d_dgrad_skip(desc, dy, w, add, a_in, slope, dx=None, ws=None):
    """dx = (bf16(dgrad(dy, w)) + add) * (a_in > 0 ? 1 : slope): the gradient that reaches the producer of a skip tensor."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(dy, ys, dt, "dy"); _chk(w, wsh, dt, "w"); _chk(add, xs, dt, "add"); _chk(a_in, xs, dt, "a_in")
    if dx is None:
        dx = torch.empty(xs, dtype=dt, device=dy.device)
    _chk(dx, xs, dt, "dx")
    ws, p, n = _ws(desc, PASS_DGRAD, ws)
    check(lib().mi3d_conv3d_dgrad_skip(ctypes.byref(desc), dy.data_ptr(), w.data_ptr(), add.data_ptr(), a_in.data_ptr(), ctypes.c_float(slope),
                                       dx.data_ptr(), p, n, _stream()), "conv3d_dgrad_skip")
    return dx


def fwd_stats_supported(desc):
    """True if the forward kernel of this geometry can produce the instance-normalisation statistics of its output."""
    return bool(lib().mi3d_conv3d_fwd_stats_supported(ctypes.byref(desc)))


def conv3d_fwd_stats(desc, x, w, stats, eps=1e-5, y=None, ws=None, x_hi=None):
    """y = conv(x, w) (x = [x | x_hi] when x_hi is given) and stats[n][c] = (mean, rstd) of y, in one kernel."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    if x_hi is None:
        _chk(x, xs, dt, "x")
    else:
        _chk(x, _half(desc), dt, "x_lo"); _chk(x_hi, _half(desc), dt, "x_hi")
    _chk(w, wsh, dt, "w")
    _chk(stats, (desc.N, desc.Cout, 2), torch.float32, "stats")
    if y is None:
        y = torch.empty(ys, dtype=dt, device=x.device)
    _chk(y, ys, dt, "y")
    ws, p, n = _ws(desc, PASS_FWD, ws)
    check(lib().mi3d_conv3d_fwd_stats(ctypes.byref(desc), x.data_ptr(), None if x_hi is None else x_hi.data_ptr(), w.data_ptr(), y.data_ptr(),
                                      ctypes.c_float(eps), stats.data_ptr(), p, n, _stream()), "conv3d_fwd_stats")
    return y


def dgrad_insums_supported(desc, with_add=False):
    """True if the data-gradient kernel of this geometry can also produce the two means of the instance-normalisation
    backward pass of the layer below (with_add: while it adds the second gradient of a skip connection)."""
    return bool(lib().mi3d_conv3d_dgrad_insums_supported(ctypes.byref(desc), int(bool(with_add))))


def conv3d_dgrad_insums(desc, dy, w, a_in, slope, sums, dx=None, ws=None, add=None):
    """dx = dgrad(dy, w) (+ add) and sums[n][c] = (mean g, mean g * xhat) with g = dx * lrelu'(a_in), xhat = lrelu^-1(a_in)."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(dy, ys, dt, "dy"); _chk(w, wsh, dt, "w"); _chk(a_in, xs, dt, "a_in")
    if add is not None:
        _chk(add, xs, dt, "add")
    _chk(sums, (desc.N, desc.Cin, 2), torch.float32, "sums")
    if dx is None:
        dx = torch.empty(xs, dtype=dt, device=dy.device)
    _chk(dx, xs, dt, "dx")
    ws, p, n = _ws(desc, PASS_DGRAD, ws)
    check(lib().mi3d_conv3d_dgrad_insums(ctypes.byref(desc), dy.data_ptr(), w.data_ptr(), None if add is None else add.data_ptr(), a_in.data_ptr(),
                                         ctypes.c_float(slope), dx.data_ptr(), sums.data_ptr(), p, n, _stream()), "conv3d_dgrad_insums")
    return dx


def pair_supported(desc, pass_):
    """True if the pass takes the tensor of x's shape as two halves along the channels (conv3d_*_pair)."""
    return bool(lib().mi3d_conv3d_pair_supported(ctypes.byref(desc), int(pass_)))


def _half(desc):
    xs, _, _ = _shapes(desc)
    return xs[:-1] + (desc.Cin // 2,)


def conv3d_fwd_pair(desc, x_lo, x_hi, w, slope=1.0, y=None, ws=None):
    """conv3d_fwd over the channel concatenation [x_lo | x_hi] (never materialised); slope != 1: LeakyReLU on y."""
    _, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x_lo, _half(desc), dt, "x_lo"); _chk(x_hi, _half(desc), dt, "x_hi"); _chk(w, wsh, dt, "w")
    if y is None:
        y = torch.empty(ys, dtype=dt, device=x_lo.device)
    _chk(y, ys, dt, "y")
    ws, p, n = _ws(desc, PASS_FWD, ws)
    check(lib().mi3d_conv3d_fwd_pair(ctypes.byref(desc), x_lo.data_ptr(), x_hi.data_ptr(), w.data_ptr(), y.data_ptr(),
                                     ctypes.c_float(slope), p, n, _stream()), "conv3d_fwd_pair")
    return y


def conv3d_dgrad_pair(desc, dy, w, dx_lo=None, dx_hi=None, ws=None):
    """conv3d_dgrad that writes the two channel halves of dx to separate tensors."""
    _, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(dy, ys, dt, "dy"); _chk(w, wsh, dt, "w")
    if dx_lo is None:
        dx_lo = torch.empty(_half(desc), dtype=dt, device=dy.device)
    if dx_hi is None:
        dx_hi = torch.empty(_half(desc), dtype=dt, device=dy.device)
    _chk(dx_lo, _half(desc), dt, "dx_lo"); _chk(dx_hi, _half(desc), dt, "dx_hi")
    ws, p, n = _ws(desc, PASS_DGRAD, ws)
    check(lib().mi3d_conv3d_dgrad_pair(ctypes.byref(desc), dy.data_ptr(), w.data_ptr(), dx_lo.data_ptr(), dx_hi.data_ptr(),
                                       p, n, _stream()), "conv3d_dgrad_pair")
    return dx_lo, dx_hi


def conv3d_wgrad_pair(desc, x_lo, x_hi, dy, dw=None, ws=None):
    """conv3d_wgrad whose x is the channel concatenation [x_lo | x_hi] (never materialised)."""
    _, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x_lo, _half(desc), dt, "x_lo"); _chk(x_hi, _half(desc), dt, "x_hi"); _chk(dy, ys, dt, "dy")
    if dw is None:
        dw = torch.empty(wsh, dtype=torch.float32, device=dy.device)
    _chk(dw, wsh, torch.float32, "dw")
    ws, p, n = _ws(desc, PASS_WGRAD, ws)
    check(lib().mi3d_conv3d_wgrad_pair(ctypes.byref(desc), x_lo.data_ptr(), x_hi.data_ptr(), dy.data_ptr(), dw.data_ptr(),
                                       p, n, _stream()), "conv3d_wgrad_pair")
    return dw


def conv3d_fwd_lrelu(desc, x, w, slope, y=None, ws=None):
    """y = LeakyReLU(conv(x, w)) in one call."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x, xs, dt, "x"); _chk(w, wsh, dt, "w")
    if y is None:
        y = torch.empty(ys, dtype=dt, device=x.device)
    _chk(y, ys, dt, "y")
    ws, p, n = _ws(desc, PASS_FWD, ws)
    check(lib().mi3d_conv3d_fwd_lrelu(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), y.data_ptr(), float(slope), p, n, _stream()), "conv3d_fwd_lrelu")
    return y


def conv3d_dgrad_lrelu(desc, dy, w, a_in, slope, dx=None, ws=None):
    """dx = dgrad(dy, w) * (a_in > 0 ? 1 : slope): the gradient with respect to the pre-activation of the layer below."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(dy, ys, dt, "dy"); _chk(w, wsh, dt, "w"); _chk(a_in, xs, dt, "a_in")
    if dx is None:
        dx = torch.empty(xs, dtype=dt, device=dy.device)
    _chk(dx, xs, dt, "dx")
    ws, p, n = _ws(desc, PASS_DGRAD, ws)
    check(lib().mi3d_conv3d_dgrad_lrelu(ctypes.byref(desc), dy.data_ptr(), w.data_ptr(), a_in.data_ptr(), float(slope), dx.data_ptr(), p, n, _stream()),
          "conv3d_dgrad_lrelu")
    return dx


def conv3d_wgrad(desc, x, dy, dw=None, ws=None):
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x, xs, dt, "x"); _chk(dy, ys, dt, "dy")
    if dw is None:
        dw = torch.empty(wsh, dtype=torch.float32, device=x.device)
    _chk(dw, wsh, torch.float32, "dw")
    ws, p, n = _ws(desc, PASS_WGRAD, ws)
    check(lib().mi3d_conv3d_wgrad(ctypes.byref(desc), x.data_ptr(), dy.data_ptr(), dw.data_ptr(), p, n, _stream()), "conv3d_wgrad")
    return dw


def static_scratch_bytes():
    return int(lib().mi3d_static_scratch_bytes())


def conv3d_wgrad_static(desc, x, dy, dw):
    """conv3d_wgrad without a workspace argument and without any allocation: dw must be given; the scratch is the
    library's static device array."""
    xs, wsh, ys = _shapes(desc)
    dt = _tdtype(desc)
    _chk(x, xs, dt, "x"); _chk(dy, ys, dt, "dy"); _chk(dw, wsh, torch.float32, "dw")
    check(lib().mi3d_conv3d_wgrad_static(ctypes.byref(desc), x.data_ptr(), dy.data_ptr(), dw.data_ptr(), _stream()), "conv3d_wgrad_static")
    return dw
