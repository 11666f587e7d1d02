"""Thin binding of the elementwise / loss / optimiser entry points (marshalling only)."""
import ctypes

import torch

from ._lib import check, lib
from .swap import _stream


def _p(t):
    return ctypes.c_void_p(t.data_ptr())


def leaky_relu_fwd(a, slope=0.01):
    check(lib().mi3d_leaky_relu_fwd(_p(a), a.numel(), slope, _stream()), "leaky_relu_fwd")


def leaky_relu_bwd(da, a, slope=0.01):
    assert da.numel() == a.numel() and da.dtype == a.dtype
    if da.dtype == torch.float32:
        check(lib().mi3d_leaky_relu_bwd_f32(_p(da), _p(a), a.numel(), slope, _stream()), "leaky_relu_bwd_f32")
    else:
        check(lib().mi3d_leaky_relu_bwd(_p(da), _p(a), a.numel(), slope, _stream()), "leaky_relu_bwd")


def concat_channels(a, b, out):
    Ca, Cb = a.shape[-1], b.shape[-1]
    vox = a.numel() // Ca
    assert b.numel() // Cb == vox and out.numel() == vox * (Ca + Cb)
    check(lib().mi3d_concat_channels(_p(a), Ca, _p(b), Cb, _p(out), vox, _stream()), "concat_channels")


def split_channels(x, a, b):
    Ca, Cb = a.shape[-1], b.shape[-1]
    vox = a.numel() // Ca
    assert b.numel() // Cb == vox and x.numel() == vox * (Ca + Cb)
    check(lib().mi3d_split_channels(_p(x), Ca, Cb, _p(a), _p(b), vox, _stream()), "split_channels")


def slice_channels(x, c_off, out):
    Ct, C = x.shape[-1], out.shape[-1]
    vox = out.numel() // C
    assert x.numel() == vox * Ct
    check(lib().mi3d_slice_channels(_p(x), Ct, c_off, C, _p(out), vox, _stream()), "slice_channels")


def place_channels(x, out, c_off):
    """out[..., c_off : c_off + C] = x; the other channels of out stay as they are."""
    C, Ct = x.shape[-1], out.shape[-1]
    vox = x.numel() // C
    assert out.numel() == vox * Ct
    check(lib().mi3d_place_channels(_p(x), C, _p(out), Ct, c_off, vox, _stream()), "place_channels")


def skip_grad(da, dcat, c_off, a, slope=0.01):
    """da <- (da + dcat[..., c_off : c_off + C]) * (a > 0 ? 1 : slope), in place on da."""
    Ct, C = dcat.shape[-1], da.shape[-1]
    vox = da.numel() // C
    assert dcat.numel() == vox * Ct and a.numel() == da.numel()
    check(lib().mi3d_skip_grad(_p(da), _p(dcat), Ct, c_off, _p(a), C, vox, slope, _stream()), "skip_grad")


def add_inplace(a, b):
    assert a.numel() == b.numel()
    check(lib().mi3d_add_inplace(_p(a), _p(b), a.numel(), _stream()), "add_inplace")


def dice_workspace(classes=3):
    return torch.empty(lib().mi3d_dice_workspace_bytes(classes), dtype=torch.uint8, device="cuda")


def dice_loss(logits, labels, ws, sums, loss, eps=1e-5):
    C = logits.shape[-1]
    vox = logits.numel() // C
    fn = lib().mi3d_dice_loss_f32 if logits.dtype == torch.float32 else lib().mi3d_dice_loss
    check(fn(_p(logits), _p(labels), vox, C, eps, _p(ws), ws.numel(), _p(sums), _p(loss), _stream()), "dice_loss")


def dice_grad(logits, labels, sums, dlogits, eps=1e-5):
    C = logits.shape[-1]
    vox = logits.numel() // C
    assert logits.dtype == dlogits.dtype
    fn = lib().mi3d_dice_grad_f32 if logits.dtype == torch.float32 else lib().mi3d_dice_grad
    check(fn(_p(logits), _p(labels), vox, C, eps, _p(sums), _p(dlogits), _stream()), "dice_grad")


def sgd_update(w32, dw32, w16, lr):
    """w16 None: no bf16 working copy (the fp32 step)."""
    assert w32.numel() == dw32.numel() and (w16 is None or w16.numel() == w32.numel())
    check(lib().mi3d_sgd_update(_p(w32), _p(dw32), None if w16 is None else _p(w16), w32.numel(), lr, _stream()), "sgd_update")


def adam_update(w32, dw32, m32, v32, w16, lr, step, beta1=0.9, beta2=0.999, eps=1e-8):
    assert w32.numel() == dw32.numel() == m32.numel() == v32.numel() and (w16 is None or w16.numel() == w32.numel())
    check(lib().mi3d_adam_update(_p(w32), _p(dw32), _p(m32), _p(v32), None if w16 is None else _p(w16), w32.numel(), lr, beta1, beta2, eps, int(step), _stream()), "adam_update")


IN_EPS = 1e-5


def instnorm_workspace(N, C):
    return torch.empty(lib().mi3d_instnorm_workspace_bytes(N, C), dtype=torch.uint8, device="cuda")


def instnorm_stats(z, stats, ws, eps=IN_EPS):
    """stats[n, c] = (mean, 1 / sqrt(var + eps)) of z[n, ..., c]."""
    N, C = z.shape[0], z.shape[-1]
    vox = z.numel() // (N * C)
    assert tuple(stats.shape) == (N, C, 2) and stats.dtype == torch.float32
    fn = lib().mi3d_instnorm_stats_f32 if z.dtype == torch.float32 else lib().mi3d_instnorm_stats
    check(fn(_p(z), N, vox, C, eps, _p(stats), _p(ws), ws.numel(), _stream()), "instnorm_stats")


def instnorm_lrelu_fwd(z, stats, slope=0.01):
    N, C = z.shape[0], z.shape[-1]
    fn = lib().mi3d_instnorm_lrelu_fwd_f32 if z.dtype == torch.float32 else lib().mi3d_instnorm_lrelu_fwd
    check(fn(_p(z), _p(stats), N, z.numel() // (N * C), C, slope, _stream()), "instnorm_lrelu_fwd")


def instnorm_lrelu_bwd_sums(da, a, stats, sums, slope=0.01):
    """da <- dz given the two means (mean g, mean g * xhat) per (sample, channel)."""
    N, C = a.shape[0], a.shape[-1]
    assert da.numel() == a.numel() and tuple(sums.shape) == (N, C, 2) and sums.dtype == torch.float32
    assert a.dtype == torch.bfloat16 and da.dtype == torch.bfloat16      # (bf16 only: the kernels that deliver the sums are)
    check(lib().mi3d_instnorm_lrelu_bwd_sums(_p(da), _p(a), _p(stats), _p(sums), N, a.numel() // (N * C), C, slope, _stream()), "instnorm_lrelu_bwd_sums")


def instnorm_lrelu_bwd(da, a, stats, ws, slope=0.01):
    N, C = a.shape[0], a.shape[-1]
    assert da.numel() == a.numel() and da.dtype == a.dtype
    fn = lib().mi3d_instnorm_lrelu_bwd_f32 if a.dtype == torch.float32 else lib().mi3d_instnorm_lrelu_bwd
    check(fn(_p(da), _p(a), _p(stats), N, a.numel() // (N * C), C, slope, _p(ws), ws.numel(), _stream()), "instnorm_lrelu_bwd")
