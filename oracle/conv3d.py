"""ctypes front end of the fp64 C oracle (test infrastructure only).

Layouts: activations NDHWC, weights [Cout][kD][kH][kW][Cin]; explicit
symmetric zero padding and stride; cross-correlation.  The paper states no
convolution formula (its layers ran in a closed vendor library, Section 4.1);
the definitions are the textbook ones spelled out in conv3d_oracle.c, whose
forward/backward roles follow the feature-map data flow of Section 3.1.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


class Shape(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "D", "H", "W", "Cin", "Cout", "kD", "kH", "kW",
                 "sD", "sH", "sW", "pD", "pH", "pW")]


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _lib = ctypes.CDLL(path)
        for name in ("oracle_conv3d_out_dims", "oracle_conv3d_fwd", "oracle_conv3d_dgrad",
                     "oracle_conv3d_wgrad", "oracle_conv3d_fwd_at", "oracle_conv3d_dgrad_at",
                     "oracle_conv3d_wgrad_at", "oracle_tconv3d_fwd"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _triple(v):
    return (v, v, v) if np.isscalar(v) else tuple(int(a) for a in v)


def shape(N, D, H, W, Cin, Cout, k, s, p):
    k, s, p = _triple(k), _triple(s), _triple(p)
    return Shape(N, D, H, W, Cin, Cout, *k, *s, *p)


def out_dims(g):
    lib = _load()
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    if lib.oracle_conv3d_out_dims(ctypes.byref(g), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)):
        raise ValueError("invalid convolution shape")
    return a.value, b.value, c.value


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a, shp):
    a = np.ascontiguousarray(a, dtype=np.float64)
    assert a.shape == tuple(shp), (a.shape, shp)
    return a


def _f32(a, shp):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.shape == tuple(shp), (a.shape, shp)
    return a


def _xs(g):
    return (g.N, g.D, g.H, g.W, g.Cin)


def _ws(g):
    return (g.Cout, g.kD, g.kH, g.kW, g.Cin)


def _ys(g):
    return (g.N,) + out_dims(g) + (g.Cout,)


def fwd(g, x, w):
    x, w = _f64(x, _xs(g)), _f64(w, _ws(g))
    y = np.empty(_ys(g), dtype=np.float64)
    assert _load().oracle_conv3d_fwd(ctypes.byref(g), _p(x), _p(w), _p(y)) == 0
    return y


def dgrad(g, dy, w):
    dy, w = _f64(dy, _ys(g)), _f64(w, _ws(g))
    dx = np.empty(_xs(g), dtype=np.float64)
    assert _load().oracle_conv3d_dgrad(ctypes.byref(g), _p(dy), _p(w), _p(dx)) == 0
    return dx


def wgrad(g, x, dy):
    x, dy = _f64(x, _xs(g)), _f64(dy, _ys(g))
    dw = np.empty(_ws(g), dtype=np.float64)
    assert _load().oracle_conv3d_wgrad(ctypes.byref(g), _p(x), _p(dy), _p(dw)) == 0
    return dw


def _idx(idx):
    return np.ascontiguousarray(idx, dtype=np.int64).ravel()


def fwd_at(g, x, w, idx):
    """y at flat NDHWC output indices (inputs float32, arithmetic in double)."""
    x, w, idx = _f32(x, _xs(g)), _f32(w, _ws(g)), _idx(idx)
    out = np.empty(idx.size, dtype=np.float64)
    assert _load().oracle_conv3d_fwd_at(ctypes.byref(g), _p(x), _p(w), _p(idx), ctypes.c_long(idx.size), _p(out)) == 0
    return out


def dgrad_at(g, dy, w, idx):
    """dx at flat NDHWC input indices."""
    dy, w, idx = _f32(dy, _ys(g)), _f32(w, _ws(g)), _idx(idx)
    out = np.empty(idx.size, dtype=np.float64)
    assert _load().oracle_conv3d_dgrad_at(ctypes.byref(g), _p(dy), _p(w), _p(idx), ctypes.c_long(idx.size), _p(out)) == 0
    return out


def wgrad_at(g, x, dy, idx):
    """dw at flat [Cout][kD][kH][kW][Cin] indices."""
    x, dy, idx = _f32(x, _xs(g)), _f32(dy, _ys(g)), _idx(idx)
    out = np.empty(idx.size, dtype=np.float64)
    assert _load().oracle_conv3d_wgrad_at(ctypes.byref(g), _p(x), _p(dy), _p(idx), ctypes.c_long(idx.size), _p(out)) == 0
    return out


def tconv_fwd(z, v):
    """Transposed convolution with stride == kernel, no pad.
    z [N][Dz][Hz][Wz][Ci], v [Ci][kD][kH][kW][Co] -> u [N][Dz*kD][Hz*kH][Wz*kW][Co]."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    N, Dz, Hz, Wz, Ci = z.shape
    Ci2, kD, kH, kW, Co = v.shape
    assert Ci == Ci2
    u = np.empty((N, Dz * kD, Hz * kH, Wz * kW, Co), dtype=np.float64)
    assert _load().oracle_tconv3d_fwd(N, Dz, Hz, Wz, Ci, Co, kD, kH, kW, _p(z), _p(v), _p(u)) == 0
    return u


def rel_err(got, ref):
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)): element-wise relative
    error with an RMS floor (outputs are signed sums, so some |ref_i| ~ 0)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(got - ref) / den))
