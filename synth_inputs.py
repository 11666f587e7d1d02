"""Seeded synthetic inputs shared by the tests, the smoke check and bench.py.

Holds no convolution arithmetic: only random draws and the one-time rounding
of host values to bfloat16, so that the CPU oracle and the GPU path consume
bit-identical numbers.

Recipe (stands in for the BRATS-2017 volumes of Section 4.1, which are not
available): the four input channels play the role of four z-scored MRI
modalities, i.i.d. N(0,1) per voxel; upstream gradients N(0,1); weights
He-normal with std = sqrt(2 / fan_in), fan_in = kD*kH*kW*Cin.
Generator: numpy Philox, seed = 181207816 + 1000*config + tensor_index.
"""
import numpy as np

BASE_SEED = 181207816


def rng(config, tensor_index):
    return np.random.Generator(np.random.Philox(BASE_SEED + 1000 * int(config) + int(tensor_index)))


def bf16_round(a):
    """Round float32 values to the nearest bfloat16 (ties to even) and return
    them as float32 (low 16 bits zero)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def bf16_bits(a):
    """uint16 bit patterns of float32 values that are already bf16-exact."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16)


def normal(config, tensor_index, shape, std=1.0, bf16=False):
    g = rng(config, tensor_index)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return bf16_round(a) if bf16 else a


def he_normal_weight(config, tensor_index, Cout, k, Cin, bf16=False):
    kD, kH, kW = (k, k, k) if np.isscalar(k) else k
    std = float(np.sqrt(2.0 / (kD * kH * kW * Cin)))
    return normal(config, tensor_index, (Cout, kD, kH, kW, Cin), std=std, bf16=bf16)


def conv_case(config, base_index, N, D, H, W, Cin, Cout, k, s, p, bf16):
    """x, w, dy for one layer; tensor indices base_index, +1, +2."""
    kD, kH, kW = (k, k, k) if np.isscalar(k) else k
    sD, sH, sW = (s, s, s) if np.isscalar(s) else s
    pD, pH, pW = (p, p, p) if np.isscalar(p) else p
    Do = (D + 2 * pD - kD) // sD + 1
    Ho = (H + 2 * pH - kH) // sH + 1
    Wo = (W + 2 * pW - kW) // sW + 1
    x = normal(config, base_index, (N, D, H, W, Cin), bf16=bf16)
    w = he_normal_weight(config, base_index + 1, Cout, (kD, kH, kW), Cin, bf16=bf16)
    dy = normal(config, base_index + 2, (N, Do, Ho, Wo, Cout), bf16=bf16)
    return x, w, dy
