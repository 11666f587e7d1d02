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


CHUNK = 1 << 24   # elements per independently generated piece of a large tensor


def normal(config, tensor_index, shape, std=1.0, bf16=False):
    """N(0, std^2) float32 values (bf16-exact if bf16).  Tensors of up to CHUNK elements come from one Philox stream;
    larger ones are filled in pieces of CHUNK elements, piece i from the tensor's stream jumped i + 1 times, on a few
    threads (the values depend on the seed and the shape only, not on the number of threads)."""
    n = int(np.prod(shape))
    if n <= CHUNK:
        a = rng(config, tensor_index).standard_normal(size=shape, dtype=np.float32)
        if std != 1.0:
            a *= np.float32(std)
        return bf16_round(a) if bf16 else a
    import concurrent.futures
    import os
    out = np.empty(n, dtype=np.float32)
    seed = BASE_SEED + 1000 * int(config) + int(tensor_index)

    def fill(i):
        piece = out[i * CHUNK:(i + 1) * CHUNK]
        g = np.random.Generator(np.random.Philox(seed).jumped(i + 1))
        g.standard_normal(size=piece.shape, dtype=np.float32, out=piece)
        if std != 1.0:
            piece *= np.float32(std)
        if bf16:
            piece[:] = bf16_round(piece)

    workers = max(1, min(16, len(os.sched_getaffinity(0))))
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(fill, range((n + CHUNK - 1) // CHUNK)))
    return out.reshape(shape)


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


# ---- whole-network inputs (full training step of the 5-level U-Net) -----------------------------

def unet_weight_shapes(channels, in_ch=4, classes=3):
    """[(name, (Cout, k, k, k, Cin))] in the fixed order used by every consumer:
    encoder convs level by level, then per decoder level (deepest first) the
    up-sampling weights and the two convs, then the 1x1x1 head.  The
    up-sampling layer is stored as the weights of the 2x2x2 / stride-2
    convolution whose data gradient it is: [C_deep][2][2][2][C_shallow]."""
    out = []
    prev = in_ch
    for l, c in enumerate(channels):
        out.append((f"enc{l}.conv1", (c, 3, 3, 3, prev)))
        out.append((f"enc{l}.conv2", (c, 3, 3, 3, c)))
        prev = c
    for l in range(len(channels) - 2, -1, -1):
        c, deep = channels[l], channels[l + 1]
        out.append((f"dec{l}.up", (deep, 2, 2, 2, c)))
        out.append((f"dec{l}.conv1", (c, 3, 3, 3, 2 * c)))
        out.append((f"dec{l}.conv2", (c, 3, 3, 3, c)))
    out.append(("head", (classes, 1, 1, 1, channels[0])))
    return out


def unet_weights(config, channels, in_ch=4, classes=3, bf16=True):
    """He-normal weights (std = sqrt(2 / fan_in); fan_in = k^3 Cin for a
    convolution, the number of input channels C_deep for the up-sampling layer,
    where every output voxel sees one tap), tensor indices 100, 101, ..."""
    ws = []
    for i, (name, shp) in enumerate(unet_weight_shapes(channels, in_ch, classes)):
        fan_in = shp[0] if name.endswith(".up") else shp[1] * shp[2] * shp[3] * shp[4]
        ws.append(normal(config, 100 + i, shp, std=float(np.sqrt(2.0 / fan_in)), bf16=bf16))
    return ws


def ellipsoid_labels(config, tensor_index, N, vol, classes=3):
    """uint8 [N, vol, vol, vol, classes]: per sample and class the union of 1-8
    axis-aligned ellipsoids, centres uniform over the volume, per-axis radii
    uniform in 8..48 voxels at vol = 192 (scaled with vol, at least 1).
    Classes are drawn independently and may overlap.  Stands in for the tumour
    sub-region labels of Section 4.1."""
    g = rng(config, tensor_index)
    lab = np.zeros((N, vol, vol, vol, classes), dtype=np.uint8)
    ax = np.arange(vol, dtype=np.float32)
    lo, hi = max(1, round(8 * vol / 192)), max(2, round(48 * vol / 192))
    for n in range(N):
        for c in range(classes):
            for _ in range(int(g.integers(1, 9))):
                ctr = g.uniform(0, vol, size=3)
                rad = g.integers(lo, hi + 1, size=3).astype(np.float32)
                dz = ((ax - ctr[0]) / rad[0]) ** 2
                dy = ((ax - ctr[1]) / rad[1]) ** 2
                dx = ((ax - ctr[2]) / rad[2]) ** 2
                inside = dz[:, None, None] + dy[None, :, None] + dx[None, None, :] <= 1.0
                lab[n, ..., c] |= inside.astype(np.uint8)
    return lab
