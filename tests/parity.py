"""Helpers for the GPU-vs-oracle parity tests (GPU side goes through the
C ABI via the ctypes binding; the oracle side is oracle/)."""
import numpy as np
import torch

import synth_inputs as si
from oracle import conv3d as oc
from paper_1812_07816_amd import conv3d as mc

TOL = {"f32": 1e-4, "bf16": 1e-2}   # max |got-ref| / max(|ref|, rms(ref))


def to_device(a, bf16):
    """float32 host array (bf16-exact when bf16=True) -> CUDA tensor."""
    if bf16:
        bits = si.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(a.shape)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t):
    return t.detach().float().cpu().numpy()


def structured_and_random(shape, n_random, seed):
    """Flat indices: every combination of {first, second, a tile seam, last}
    coordinates on each spatial axis (for the first, last and a middle
    channel) plus n_random uniform picks."""
    N, A, B, C, Ch = shape
    def pts(n):
        c = {0, 1, n // 2, n - 2, n - 1, 11, 12, 15, 16, 23, 24, 31, 32, 33, 35, 36, 47, 48, 63, 64, 65}   # seams of 12-, 16- and 32-wide tiles
        return sorted(v for v in c if 0 <= v < n)
    chans = sorted({0, Ch // 2, Ch - 1})
    grid = np.array(np.meshgrid([0, N - 1], pts(A), pts(B), pts(C), chans, indexing="ij")).reshape(5, -1)
    flat = np.ravel_multi_index(tuple(grid), shape)
    total = int(np.prod(shape))
    rnd = np.random.default_rng(seed).integers(0, total, size=n_random)
    return np.unique(np.concatenate([flat, rnd]))


def run_case(config, base_index, N, D, H, W, Cin, Cout, k, s, p, bf16, passes=("fwd", "dgrad", "wgrad"),
             full=None, n_samples=100000, n_wgrad_samples=96):
    """Runs the passes on the GPU and returns {pass: rel_err vs oracle}.
    full=True compares every element (oracle full passes); otherwise sampled."""
    x, w, dy = si.conv_case(config, base_index, N, D, H, W, Cin, Cout, k, s, p, bf16)
    g = oc.shape(N, D, H, W, Cin, Cout, k, s, p)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16 if bf16 else torch.float32)
    if full is None:
        full = x.size * max(Cout, 1) * 27 < 2e9
    xd, wd, dyd = to_device(x, bf16), to_device(w, bf16), to_device(dy, bf16)
    errs = {}
    if "fwd" in passes:
        y = to_host(mc.conv3d_fwd(desc, xd, wd))
        if full:
            errs["fwd"] = oc.rel_err(y, oc.fwd(g, x, w))
        else:
            idx = structured_and_random(y.shape, n_samples, 1)
            ref = oc.fwd_at(g, x, w, idx)
            errs["fwd"] = _sampled_err(y.ravel()[idx], ref)
    if "dgrad" in passes:
        dx = to_host(mc.conv3d_dgrad(desc, dyd, wd))
        if full:
            errs["dgrad"] = oc.rel_err(dx, oc.dgrad(g, dy, w))
        else:
            idx = structured_and_random(dx.shape, n_samples, 2)
            ref = oc.dgrad_at(g, dy, w, idx)
            errs["dgrad"] = _sampled_err(dx.ravel()[idx], ref)
    if "wgrad" in passes:
        dw = to_host(mc.conv3d_wgrad(desc, xd, dyd))
        if full:
            errs["wgrad"] = oc.rel_err(dw, oc.wgrad(g, x, dy))
        else:
            total = dw.size
            idx = np.unique(np.concatenate([
                np.array([0, total - 1]),
                np.random.default_rng(3).integers(0, total, size=n_wgrad_samples)]))
            ref = oc.wgrad_at(g, x, dy, idx)
            errs["wgrad"] = _sampled_err(dw.ravel()[idx], ref)
    torch.cuda.synchronize()
    return errs


def _sampled_err(got, ref):
    return oc.rel_err(got, ref)
