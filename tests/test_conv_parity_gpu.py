"""GPU-vs-oracle parity of conv3d_fwd / dgrad / wgrad through the C ABI.

Tolerances (max |got-ref| / max(|ref|, rms(ref))): 1e-4 for the fp32 path,
1e-2 for bf16 inputs with fp32 accumulation and bf16-rounded outputs."""
import ctypes

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from paper_1812_07816_amd import _lib
from paper_1812_07816_amd import conv3d as mc
from tests import parity

pytestmark = pytest.mark.gpu


def _check(errs, bf16, what):
    tol = parity.TOL["bf16" if bf16 else "f32"]
    print(what, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= tol, (what, k, v)


# ---- config 1: single fp32 layer, full comparison --------------------------
def test_config1_fp32_16cube(device):
    _check(parity.run_case(1, 0, 1, 16, 16, 16, 4, 8, 3, 1, 1, bf16=False, full=True), False, "cfg1")


SMALL = [
    # N, D, H, W, Cin, Cout, k, s, p   (ragged sizes, several tiles, odd tails)
    (1, 5, 6, 7, 3, 5, 3, 1, 1),
    (2, 9, 10, 37, 4, 8, 3, 1, 1),
    (1, 7, 9, 11, 2, 3, 3, 2, 1),
    (1, 8, 8, 8, 5, 4, 3, 2, 0),
    (2, 6, 5, 9, 8, 3, 1, 1, 0),
    (1, 6, 8, 10, 6, 4, 2, 2, 0),
    (1, 4, 5, 7, 2, 2, (1, 2, 3), (1, 2, 1), (0, 1, 2)),
    (1, 3, 3, 3, 1, 1, 3, 1, 1),
    (1, 1, 1, 1, 1, 1, 1, 1, 0),
]


@pytest.mark.parametrize("case", SMALL)
@pytest.mark.parametrize("bf16", [False, True])
def test_small_ragged_shapes_full(device, case, bf16):
    _check(parity.run_case(90, 10 * SMALL.index(case), *case, bf16=bf16, full=True), bf16, f"small{case}")


MID = [
    # shapes that exercise the tuned-kernel tile seams; full oracle in seconds
    (1, 10, 20, 40, 32, 32, 3, 1, 1),
    (2, 6, 18, 70, 32, 32, 3, 1, 1),
    (1, 9, 17, 33, 32, 32, 3, 1, 1),
    (1, 8, 16, 32, 64, 32, 3, 1, 1),
    (1, 12, 14, 34, 32, 64, 3, 2, 1),
    (1, 9, 21, 37, 32, 32, 3, 2, 1),
    (1, 8, 10, 12, 32, 96, 3, 2, 0),
    (1, 7, 9, 20, 64, 64, 3, 1, 1),
    (1, 6, 6, 12, 128, 64, 3, 1, 1),
    (1, 12, 12, 12, 64, 128, 3, 2, 1),
    (1, 4, 4, 6, 320, 320, 3, 1, 1),
    (1, 4, 6, 6, 256, 320, 3, 2, 1),
    (2, 12, 20, 36, 4, 32, 3, 1, 1),
    (1, 5, 19, 45, 4, 32, 3, 1, 0),
    (1, 4, 16, 33, 4, 32, 3, 1, 2),
    (2, 7, 11, 70, 4, 32, 3, 1, 1),
    (1, 5, 6, 35, 3, 40, 3, 1, 1),
    (2, 3, 9, 31, 1, 8, 3, 1, 0),
    (1, 6, 10, 40, 32, 3, 1, 1, 0),
    (1, 8, 8, 16, 32, 64, 2, 2, 0),
    (2, 6, 10, 14, 64, 128, 2, 2, 0),
    (1, 4, 6, 6, 256, 320, 2, 2, 0),
    (1, 4, 4, 8, 32, 96, 2, 2, 0),
    # a last column of patches at most half inside the tensor, taken two patch rows at a time (12-row patches)
    (1, 5, 24, 48, 32, 32, 3, 1, 1),
    (2, 4, 36, 16, 64, 64, 3, 1, 1),      # no other column; odd number of patch rows
    (1, 4, 48, 48, 128, 64, 3, 1, 1),     # streamed weights
    (1, 5, 26, 50, 32, 32, 3, 1, 0),      # 24 x 48 output without padding
    (1, 5, 22, 46, 64, 32, 3, 1, 2),      # 24 x 48 output, padding 2
]


@pytest.mark.parametrize("case", MID)
def test_mid_shapes_bf16_full(device, case):
    _check(parity.run_case(91, 10 * MID.index(case), *case, bf16=True, full=True), True, f"mid{case}")


# ---- the fp32 path on the fp32 matrix cores: every kind of layer of the network, full oracle, 1e-4
MID_F32 = [
    (1, 10, 20, 40, 32, 32, 3, 1, 1),
    (2, 6, 18, 70, 32, 32, 3, 1, 1),
    (1, 9, 17, 33, 4, 32, 3, 1, 1),
    (1, 8, 16, 32, 64, 32, 3, 1, 1),
    (1, 12, 14, 34, 32, 64, 3, 2, 1),
    (1, 9, 21, 37, 32, 32, 3, 2, 1),
    (1, 8, 10, 12, 32, 96, 3, 2, 0),
    (1, 6, 6, 12, 128, 64, 3, 1, 1),
    (1, 4, 4, 6, 320, 320, 3, 1, 1),
    (1, 4, 6, 6, 256, 320, 3, 2, 1),
    (1, 5, 19, 45, 4, 32, 3, 1, 0),
    (1, 4, 16, 33, 4, 32, 3, 1, 2),
    (1, 6, 10, 40, 32, 3, 1, 1, 0),
    (2, 5, 9, 13, 64, 4, 1, 1, 0),
    (3, 4, 5, 7, 8, 1, 1, 1, 0),
    (1, 3, 5, 9, 16, 2, 1, 1, 0),
    (1, 8, 8, 16, 32, 64, 2, 2, 0),
    (2, 6, 10, 14, 64, 128, 2, 2, 0),
    (1, 7, 9, 11, 6, 10, 3, 2, 1),
    (1, 6, 7, 9, 34, 36, (3, 2, 3), (1, 2, 1), (1, 0, 2)),
    # planes that 16 x 16 (weight gradient: 4 x 16) tiles cover better than 8 x 32 (2 x 32)
    (1, 4, 30, 46, 32, 64, 3, 1, 1),
    (2, 5, 31, 93, 32, 64, 3, 2, 1),
    (1, 4, 11, 12, 64, 96, 3, 1, 1),
    (1, 4, 22, 24, 32, 64, 2, 2, 0),
]


@pytest.mark.parametrize("case", MID_F32)
def test_mid_shapes_fp32_full(device, case):
    desc = mc.make_desc(*case, torch.float32)
    head = case[6] == 1 and case[5] <= 4     # 1x1x1 to a handful of channels: VALU kernels
    fold = case[4] <= 4 and case[6] == 3 and case[7] == 1 and case[5] % 4 == 0   # few input channels: taps folded into the weight gradient's columns
    for q in range(3):
        want = "valu_pointwise_head_f32" if head else "mfma_f32_wgrad_cin4_folded_taps" if fold and q == 2 else "mfma_f32_gather"
        assert mc.kernel_name(desc, q) == want
    _check(parity.run_case(96, 10 * MID_F32.index(case), *case, bf16=False, full=True), False, f"mid fp32 {case}")


# ---- config 2: 128^3 first level ------------------------------------------
@pytest.mark.parametrize("cin", [4, 32])
def test_config2_128cube(device, cin):
    _check(parity.run_case(2, 10 * (cin == 32), 1, 128, 128, 128, cin, 32, 3, 1, 1, bf16=True, full=False), True, f"cfg2 {cin}->32")


# ---- config 3: 192^3 first level + stride-2 downsampling -------------------
@pytest.mark.parametrize("layer", [(4, 32, 1), (32, 32, 1), (32, 64, 2)])
def test_config3_192cube(device, layer):
    cin, cout, s = layer
    _check(parity.run_case(3, 10 * [4, 32].index(cin) + 20 * (s == 2), 1, 192, 192, 192, cin, cout, 3, s, 1,
                           bf16=True, full=False), True, f"cfg3 {cin}->{cout} s{s}")


# ---- the second workload shape: a 208^3 volume (Section 5), whose extents are no multiple of the 32-column patches
@pytest.mark.parametrize("layer", [(208, 4, 32, 3, 1, 1), (208, 32, 32, 3, 1, 1), (208, 32, 64, 3, 2, 1), (104, 64, 64, 3, 1, 1),
                                   (26, 256, 320, 3, 2, 1), (13, 320, 320, 3, 1, 1), (26, 256, 320, 2, 2, 0), (208, 32, 64, 2, 2, 0)])
def test_208cube_layers(device, layer):
    vol, cin, cout, k, s, p = layer
    _check(parity.run_case(6, 10 * (cin % 7) + vol % 5, 1, vol, vol, vol, cin, cout, k, s, p, bf16=True, full=False,
                           n_samples=40000, n_wgrad_samples=48), True, f"208 {layer}")


# ---- the fp32 step's layers at their own size (N = 2): launch shapes that depend on the size of the grid (32- or
# 64-channel workgroups, 8 x 32 or 16 x 16 tiles, merged parity classes, folded taps), sampled against the oracle
FULL_F32 = [(192, 4, 32, 3, 1, 1), (192, 32, 32, 3, 1, 1), (96, 64, 128, 3, 2, 1), (48, 128, 128, 3, 1, 1), (24, 256, 256, 3, 1, 1),
            (12, 320, 320, 3, 1, 1), (192, 32, 64, 2, 2, 0), (192, 32, 3, 1, 1, 0)]


@pytest.mark.parametrize("layer", FULL_F32)
def test_fp32_layers_at_the_size_of_the_step(device, layer):
    vol, cin, cout, k, s, p = layer
    _check(parity.run_case(5, 100 + 10 * FULL_F32.index(layer), 2, vol, vol, vol, cin, cout, k, s, p, bf16=False, full=False,
                           n_samples=40000, n_wgrad_samples=48), False, f"fp32 N=2 {layer}")


# ---- config 4: every layer shape of the 5-level U-Net at 192^3 -------------
CH = [32, 64, 128, 256, 320]
VOL = [192, 96, 48, 24, 12]


def unet_layers():
    """(name, vol_in, Cin, Cout, k, s, p, transposed) for the 23 layers."""
    L = [("enc0.conv1", 192, 4, 32, 3, 1, 1, False), ("enc0.conv2", 192, 32, 32, 3, 1, 1, False)]
    for l in range(1, 5):
        L.append((f"enc{l}.conv1", VOL[l - 1], CH[l - 1], CH[l], 3, 2, 1, False))
        L.append((f"enc{l}.conv2", VOL[l], CH[l], CH[l], 3, 1, 1, False))
    for l in range(3, -1, -1):
        # transposed conv C_{l+1} -> C_l == data-gradient of a k2/s2/p0 conv with
        # Cin' = C_l (fine side), Cout' = C_{l+1} (coarse side) on the fine volume
        L.append((f"dec{l}.up", VOL[l], CH[l], CH[l + 1], 2, 2, 0, True))
        L.append((f"dec{l}.conv1", VOL[l], 2 * CH[l], CH[l], 3, 1, 1, False))
        L.append((f"dec{l}.conv2", VOL[l], CH[l], CH[l], 3, 1, 1, False))
    L.append(("head.1x1", 192, 32, 3, 1, 1, 0, False))
    return L


LAYERS = unet_layers()
# the 192^3 stride-1/2 3x3x3 layers with C<=64 are covered by the config-3 tests
CFG4 = [l for l in LAYERS if l[0] not in ("enc0.conv1", "enc0.conv2", "dec0.conv2", "enc1.conv1")]


def test_unet_layer_table_matches_the_stated_totals():
    assert len(LAYERS) == 23
    flop = 0
    for (_n, vol, cin, cout, k, s, _p, _t) in LAYERS:
        vo = vol // s
        flop += 2 * vo ** 3 * k ** 3 * cin * cout
    assert abs(flop / 1e9 - 3227) < 2          # GFLOP per pass at N=1


@pytest.mark.parametrize("layer", CFG4, ids=[l[0] for l in CFG4])
def test_config4_layer(device, layer):
    name, vol, cin, cout, k, s, p, _t = layer
    i = [l[0] for l in LAYERS].index(name)
    _check(parity.run_case(4, 10 * i, 1, vol, vol, vol, cin, cout, k, s, p, bf16=True, full=False,
                           n_samples=50000, n_wgrad_samples=64), True, f"cfg4 {name}")


def test_transposed_conv_role_swap_matches_direct_oracle(device):
    # decoder upsampling z[.,j,ci] -> u[.,2j+t,co] run as conv3d_dgrad with roles swapped
    N, Dz, Ci, Co = 1, 6, 64, 32
    z = si.normal(92, 0, (N, Dz, Dz, Dz, Ci), bf16=True)
    v = si.normal(92, 1, (Ci, 2, 2, 2, Co), std=float(np.sqrt(2.0 / Ci)), bf16=True)
    desc = mc.make_desc(N, 2 * Dz, 2 * Dz, 2 * Dz, Co, Ci, 2, 2, 0, torch.bfloat16)
    u = parity.to_host(mc.conv3d_dgrad(desc, parity.to_device(z, True), parity.to_device(v, True)))
    assert oc.rel_err(u, oc.tconv_fwd(z, v)) <= 1e-2


# ---- batch 2, determinism, overwrite semantics, error paths ----------------
def test_batch2_192_level0_sampled(device):
    _check(parity.run_case(5, 0, 2, 64, 64, 96, 32, 32, 3, 1, 1, bf16=True, full=False), True, "N=2")


# ---- config 5's own shapes: batch 2 at full size.  The dispatcher counts work units, so several layers take another
# kernel variant (or another unit mapping of the same one) at N = 2 than at N = 1: the 24^3 layers run the
# streamed-weight plane kernel instead of the chunked one, and every persistent kernel deals twice the units.
N2_LAYERS = [
    # name, vol, Cin, Cout, k, s, p, kernels (fwd, dgrad, wgrad)
    ("enc0.conv1", 192, 4, 32, 3, 1, 1, ("mfma_cin4_folded_taps", "mfma_dgrad_cin4_folded_taps", "mfma_wgrad_cin4_folded_taps")),
    ("enc0.conv2", 192, 32, 32, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("dec0.conv1", 192, 64, 32, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("enc1.conv1", 192, 32, 64, 3, 2, 1, ("mfma_stride2_plane_stream", "mfma_dgrad_stride2_parity", "mfma_wgrad_stride2")),
    ("dec0.up", 192, 32, 64, 2, 2, 0, ("mfma_k2s2_panel_gemm",) * 3),
    ("head.1x1", 192, 32, 3, 1, 1, 0, ("valu_pointwise_head",) * 3),
    ("enc2.conv1", 96, 64, 128, 3, 2, 1, ("mfma_stride2_plane_stream", "mfma_dgrad_stride2_parity", "mfma_wgrad_stride2")),
    ("dec1.conv1", 96, 128, 64, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("dec2.conv1", 48, 256, 128, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("enc3.conv2", 24, 256, 256, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("dec3.conv1", 24, 512, 256, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("enc4.conv1", 24, 256, 320, 3, 2, 1, ("mfma_stride2_plane_stream", "mfma_dgrad_stride2_parity", "mfma_wgrad_stride2")),
    ("enc4.conv2", 12, 320, 320, 3, 1, 1, ("mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream")),
    ("dec3.up", 24, 256, 320, 2, 2, 0, ("mfma_k2s2_panel_gemm",) * 3),
]


@pytest.mark.parametrize("layer", N2_LAYERS, ids=[l[0] for l in N2_LAYERS])
def test_config5_batch2_layers_at_full_size(device, layer):
    name, vol, cin, cout, k, s, p, kernels = layer
    desc = mc.make_desc(2, vol, vol, vol, cin, cout, k, s, p, torch.bfloat16)
    assert tuple(mc.kernel_name(desc, q) for q in range(3)) == kernels
    i = [l[0] for l in N2_LAYERS].index(name)
    _check(parity.run_case(5, 300 + 10 * i, 2, vol, vol, vol, cin, cout, k, s, p, bf16=True, full=False,
                           n_samples=30000, n_wgrad_samples=32), True, f"cfg5 N=2 {name}")


def test_wgrad_is_bit_reproducible_and_overwrites(device):
    x, w, dy = si.conv_case(93, 0, 1, 12, 20, 36, 32, 32, 3, 1, 1, True)
    desc = mc.make_desc(1, 12, 20, 36, 32, 32, 3, 1, 1, torch.bfloat16)
    xd, dyd = parity.to_device(x, True), parity.to_device(dy, True)
    dw = torch.full((32, 3, 3, 3, 32), 7.0, device="cuda")
    a = mc.conv3d_wgrad(desc, xd, dyd, dw=dw).clone()
    b = mc.conv3d_wgrad(desc, xd, dyd, dw=dw).clone()
    assert torch.equal(a, b)
    assert oc.rel_err(a.cpu().numpy(), oc.wgrad(oc.shape(1, 12, 20, 36, 32, 32, 3, 1, 1), x, dy)) <= 1e-2


def test_outputs_are_fully_overwritten(device):
    # stride-2 dgrad leaves input positions nobody read: they must become 0
    desc = mc.make_desc(1, 6, 6, 6, 32, 32, 3, 2, 0, torch.bfloat16)
    dy = torch.ones((1, 2, 2, 2, 32), dtype=torch.bfloat16, device="cuda")
    w = torch.ones((32, 3, 3, 3, 32), dtype=torch.bfloat16, device="cuda")
    dx = torch.full((1, 6, 6, 6, 32), float("nan"), dtype=torch.bfloat16, device="cuda")
    mc.conv3d_dgrad(desc, dy, w, dx=dx)
    assert not torch.isnan(dx).any()
    assert float(dx[0, 5].abs().max()) == 0.0 and float(dx[0, 2, 2, 2, 0]) == 8 * 32


def test_error_paths_launch_nothing(device):
    l = _lib.lib()
    desc = mc.make_desc(1, 8, 8, 8, 32, 32, 3, 1, 1, torch.bfloat16)
    x = torch.zeros((1, 8, 8, 8, 32), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((32, 3, 3, 3, 32), dtype=torch.bfloat16, device="cuda")
    dw = torch.zeros((32, 3, 3, 3, 32), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(mc.workspace_bytes(desc, mc.PASS_WGRAD), 64), dtype=torch.uint8, device="cuda")
    p = ctypes.byref(desc)
    assert l.mi3d_conv3d_fwd(p, x.data_ptr() + 2, w.data_ptr(), x.data_ptr(), None, 0, None) == -1   # misaligned
    assert l.mi3d_conv3d_fwd(p, x.data_ptr(), None, x.data_ptr(), None, 0, None) == -1               # null
    need = mc.workspace_bytes(desc, mc.PASS_WGRAD)
    if need:
        assert l.mi3d_conv3d_wgrad(p, x.data_ptr(), x.data_ptr(), dw.data_ptr(), ws.data_ptr(), need - 1, None) == -3
    torch.cuda.synchronize()
