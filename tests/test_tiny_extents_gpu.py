"""GPU-vs-oracle parity on degenerate volumes of every MFMA kernel family: extents of one or two voxels, single output
planes, fewer work units than workgroups, patches that hold a single voxel (full fp64 oracle on each case).  The
routing is asserted, so that these shapes do run through the tiled kernels and not through the plain ones."""
import pytest
import torch

from paper_1812_07816_amd import conv3d as mc
from tests import parity

pytestmark = pytest.mark.gpu

CASES = [
    # N, D, H, W, Cin, Cout, k, s, p
    (1, 1, 1, 1, 32, 32, 3, 1, 1),      # one voxel: every tap but the centre falls into the padding
    (2, 1, 5, 9, 32, 64, 3, 1, 1),      # single plane, two samples, two cout tiles
    (1, 2, 1, 40, 64, 32, 3, 1, 1),     # single row
    (1, 1, 2, 2, 128, 32, 3, 1, 1),     # many channels on four voxels
    (1, 2, 2, 1, 320, 320, 3, 1, 1),    # single column, the deepest level's channels
    (1, 1, 1, 1, 32, 64, 3, 2, 1),      # stride 2 on one voxel
    (1, 2, 3, 5, 32, 64, 3, 2, 1),      # stride 2: one output plane, ragged parity classes
    (2, 1, 4, 2, 64, 128, 3, 2, 1),     # stride 2, chunked channels
    (1, 3, 3, 3, 32, 32, 3, 2, 0),      # no padding: a single output voxel
    (1, 1, 1, 1, 4, 32, 3, 1, 1),       # first layer on one voxel
    (1, 1, 3, 7, 4, 32, 3, 1, 1),
    (2, 2, 1, 2, 4, 32, 3, 1, 2),       # pad 2: the output is larger than the input
    (1, 2, 2, 2, 32, 64, 2, 2, 0),      # up-sampling layer, one small-volume voxel
    (1, 2, 4, 2, 64, 128, 2, 2, 0),
    (1, 1, 1, 1, 32, 3, 1, 1, 0),       # head on one voxel
    (2, 1, 1, 5, 64, 2, 1, 1, 0),
]


@pytest.mark.parametrize("case", CASES)
def test_tiny_volume_matches_oracle(device, case):
    N, D, H, W, Cin, Cout, k, s, p = case
    desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16)
    names = [mc.kernel_name(desc, q) for q in range(3)]
    print(case, names, flush=True)
    assert all(n.startswith("mfma_") or n == "valu_pointwise_head" for n in names), names
    errs = parity.run_case(96, 10 * CASES.index(case), N, D, H, W, Cin, Cout, k, s, p, bf16=True, full=True)
    print({q: f"{v:.2e}" for q, v in errs.items()}, flush=True)
    for q, v in errs.items():
        assert v <= parity.TOL["bf16"], (case, q, v)
