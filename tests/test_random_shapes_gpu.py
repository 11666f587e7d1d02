"""GPU-vs-oracle parity on seeded random geometries of every kernel family (full fp64 oracle on each case).

The hand-picked cases of test_conv_parity_gpu.py aim at known tile seams; these cases draw extents, batch sizes,
channel counts and pads at random inside each family's supported range, so that ragged tails and odd extents nobody
thought of are met too.  The list is fixed by its seed: the same cases every run."""
import numpy as np
import pytest
import torch

from paper_1812_07816_amd import conv3d as mc
from tests import parity

pytestmark = pytest.mark.gpu


def _cases():
    r = np.random.RandomState(181207816)
    out = []

    def dims(lo, dmax, hmax, wmax, even=False):
        d, h, w = int(r.randint(lo, dmax + 1)), int(r.randint(lo, hmax + 1)), int(r.randint(lo, wmax + 1))
        if even:
            d, h, w = d + d % 2, h + h % 2, w + w % 2
        return d, h, w

    for _ in range(10):     # 3x3x3 stride 1, channels in multiples of 32: plane streaming, weight gradient
        cin, cout = int(r.choice([32, 64, 96, 128, 160])), int(r.choice([32, 64, 96]))
        p = int(r.choice([0, 1, 1, 2]))
        d, h, w = dims(3, 9, 24, 70)
        out.append(("s1", int(r.randint(1, 3)), d, h, w, cin, cout, 3, 1, p))
    for _ in range(8):      # 3x3x3 stride 2
        cin, cout = int(r.choice([32, 64, 96])), int(r.choice([32, 64, 96, 128]))
        p = int(r.choice([0, 1, 1]))
        d, h, w = dims(4, 13, 22, 72)
        out.append(("s2", int(r.randint(1, 3)), d, h, w, cin, cout, 3, 2, p))
    for _ in range(5):      # first layer
        d, h, w = dims(3, 12, 40, 75)
        out.append(("c4", int(r.randint(1, 3)), d, h, w, 4, 32, 3, 1, int(r.choice([0, 1, 1, 2]))))
    for _ in range(4):      # up-sampling layers (even extents)
        cin, cout = int(r.choice([32, 64])), int(r.choice([64, 128]))
        d, h, w = dims(2, 10, 20, 40, even=True)
        out.append(("k2", int(r.randint(1, 3)), d, h, w, cin, cout, 2, 2, 0))
    for _ in range(3):      # head
        d, h, w = dims(2, 8, 20, 50)
        out.append(("head", int(r.randint(1, 3)), d, h, w, int(r.choice([32, 64])), int(r.randint(1, 5)), 1, 1, 0))
    for _ in range(5):      # anything else: operand embeddings and the plain kernels
        k = int(r.choice([1, 2, 3]))
        s = int(r.choice([1, 2]))
        p = int(r.randint(0, k))
        d, h, w = dims(k + 1, 9, 12, 20)
        out.append(("other", int(r.randint(1, 3)), d, h, w, int(r.choice([3, 8, 16, 40])), int(r.choice([5, 8, 24])), k, s, p))
    return out


CASES = _cases()


@pytest.mark.parametrize("case", CASES, ids=[f"{c[0]}-{i}" for i, c in enumerate(CASES)])
def test_random_geometry_matches_oracle(device, case):
    family, N, D, H, W, Cin, Cout, k, s, p = case
    errs = parity.run_case(97, 10 * CASES.index(case), N, D, H, W, Cin, Cout, k, s, p, bf16=True, full=True)
    desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16)
    names = [mc.kernel_name(desc, q) for q in range(3)]
    print(case, names, {q: f"{v:.2e}" for q, v in errs.items()}, flush=True)
    for q, v in errs.items():
        assert v <= parity.TOL["bf16"], (case, q, v)


def _tall_cases():
    """3x3x3 stride-1 layers on planes of 10 to 60 rows and 9 to 100 columns: one to five patch rows of 16 or 12 rows,
    last columns of patches that are paired two patch rows at a time (at most 16 columns inside the tensor) or not, few
    and many units (chunked, streamed and resident weights).  Sampled oracle: every patch seam plus random positions."""
    r = np.random.RandomState(181207817)
    out = []
    for _ in range(16):
        cin, cout = int(r.choice([32, 64, 128, 256])), int(r.choice([32, 64, 128]))
        d, h, w = int(r.randint(2, 7)), int(r.randint(10, 61)), int(r.randint(9, 101))
        out.append((int(r.randint(1, 4)), d, h, w, cin, cout, 3, 1, int(r.choice([0, 1, 1, 2]))))
    return out


TALL = _tall_cases()


@pytest.mark.parametrize("case", TALL, ids=[f"s1tall-{i}" for i in range(len(TALL))])
def test_random_tall_planes_match_oracle(device, case):
    N, D, H, W, Cin, Cout, k, s, p = case
    errs = parity.run_case(98, 10 * TALL.index(case), N, D, H, W, Cin, Cout, k, s, p, bf16=True, full=False,
                           n_samples=30000, n_wgrad_samples=48)
    print(case, {q: f"{v:.2e}" for q, v in errs.items()}, flush=True)
    for q, v in errs.items():
        assert v <= parity.TOL["bf16"], (case, q, v)
