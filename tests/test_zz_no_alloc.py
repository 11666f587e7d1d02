"""The entry point that allocates nothing (mi3d_conv3d_wgrad_static: scratch in a static device array of the
library) against mi3d_conv3d_wgrad, through the C ABI: two calls in a row, the second on a smaller input, so that
whatever the first call left in the shared scratch would show."""
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

# (N, D, H, W, Cin, Cout, k, s, p): a 3x3x3 layer over several patches with ragged tails, then smaller ones of the
# same and of other kernel families (stride 2, first layer, up-sampling)
SEQUENCES = [
    [(1, 20, 36, 70, 32, 32, 3, 1, 1), (1, 6, 10, 12, 32, 32, 3, 1, 1)],
    [(2, 12, 24, 40, 64, 32, 3, 1, 1), (1, 12, 14, 34, 32, 64, 3, 2, 1), (1, 9, 19, 33, 4, 32, 3, 1, 1), (1, 8, 8, 16, 32, 64, 2, 2, 0)],
]


@pytest.mark.parametrize("seq", SEQUENCES, ids=["3x3x3", "families"])
def test_static_scratch_weight_gradient_equals_the_workspace_one(device, seq):
    for i, case in enumerate(seq):
        N, D, H, W, Cin, Cout, k, s, p = case
        x, w, dy = si.conv_case(95, 10 * i, N, D, H, W, Cin, Cout, k, s, p, True)
        desc = mc.make_desc(N, D, H, W, Cin, Cout, k, s, p, torch.bfloat16)
        assert 0 < mc.workspace_bytes(desc, mc.PASS_WGRAD) <= mc.static_scratch_bytes()
        xd, dyd = parity.to_device(x, True), parity.to_device(dy, True)
        ref = mc.conv3d_wgrad(desc, xd, dyd)                       # caller-provided workspace
        got = torch.full_like(ref, float("nan"))
        mc.conv3d_wgrad_static(desc, xd, dyd, got)                 # the library's static array
        torch.cuda.synchronize()
        assert torch.equal(got, ref), case                         # same kernels, fixed reduction order: same bits
        g = oc.shape(N, D, H, W, Cin, Cout, k, s, p)
        assert oc.rel_err(got.cpu().numpy(), oc.wgrad(g, x, dy)) <= 1e-2, case


def test_static_scratch_entry_refuses_what_does_not_fit_and_bad_arguments(device):
    l = _lib.lib()
    big = mc.make_desc(1, 16, 16, 32, 1024, 1024, 3, 1, 1, torch.bfloat16)   # 108 MiB of partial sums
    assert mc.workspace_bytes(big, mc.PASS_WGRAD) > mc.static_scratch_bytes()
    buf = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    # refused by size before any pointer is looked at or anything is launched
    assert l.mi3d_conv3d_wgrad_static(ctypes.byref(big), buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), None) == -3
    ok = mc.make_desc(1, 8, 8, 8, 32, 32, 3, 1, 1, torch.bfloat16)
    assert l.mi3d_conv3d_wgrad_static(ctypes.byref(ok), None, buf.data_ptr(), buf.data_ptr(), None) == -1
    assert l.mi3d_conv3d_wgrad_static(ctypes.byref(ok), buf.data_ptr() + 2, buf.data_ptr(), buf.data_ptr(), None) == -1
    assert l.mi3d_conv3d_wgrad_static(None, buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), None) == -1
    torch.cuda.synchronize()
