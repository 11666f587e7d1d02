"""Conv chain step with data swapping: swapped and unswapped runs must give
bit-identical weight gradients, and every layer must match the oracle when
the oracle is fed the GPU's own saved activations (teacher forcing, so bf16
rounding does not compound across layers)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from paper_1812_07816_amd import chain, swap as sw
from tests import parity

pytestmark = pytest.mark.gpu


def _make(vol, **kw):
    layers = [chain.Layer(4, 32), chain.Layer(32, 32), chain.Layer(32, 64, s=2)]
    x0 = si.normal(95, 0, (1, vol, vol, vol, 4), bf16=True)
    ws = [si.he_normal_weight(95, 1 + i, ly.Cout, ly.k, ly.Cin, bf16=True) for i, ly in enumerate(layers)]
    dy = si.normal(95, 9, (1, vol // 2, vol // 2, vol // 2, 64), bf16=True)
    st = chain.ChainStep(1, vol, layers, [parity.to_device(w, True) for w in ws], parity.to_device(x0, True),
                         parity.to_device(dy, True), **kw)
    return st, layers, x0, ws, dy


def test_swapped_step_is_bit_identical_and_matches_oracle(device):
    vol = 24
    ref, layers, x0, ws, dy = _make(vol, swap=False)
    ref.run()
    torch.cuda.synchronize()
    # teacher-forced oracle check of every layer and pass
    acts = [parity.to_host(a) for a in ref.acts]
    grads = [parity.to_host(g) for g in ref.grad]
    for i, ly in enumerate(layers):
        g = oc.shape(1, acts[i].shape[1], acts[i].shape[2], acts[i].shape[3], ly.Cin, ly.Cout, ly.k, ly.s, ly.p)
        y = parity.to_host(ref.acts[i + 1]) if i + 1 < len(layers) else parity.to_host(ref.y_last)
        assert oc.rel_err(y, oc.fwd(g, acts[i], ws[i])) <= 1e-2
        assert oc.rel_err(grads[i], oc.dgrad(g, grads[i + 1], ws[i])) <= 1e-2
        assert oc.rel_err(ref.dw[i].cpu().numpy(), oc.wgrad(g, acts[i], grads[i + 1])) <= 1e-2
    for policy, kw in [(sw.POLICY_ALL, {}), (sw.POLICY_BUDGET, {"budget_bytes": None}),
                       (sw.POLICY_FIRST_N, {"n_tensors": 1}), (sw.POLICY_ALL, {"lookahead": 3})]:
        st, *_ = _make(vol, swap=True, policy=policy, **kw)
        for _ in range(2):     # the second run reuses arena blocks and host slots
            st.run()
        torch.cuda.synchronize()
        for a, b in zip(ref.dw, st.dw):
            assert torch.equal(a, b)
        assert torch.equal(ref.grad[0].view(torch.int16), st.grad[0].view(torch.int16))
        stats = st.engine.stats()
        n_planned = sum(st.planned)
        assert stats["n_swapped_out"] == stats["n_swapped_in"] == n_planned
        if policy == sw.POLICY_ALL:
            assert n_planned == 3 and stats["bytes_out"] == sum(st.saved_bytes)
        if policy == sw.POLICY_BUDGET:
            assert n_planned == 0
        st.close()


def test_budget_forces_minimal_swap(device):
    vol = 24
    probe, *_ = _make(vol, swap=True)
    peak = probe.engine.stats()["unswapped_peak_bytes"]
    probe.close()
    st, *_ = _make(vol, swap=True, budget_bytes=peak - 1024)
    assert st.plan_status == 0 and sum(st.planned) == 1
    st.run()
    torch.cuda.synchronize()
    s = st.engine.stats()
    assert s["planned_peak_bytes"] <= peak - 1024 and s["bytes_out"] == s["bytes_in"] > 0
    st.close()
