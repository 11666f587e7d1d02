"""Whole training step on the GPU (every step through the C ABI) against the
fp64 oracle at a reduced volume, and swap-on against swap-off.

Two bf16 pipelines whose sums differ in the last bit do not stay within a
fixed tolerance of each other over 23 layers: a difference far below one bf16
ulp becomes a different rounding for some elements of the next stored tensor,
and values near zero then take the other LeakyReLU branch, which changes their
gradient a hundredfold (measured: 6 % L2 difference of the first backward
tensor although the logits agree to 0.5 %).  The step is therefore checked

  (a) op by op, each op's output against the oracle's definition of that op
      applied to the tensors the GPU step itself fed it (bf16 tolerance 1e-2
      of max(|ref|, rms(ref)); fp32 weight gradients likewise); this covers
      every kernel call and which tensor goes where;
  (b) end to end against the oracle step on the same inputs: loss within 1e-4
      relative and every weight gradient pointing the same way (cosine
      similarity >= 0.97), which the wrong graph (a dropped skip gradient, a
      transposed operand) does not survive;
  (c) swap on against swap off: bit-identical.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import conv3d as oc
from oracle import unet as ou

pytestmark = pytest.mark.gpu

CH = [32, 64, 128, 256, 320]
TOL = 1e-2


@pytest.fixture(scope="module")
def unet():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1812_07816_amd import unet as u
    return u


def _inputs(N, vol, channels, config):
    x = si.normal(config, 0, (N, vol, vol, vol, 4), bf16=True)
    labels = si.ellipsoid_labels(config, 1, N, vol)
    ws = si.unet_weights(config, channels)
    xd = torch.from_numpy(si.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16).reshape(x.shape)
    return x, labels, ws, xd, torch.from_numpy(labels).cuda()


def _h(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


# 48 = 16 x 3: odd extents at the two deepest levels, as in the 208^3 volume (16 x 13)
# (last flag: the decoder reads [up-sampled | skip] as two tensors / materialises the concatenation)
# (last flag but one: fp32 step, every convolution on the fp32 matrix cores, tolerance 1e-4)
@pytest.mark.parametrize("N,vol,channels,virtual_cat,f32", [(2, 32, CH, True, False), (1, 16, CH[:4], True, False), (1, 48, CH, True, False),
                                                            (2, 32, CH, False, False), (2, 32, CH, True, True), (1, 48, CH, True, True)])
def test_every_op_matches_oracle_on_the_steps_own_tensors(unet, N, vol, channels, virtual_cat, f32):
    x, labels, ws, xd, ld = _inputs(N, vol, channels, 5)
    L = len(channels)
    TOL = 1e-4 if f32 else 1e-2
    if f32:
        xd = xd.float()
    step = unet.UNetStep(N, vol, channels, ws, xd, ld, swap=False, virtual_cat=virtual_cat, dtype=torch.float32 if f32 else torch.bfloat16)
    if f32:
        # (the head runs through VALU kernels of its own, every other layer on the fp32 matrix cores)
        def expected(op, q):
            if op["kind"] == "head":
                return "valu_pointwise_head_f32"
            return "mfma_f32_wgrad_cin4_folded_taps" if q == 2 and op["name"] == "enc0.conv1" else "mfma_f32_gather"
        assert all(unet.mc.kernel_name(op["desc"], q) == expected(op, q) for op in step.ops if "desc" in op for q in range(3))
    assert all(op["virtual"] == virtual_cat for op in step.ops if op["kind"] == "cat")
    tr = {}
    step.run(update=False, trace=tr)
    torch.cuda.synchronize()
    t = {k: _h(v) for k, v in tr.items()}
    w = {n: np.asarray(a, dtype=np.float64) for (n, _), a in zip(si.unet_weight_shapes(channels), ws)}
    dw = {n: _h(g) for (n, _), g in zip(si.unet_weight_shapes(channels), step.dw)}
    worst = [0.0, ""]

    def close(name, got, ref):
        e = oc.rel_err(got, ref)
        if e > worst[0]:
            worst[:] = [e, name]
        assert e <= TOL, (name, e)

    assert np.array_equal(t["input.a"], x.astype(np.float64))
    # ---- the graph, written out here independently of the driver: (name, input tensor, volume in, Cin, Cout, stride)
    convs, v, prev, cin = [], vol, "input", 4
    for l in range(L):
        s = 1 if l == 0 else 2
        convs.append((f"enc{l}.conv1", prev, v, cin, channels[l], s)); v //= s
        convs.append((f"enc{l}.conv2", f"enc{l}.conv1", v, channels[l], channels[l], 1))
        prev, cin = f"enc{l}.conv2", channels[l]
    ups = []
    for l in range(L - 2, -1, -1):
        v *= 2
        ups.append((f"dec{l}", prev, v, channels[l], channels[l + 1]))
        convs.append((f"dec{l}.conv1", f"dec{l}.cat", v, 2 * channels[l], channels[l], 1))
        convs.append((f"dec{l}.conv2", f"dec{l}.conv1", v, channels[l], channels[l], 1))
        prev = f"dec{l}.conv2"
    # ---- forward ops
    for name, src, vin, ci, co, s in convs:
        g = oc.shape(N, vin, vin, vin, ci, co, 3, s, 1)
        close(name + " fwd", t[name + ".a"], ou._lrelu(oc.fwd(g, t[src + ".a"], w[name])))
    for dn, src, vbig, c, deep in ups:
        g = oc.shape(N, vbig, vbig, vbig, c, deep, 2, 2, 0)
        close(dn + ".up fwd", t[dn + ".up.a"], oc.tconv_fwd(t[src + ".a"], w[dn + ".up"]))
        l = int(dn[3:])
        assert np.array_equal(t[dn + ".cat.a"], np.concatenate([t[dn + ".up.a"], t[f"enc{l}.conv2.a"]], axis=-1))
    gh = oc.shape(N, vol, vol, vol, channels[0], 3, 1, 1, 0)
    close("head fwd", t["head.a"], oc.fwd(gh, t["dec0.conv2.a"], w["head"]))
    loss_ref, dl_ref = ou.dice_loss(t["head.a"], labels)
    assert abs(float(step.loss.item()) - loss_ref) <= 1e-5
    close("loss grad", t["loss.din"], dl_ref)
    # ---- backward ops
    close("head wgrad", dw["head"], oc.wgrad(gh, t["dec0.conv2.a"], t["head.dout"]))
    close("head dgrad", t["head.din"], ou._lrelu_grad(t["dec0.conv2.a"], oc.dgrad(gh, t["head.dout"], w["head"])))
    # The LeakyReLU derivative of a layer is applied by whoever hands the gradient down to it where that is one
    # call: the second convolution of a level (to the first), the head (to the last convolution) and the pass that
    # adds the skip half of a concatenated gradient (to the skip tensor's producer).  Elsewhere (below an
    # up-sampling layer) it is a step of its own.
    through = {name: src for name, src, *_ in convs if name.endswith("conv2")}
    skip_src = {f"enc{l}.conv2" for l in range(L - 1)}
    handed_down = set(through.values()) | skip_src | {"dec0.conv2"}
    for name, src, vin, ci, co, s in convs:
        g = oc.shape(N, vin, vin, vin, ci, co, 3, s, 1)
        if name in handed_down:
            assert np.array_equal(t[name + ".dz"], t[name + ".dout"])
        else:
            dz_ref = ou._lrelu_grad(t[name + ".a"], t[name + ".dout"])     # the output has the sign of the pre-activation
            close(name + " lrelu bwd", t[name + ".dz"], dz_ref)
        close(name + " wgrad", dw[name], oc.wgrad(g, t[src + ".a"], t[name + ".dz"]))
        if name == "enc0.conv1":
            assert name + ".din" not in t
            continue
        din_ref = oc.dgrad(g, t[name + ".dz"], w[name])
        if name in through:
            din_ref = ou._lrelu_grad(t[src + ".a"], din_ref)
        if name.startswith("enc") and name.endswith("conv1") and name + ".skip_add" in t:
            # (fp32 step: the skip tensor's second gradient joins inside the data-gradient call, no rounding between)
            l = int(name[3]) - 1
            assert np.array_equal(t[name + ".skip_add"], t[f"dec{l}.cat.dskip"])
            close(name + " dgrad + skip", t[name + ".din"], ou._lrelu_grad(t[src + ".a"], din_ref + t[name + ".skip_add"]))
        elif name.startswith("enc") and name.endswith("conv1"):          # its input is a skip tensor: second gradient
            l = int(name[3]) - 1
            close(name + " dgrad", t[name + ".dgrad"], din_ref)
            close(name + " skip add", t[name + ".din"], ou._lrelu_grad(t[src + ".a"], t[name + ".dgrad"] + t[f"dec{l}.cat.dskip"]))
        else:
            close(name + " dgrad", t[name + ".din"], din_ref)
    for dn, src, vbig, c, deep in ups:
        g = oc.shape(N, vbig, vbig, vbig, c, deep, 2, 2, 0)
        dcat = t[dn + ".cat.dout"]
        assert np.array_equal(t[dn + ".cat.din"], dcat[..., :c]) and np.array_equal(t[dn + ".cat.dskip"], dcat[..., c:])
        close(dn + ".up wgrad", dw[dn + ".up"], oc.wgrad(g, t[dn + ".up.dout"], t[src + ".a"]))
        close(dn + ".up dgrad", t[dn + ".up.din"], oc.fwd(g, t[dn + ".up.dout"], w[dn + ".up"]))
    # the gradient that enters an op is the one that left its consumer
    for name, src, *_ in convs:
        if name != "enc0.conv1" and not src.endswith(".cat"):
            assert np.array_equal(t[src + ".dout"], t[name + ".din"]), (name, src)
    assert np.array_equal(t["dec0.conv2.dout"], t["head.din"]) and np.array_equal(t["head.dout"], t["loss.din"])
    print(f"worst op error {worst[0]:.2e} ({worst[1]})")


def test_step_end_to_end_against_oracle_step(unet):
    N, vol = 2, 32
    x, labels, ws, xd, ld = _inputs(N, vol, CH, 5)
    lr = 1e-2
    step = unet.UNetStep(N, vol, CH, ws, xd, ld, lr=lr, swap=False)
    step.run(update=True)
    torch.cuda.synchronize()
    loss_ref, grads_ref, _ = ou.train_step(x.astype(np.float64), labels, ws, CH, lr, q=ou.bf16)
    assert abs(float(step.loss.item()) - loss_ref) <= 1e-4 * abs(loss_ref)
    for (name, _), g, r, wm, w0 in zip(si.unet_weight_shapes(CH), step.dw, grads_ref, step.wm, ws):
        gg = _h(g)
        cos = np.sum(gg * r) / np.sqrt(np.sum(gg * gg) * np.sum(r * r))
        assert cos >= 0.97, (name, cos)
        assert 0.9 <= np.sqrt(np.sum(gg * gg) / np.sum(r * r)) <= 1.1, name
        # SGD on the fp32 master weights with the GPU's own gradient
        expect = w0.astype(np.float32) - np.float32(lr) * g.cpu().numpy()
        assert np.allclose(wm.cpu().numpy(), expect, rtol=1e-6, atol=1e-8), name


def test_fp32_step_end_to_end_against_the_exact_oracle_step(unet):
    """In fp32 the GPU pipeline and the fp64 oracle step stay together over all 23 layers (no storage rounding that
    could tip a value over a LeakyReLU kink by more than 1e-7 of its size), so the whole step is pinned tightly: loss,
    length and direction of every weight gradient, and the updated weights."""
    N, vol = 2, 32
    x, labels, ws, xd, ld = _inputs(N, vol, CH, 5)
    lr = 1e-2
    step = unet.UNetStep(N, vol, CH, ws, xd.float(), ld, lr=lr, swap=False, dtype=torch.float32)
    step.run(update=True)
    torch.cuda.synchronize()
    loss_ref, grads_ref, w_ref = ou.train_step(x.astype(np.float64), labels, ws, CH, lr)
    assert abs(float(step.loss.item()) - loss_ref) <= 1e-5 * abs(loss_ref)
    worst = 0.0
    for (name, _), g, r, wm, wr in zip(si.unet_weight_shapes(CH), step.dw, grads_ref, step.wm, w_ref):
        gg = _h(g)
        e = oc.rel_err(gg, r)
        worst = max(worst, e)
        ratio = np.sqrt(np.sum(gg * gg) / np.sum(r * r))
        cos = np.sum(gg * r) / np.sqrt(np.sum(gg * gg) * np.sum(r * r))
        print(f"{name}: max error {e:.2e}, norm ratio - 1 = {ratio - 1.0:+.1e}, 1 - cos = {1.0 - cos:.1e}")
        # A handful of pre-activations lie so close to zero that the fp32 and the fp64 sums put them on different
        # LeakyReLU branches; each such voxel changes a few gradient elements by a few 1e-2 of the rms (which voxels
        # depends on the order of the fp32 sums: 1.4e-2 at worst with 16 contracted channels per stage, 3.9e-2 with 8).
        # Length and direction of every gradient are what a wrong scale, a dropped term or a wrong operand would move.
        assert abs(ratio - 1.0) <= 2e-4 and 1.0 - cos <= 1e-6, (name, ratio, cos)
        assert e <= 6e-2, (name, e)
        assert np.allclose(wm.cpu().numpy(), wr, rtol=1e-4, atol=1e-6), name
    print(f"worst weight-gradient error of the fp32 step against the exact oracle step: {worst:.2e}")


def test_fp32_normalised_step_end_to_end_against_the_exact_oracle_step(unet):
    """The paper's block (Section 4.1: convolution -> instance normalisation -> LeakyReLU) in fp32 against the fp64
    oracle step with the same block: loss, length and direction of every weight gradient."""
    N, vol = 2, 32
    x, labels, ws, xd, ld = _inputs(N, vol, CH, 5)
    step = unet.UNetStep(N, vol, CH, ws, xd.float(), ld, swap=False, norm=True, dtype=torch.float32)
    step.run(update=False)
    torch.cuda.synchronize()
    loss_ref, grads_ref, _ = ou.train_step(x.astype(np.float64), labels, ws, CH, 0.0, norm=True)
    assert abs(float(step.loss.item()) - loss_ref) <= 1e-5 * abs(loss_ref)
    for (name, _), g, r in zip(si.unet_weight_shapes(CH), step.dw, grads_ref):
        gg = _h(g)
        ratio = np.sqrt(np.sum(gg * gg) / np.sum(r * r))
        cos = np.sum(gg * r) / np.sqrt(np.sum(gg * gg) * np.sum(r * r))
        print(f"{name}: max error {oc.rel_err(gg, r):.2e}, norm ratio - 1 = {ratio - 1.0:+.1e}, 1 - cos = {1.0 - cos:.1e}")
        # (as in the step without normalisation: a few pre-activations next to zero take the other LeakyReLU branch)
        assert abs(ratio - 1.0) <= 2e-4 and 1.0 - cos <= 5e-6, (name, ratio, cos)


def test_fp32_step_swapped_recomputed_and_hybrid_are_bit_identical(unet):
    from paper_1812_07816_amd import swap as sw
    N, vol = 1, 32
    _, _, ws, xd, ld = _inputs(N, vol, CH, 5)
    xf = xd.float()
    plain = unet.UNetStep(N, vol, CH, ws, xf, ld, swap=False, dtype=torch.float32)
    plain.run(update=False)
    torch.cuda.synchronize()
    ref, ref_loss = plain.dw32.clone(), plain.loss.clone()
    for eviction in (sw.EVICT_SWAP, sw.EVICT_RECOMPUTE, sw.EVICT_HYBRID):
        st = unet.UNetStep(N, vol, CH, ws, xf, ld, swap=True, budget_bytes=None, lookahead=2, policy=sw.POLICY_ALL, eviction=eviction,
                           dtype=torch.float32)
        st.run(update=False)
        torch.cuda.synchronize()
        s = st.engine.stats()
        assert s["n_swapped_out"] + st.n_recomputed > 0
        assert torch.equal(st.dw32, ref) and torch.equal(st.loss, ref_loss)
        st.close()


def test_virtual_concatenation_gives_the_bits_of_the_materialised_one_and_needs_less_memory(unet):
    N, vol = 2, 32
    _, _, ws, xd, ld = _inputs(N, vol, CH, 5)
    out = {}
    for virtual in (False, True):
        st = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True, virtual_cat=virtual)
        st.run(update=False)
        torch.cuda.synchronize()
        out[virtual] = (st.dw32.clone(), st.loss.clone(), st.engine.stats()["unswapped_peak_bytes"], sum(s.bytes for s in st.saved))
        st.close()
    assert torch.equal(out[True][0], out[False][0]) and torch.equal(out[True][1], out[False][1])
    # one tensor of C channels per decoder level is no longer kept
    dropped = sum(N * (vol >> l) ** 3 * CH[l] * 2 for l in range(len(CH) - 1))
    assert out[False][3] - out[True][3] == dropped
    assert out[True][2] < out[False][2]


def test_swapped_step_is_bit_identical(unet):
    from paper_1812_07816_amd import swap as sw
    N, vol = 2, 32
    _, _, ws, xd, ld = _inputs(N, vol, CH, 5)
    plain = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=False)
    plain.run(update=False)
    torch.cuda.synchronize()
    ref = plain.dw32.clone()
    ref_loss = plain.loss.clone()
    probe = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True)
    peak = probe.engine.stats()["unswapped_peak_bytes"]
    probe_fixed = probe._transient(0)     # weights, workspace, labels
    probe.close()
    for policy, budget in ((sw.POLICY_BUDGET, int(peak * 0.8)), (sw.POLICY_ALL, None)):
        st = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True, budget_bytes=budget, lookahead=2, policy=policy)
        st.engine.set_verify(True)
        st.run(update=False)
        torch.cuda.synchronize()
        s = st.engine.stats()
        assert s["n_swapped_out"] > 0 and s["n_swapped_out"] == s["n_swapped_in"], s
        assert torch.equal(st.dw32, ref) and torch.equal(st.loss, ref_loss)
        assert s["n_checksummed"] == s["n_swapped_in"] and s["n_checksum_mismatch"] == 0, s
        # the arena the step really needed, counting blocks a swap-out was still reading, against the plan's share
        print("policy", policy, "arena high water", s["arena_high_water_bytes"], "planned", s["planned_arena_bytes"], "overflows", s["n_arena_overflow"])
        # every saved tensor sat at its planned place: the arena is exactly the plan's static placement
        assert s["n_arena_overflow"] == 0 and s["arena_high_water_bytes"] <= s["static_arena_bytes"], s
        assert st.arena.numel() == s["static_arena_bytes"] + 256
        if st.plan_status == 0 and budget is not None:
            assert s["static_arena_bytes"] + probe_fixed <= budget, s
        st.run(update=False)          # a second step reuses the arena and the host pool
        torch.cuda.synchronize()
        assert torch.equal(st.dw32, ref)
        st.close()


def test_measured_device_footprint_meets_the_budget(unet):
    """The budget is physical: the arena is allocated at the size of the plan's static placement, and fit_budget
    tightens the planner's budget until the peak of the device allocator over a whole step (arena, gradients, weights,
    workspaces, labels, input) is within the budget the step was given."""
    N, vol = 2, 32
    _, _, ws, xd, ld = _inputs(N, vol, CH, 5)
    plain = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=False)
    plain.run(update=False)
    torch.cuda.synchronize()
    ref = plain.dw32.clone()
    del plain
    torch.cuda.empty_cache()
    held = torch.cuda.memory_allocated()            # what the test itself keeps alive (inputs, reference gradients)
    probe = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True)
    free_peak = probe.fit_budget() - held           # footprint of the step without a budget
    fixed = probe._transient(0)                     # weights, workspace, labels: nothing a plan can move
    probe.close()
    del probe
    torch.cuda.empty_cache()
    budget = int(free_peak - 0.15 * (free_peak - fixed))   # (at this size weights and workspaces are five sixths of the footprint)
    st = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True, budget_bytes=budget + held, lookahead=2)
    peak = st.fit_budget()
    assert peak - held <= budget, (peak - held, budget, st.fit_log)
    s = st.engine.stats()
    assert s["n_swapped_out"] > 0 and s["n_arena_overflow"] == 0
    assert torch.equal(st.dw32, ref)
    print(f"unbudgeted {free_peak} B, budget {budget} B, measured {peak - held} B, swapped {s['n_swapped_out']} tensors, arena {s['static_arena_bytes']} B")
    st.close()


def test_recomputed_and_hybrid_steps_are_bit_identical(unet):
    """Section 5: dropped tensors are produced again by their convolution at their first backward use; the kernels
    are deterministic, so the gradients are those of the plain step bit for bit."""
    from paper_1812_07816_amd import swap as sw
    N, vol = 2, 32
    _, _, ws, xd, ld = _inputs(N, vol, CH, 5)
    plain = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=False)
    plain.run(update=False)
    torch.cuda.synchronize()
    ref, ref_loss = plain.dw32.clone(), plain.loss.clone()
    probe = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True)
    peak = probe.engine.stats()["unswapped_peak_bytes"]
    fixed = probe._transient(0)           # weights, workspace, labels: nothing the plan can move
    probe.close()

    def check(st, budget, hybrid):
        for calibrated in (False, True):
            if calibrated:
                st.calibrate()
                # measured op durations with the waits for swap-ins taken off: one per op, none negative
                assert len(st.op_ms) == st.n_ops and min(st.op_ms) >= 0.0
            st.run(update=False)
            torch.cuda.synchronize()
            s = st.engine.stats()
            assert st.n_recomputed == s["n_recompute"], (s, st.n_recomputed)
            # (with measured op times the hybrid swaps what the link can hide and may need no re-computation at all)
            if calibrated and hybrid:
                assert s["n_recompute"] + s["n_planned"] > 0, s
            else:
                assert s["n_recompute"] > 0, s
            if budget is not None and st.plan_status == 0:
                assert s["planned_peak_bytes"] <= budget and s["peak_arena_bytes"] <= s["planned_peak_bytes"] - fixed
                assert s["n_arena_overflow"] == 0 and s["arena_high_water_bytes"] <= s["static_arena_bytes"]
            assert torch.equal(st.dw32, ref) and torch.equal(st.loss, ref_loss)
        return s

    for eviction in (sw.EVICT_RECOMPUTE, sw.EVICT_HYBRID):
        # a budget that takes a part of the movable bytes away; the largest cut this eviction mode can meet
        for cut in (0.5, 0.35, 0.2, 0.1):
            budget = int(peak - cut * (peak - fixed))
            st = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True, budget_bytes=budget, lookahead=2, eviction=eviction)
            if st.plan_status == 0:
                break
            st.close()
        assert st.plan_status == 0, "no cut of the movable bytes is feasible"
        s = check(st, budget, eviction == sw.EVICT_HYBRID)
        print("eviction", eviction, "cut", cut, "recomputed", s["n_recompute"], "swapped", s["n_planned"])
        if eviction == sw.EVICT_RECOMPUTE:
            assert s["n_swapped_out"] == 0
        st.close()
        st = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True, budget_bytes=None, lookahead=2, policy=sw.POLICY_ALL, eviction=eviction)
        s = check(st, None, eviction == sw.EVICT_HYBRID)
        assert (s["n_swapped_out"] == 0) if eviction == sw.EVICT_RECOMPUTE else (s["n_swapped_out"] > 0 and s["n_swapped_out"] == s["n_swapped_in"])
        st.close()


def test_adam_steps_follow_the_oracle_update_on_the_steps_own_gradients(unet):
    N, vol = 1, 16
    ch = CH[:4]
    _, _, ws, xd, ld = _inputs(N, vol, ch, 5)
    lr = 5e-4
    step = unet.UNetStep(N, vol, ch, ws, xd, ld, lr=lr, swap=False, optimizer="adam")
    w = step.w32.cpu().numpy().astype(np.float64)
    m, v = np.zeros_like(w), np.zeros_like(w)
    for k in range(1, 4):
        step.run(update=True)
        torch.cuda.synchronize()
        g = step.dw32.cpu().numpy().astype(np.float64)
        # the C ABI takes the coefficients as floats: the oracle gets the same (float32-rounded) values
        w, m, v = ou.adam_step(w, g, m, v, float(np.float32(lr)), k, float(np.float32(0.9)), float(np.float32(0.999)), float(np.float32(1e-8)))
        assert np.allclose(step.w32.cpu().numpy(), w, rtol=1e-5, atol=1e-7), k
        assert torch.equal(step.w16, step.w32.to(torch.bfloat16))
    assert float(np.max(np.abs(w - step.w32.cpu().numpy()))) < 1e-6


@pytest.mark.parametrize("N,vol,channels,f32", [(2, 32, CH, False), (1, 16, CH[:4], False), (2, 32, CH, True), (1, 16, CH[:4], True)])
def test_every_op_with_instance_normalisation_matches_oracle(unet, N, vol, channels, f32):
    """The network of Section 4.1 proper: convolution -> instance normalisation -> LeakyReLU.  Every op of the GPU
    step against the oracle's definition of it on the tensors the step itself fed it (fp32: at fp32 accuracy; the
    normalisation's one-pass variance from fp32 block sums is the least accurate op)."""
    x, labels, ws, xd, ld = _inputs(N, vol, channels, 5)
    L = len(channels)
    TOL = 2e-4 if f32 else 1e-2
    step = unet.UNetStep(N, vol, channels, ws, xd.float() if f32 else xd, ld, swap=False, norm=True,
                         dtype=torch.float32 if f32 else torch.bfloat16)
    tr = {}
    step.run(update=False, trace=tr)
    torch.cuda.synchronize()
    t = {k: _h(v) for k, v in tr.items()}
    w = {n: np.asarray(a, dtype=np.float64) for (n, _), a in zip(si.unet_weight_shapes(channels), ws)}
    dw = {n: _h(g) for (n, _), g in zip(si.unet_weight_shapes(channels), step.dw)}
    worst = [0.0, ""]

    def close(name, got, ref):
        e = oc.rel_err(got, ref)
        if e > worst[0]:
            worst[:] = [e, name]
        assert e <= TOL, (name, e)

    convs, v, prev, cin = [], vol, "input", 4
    for l in range(L):
        s = 1 if l == 0 else 2
        convs.append((f"enc{l}.conv1", prev, v, cin, channels[l], s)); v //= s
        convs.append((f"enc{l}.conv2", f"enc{l}.conv1", v, channels[l], channels[l], 1))
        prev, cin = f"enc{l}.conv2", channels[l]
    for l in range(L - 2, -1, -1):
        v *= 2
        convs.append((f"dec{l}.conv1", f"dec{l}.cat", v, 2 * channels[l], channels[l], 1))
        convs.append((f"dec{l}.conv2", f"dec{l}.conv1", v, channels[l], channels[l], 1))
    for name, src, vin, ci, co, s in convs:
        g = oc.shape(N, vin, vin, vin, ci, co, 3, s, 1)
        close(name + " conv", t[name + ".z"], oc.fwd(g, t[src + ".a"], w[name]))
        xhat, _, rstd = ou.instnorm(t[name + ".z"])          # of the stored (bf16) convolution output
        close(name + " norm fwd", t[name + ".a"], ou._lrelu(xhat))
        # backward through LeakyReLU and normalisation from the stored activation, then the two gradients
        dz_ref = ou.instnorm_lrelu_bwd(ou.lrelu_inverse(t[name + ".a"]), rstd, t[name + ".dout"])
        close(name + " norm bwd", t[name + ".dz"], dz_ref)
        close(name + " wgrad", dw[name], oc.wgrad(g, t[src + ".a"], t[name + ".dz"]))
        if name == "enc0.conv1":
            continue
        din_ref = oc.dgrad(g, t[name + ".dz"], w[name])
        if name.startswith("enc") and name.endswith("conv1") and name + ".skip_add" in t:
            # (fp32: the data gradient adds the skip connection's second gradient itself)
            l = int(name[3]) - 1
            assert np.array_equal(t[name + ".skip_add"], t[f"dec{l}.cat.dskip"])
            close(name + " dgrad + skip", t[name + ".din"], din_ref + t[name + ".skip_add"])
        elif name.startswith("enc") and name.endswith("conv1"):
            l = int(name[3]) - 1
            close(name + " dgrad", t[name + ".dgrad"], din_ref)
            close(name + " skip add", t[name + ".din"], t[name + ".dgrad"] + t[f"dec{l}.cat.dskip"])
        else:
            close(name + " dgrad", t[name + ".din"], din_ref)
    gh = oc.shape(N, vol, vol, vol, channels[0], 3, 1, 1, 0)
    close("head fwd", t["head.a"], oc.fwd(gh, t["dec0.conv2.a"], w["head"]))
    close("head dgrad", t["head.din"], oc.dgrad(gh, t["head.dout"], w["head"]))
    print(f"worst op error {worst[0]:.2e} ({worst[1]})")


def test_backward_sums_from_the_data_gradient_give_the_step_of_the_separate_reductions(unet):
    """The data gradients that also deliver the sums of the normalisation's backward pass against the step that takes
    them in reduction passes of its own: same sums up to the order of fp32 additions, so the weight gradients agree to
    bf16 rounding noise (not bit for bit: a sum that differs in its last bits rounds a few stored values the other
    way, and the layers below inherit that)."""
    N, vol = 2, 32
    x, labels, ws, xd, ld = _inputs(N, vol, CH, 5)
    a = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=False, norm=True)
    b = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=False, norm=True, fused_bwd_sums=False)
    assert sum(1 for op in a.ops if op.get("through_norm")) >= 5 and sum(1 for op in a.ops if op.get("skip_sums")) == 1
    assert not any(op.get("through_norm") or op.get("skip_sums") for op in b.ops)
    a.run(update=False); b.run(update=False)
    torch.cuda.synchronize()
    assert torch.equal(a.loss, b.loss)
    worst = {}
    for (name, _), ga, gb in zip(si.unet_weight_shapes(CH), a.dw, b.dw):
        ga, gb = _h(ga), _h(gb)
        e = np.max(np.abs(ga - gb)) / np.max(np.abs(gb))
        l2 = np.sqrt(np.sum((ga - gb) ** 2) / np.sum(gb * gb))
        print(f"{name}: max {e:.1e}, l2 {l2:.1e}")
        worst[name] = max(e, l2)
    # The head's gradient is formed before the first such data gradient and sees the same bits.  From there on a
    # stored bf16 value that rounds the other way is a relative step of 2^-8, and every layer further down the
    # backward pass inherits the noise of those above it: the first layer's gradient (formed last) the most.
    assert worst["head"] == 0.0
    assert max(worst.values()) <= 3e-2, worst


def test_normalised_step_end_to_end_and_under_eviction(unet):
    from paper_1812_07816_amd import swap as sw
    N, vol = 2, 32
    x, labels, ws, xd, ld = _inputs(N, vol, CH, 5)
    step = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=False, norm=True)
    step.run(update=False)
    torch.cuda.synchronize()
    loss_ref, grads_ref, _ = ou.train_step(x.astype(np.float64), labels, ws, CH, 0.0, q=ou.bf16, norm=True)
    assert abs(float(step.loss.item()) - loss_ref) <= 2e-3 * abs(loss_ref)
    for (name, _), g, r in zip(si.unet_weight_shapes(CH), step.dw, grads_ref):
        gg = _h(g)
        cos = np.sum(gg * r) / np.sqrt(np.sum(gg * gg) * np.sum(r * r))
        # two bf16 pipelines drift apart layer by layer (see the module docstring), the more the more roundings
        # a layer's gradient has behind it; the first layer's is the last one formed
        assert cos >= 0.9, (name, cos)
    ref, ref_loss = step.dw32.clone(), step.loss.clone()
    # swapped, re-computed and mixed steps repeat the statistics bit for bit as well
    for eviction in (sw.EVICT_SWAP, sw.EVICT_RECOMPUTE, sw.EVICT_HYBRID):
        st = unet.UNetStep(N, vol, CH, ws, xd, ld, swap=True, budget_bytes=None, lookahead=2, policy=sw.POLICY_ALL, eviction=eviction, norm=True)
        st.run(update=False)
        torch.cuda.synchronize()
        s = st.engine.stats()
        assert s["n_swapped_out"] + st.n_recomputed > 0
        assert torch.equal(st.dw32, ref) and torch.equal(st.loss, ref_loss)
        st.close()
