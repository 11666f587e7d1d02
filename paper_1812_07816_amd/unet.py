"""One training step of the 3D U-Net with data swapping (host-side orchestration).

Every arithmetic step is a call into libmi3d.so: the convolutions
(conv3d_fwd / dgrad / wgrad; the 2x2x2 stride-2 transposed convolution is the
data gradient of a 2x2x2 / stride-2 convolution with roles swapped; LeakyReLU
rides in the convolution calls where it can), channel concatenation, sigmoid + soft Dice, SGD or Adam.  Saved feature maps (the
inputs of the convolutions, Section 3.1 of the paper) live in the swap engine's
arena and are moved to pinned host memory and back according to its plan.

Network: L encoder levels of two 3x3x3 convolutions (the first of each level
but the top with stride 2), decoder levels of up-sampling, concatenation
[upsampled, skip] and two 3x3x3 convolutions, a 1x1x1 head; LeakyReLU after
every 3x3x3 convolution, optionally behind an instance normalisation
(norm=True); no bias.

Op timeline for the planner: forward ops in program order, then one backward
op per forward op in reverse order (backward op of forward op f is
n_fwd + (n_fwd - 1 - f)).
"""
import torch

from . import conv3d as mc
from . import glue
from . import swap as sw

SLOPE = 0.01


def _numel(shape):
    n = 1
    for v in shape:
        n *= v
    return n


class _Saved:
    """A tensor produced in the forward pass and needed again in the backward pass."""

    def __init__(self, sid, shape, produce, tag, esize=2):
        self.id, self.shape, self.bytes = sid, tuple(shape), _numel(shape) * esize
        self.produce, self.last_fwd, self.tag = produce, produce, tag
        self.complete = produce    # forward op after which the contents are final (a swap-out may start)
        self.bwd_ops = []          # backward ops that read it
        self.ptr, self.view = None, None


class UNetStep:
    def __init__(self, N, vol, channels, weights, x, labels, lr=1e-2, in_ch=4, classes=3, swap=True,
                 budget_bytes=None, lookahead=2, policy=sw.POLICY_BUDGET, n_tensors=-1, exclude_tags=0,
                 eviction=sw.EVICT_SWAP, optimizer="sgd", norm=False, virtual_cat=True, fused_stats=True, fused_bwd_sums=True, dtype=torch.bfloat16):
        """weights: list of float32 CPU tensors/arrays (bf16-exact start values) in the order enc convs,
        (dec up, conv1, conv2) from the deepest decoder level up, head; x: CUDA [N,vol,vol,vol,in_ch] of `dtype`;
        labels: uint8 CUDA [N,vol,vol,vol,classes].  dtype: torch.bfloat16 (bf16 activations and working weights, fp32
        master weights) or torch.float32 (everything fp32: the convolutions run on the fp32 matrix cores and read the
        master weights themselves)."""
        assert dtype in (torch.bfloat16, torch.float32) and x.dtype == dtype
        assert virtual_cat or dtype == torch.bfloat16, "the materialised concatenation is bf16 only"
        self.dtype, self.esize = dtype, (2 if dtype == torch.bfloat16 else 4)
        self.N, self.vol, self.ch, self.L = N, vol, list(channels), len(channels)
        self.lr, self.classes, self.swap_on = lr, classes, swap
        self.x_in, self.labels = x, labels
        L, ch = self.L, self.ch
        # ---- parameters: flat fp32 master / gradient buffers and a flat bf16 working copy, 64-element aligned views
        offs, total = [], 0
        for w in weights:
            offs.append(total)
            total += (_numel(w.shape) + 63) // 64 * 64
        assert optimizer in ("sgd", "adam")
        self._trace = None
        self.norm = bool(norm)     # instance normalisation between every 3x3x3 convolution and its LeakyReLU (Section 4.1)
        self.optimizer, self.opt_step = optimizer, 0
        self.w32 = torch.zeros(total, dtype=torch.float32, device="cuda")
        self.dw32 = torch.zeros(total, dtype=torch.float32, device="cuda")
        if optimizer == "adam":    # first and second moments (Section 4.1 trains with Adam)
            self.m32 = torch.zeros(total, dtype=torch.float32, device="cuda")
            self.v32 = torch.zeros(total, dtype=torch.float32, device="cuda")
        self.w16 = torch.zeros(total, dtype=torch.bfloat16, device="cuda") if dtype == torch.bfloat16 else None
        self.w, self.dw, self.wm = [], [], []
        for w, o in zip(weights, offs):
            n = _numel(w.shape)
            wt = torch.as_tensor(w, dtype=torch.float32).reshape(-1).cuda()
            self.w32[o:o + n].copy_(wt)
            if self.w16 is not None:
                self.w16[o:o + n].copy_(wt.to(torch.bfloat16))
            self.w.append((self.w32 if self.w16 is None else self.w16)[o:o + n].view(tuple(w.shape)))
            self.dw.append(self.dw32[o:o + n].view(tuple(w.shape)))
            self.wm.append(self.w32[o:o + n].view(tuple(w.shape)))
        # ---- forward program
        self.ops, self.saved = [], []
        self.flops = 0.0

        def new_saved(shape, tag):
            s = _Saved(len(self.saved), shape, len(self.ops), tag, self.esize)
            self.saved.append(s)
            return s

        def conv_op(name, src, vol_in, cin, cout, s, widx, tag, first=False, src2=None):
            d = mc.make_desc(N, vol_in, vol_in, vol_in, cin, cout, 3, s, 1, dtype)
            vo = vol_in // s
            out = new_saved((N, vo, vo, vo, cout), tag)
            src.last_fwd = len(self.ops)
            if src2 is not None:     # the input is [src | src2] along the channels, never materialised
                src2.last_fwd = len(self.ops)
            self.ops.append(dict(kind="conv", name=name, desc=d, src=src, src2=src2, out=out, w=widx, first=first))
            fl = 2.0 * N * vo ** 3 * 27 * cin * cout
            self.flops += fl * (2 if first else 3)
            return out, vo

        xs = _Saved(0, (N, vol, vol, vol, in_ch), 0, sw.TAG_INPUT, self.esize)
        self.saved.append(xs)
        self.ops.append(dict(kind="input", name="input", out=xs))
        a, v, wi = xs, vol, 0
        skips = []
        for l in range(L):
            a, v = conv_op(f"enc{l}.conv1", a, v, in_ch if l == 0 else ch[l - 1], ch[l], 1 if l == 0 else 2, wi, sw.TAG_ENCODER, first=(l == 0)); wi += 1
            a, v = conv_op(f"enc{l}.conv2", a, v, ch[l], ch[l], 1, wi, sw.TAG_ENCODER); wi += 1
            if l < L - 1:
                skips.append(a)
        for l in range(L - 2, -1, -1):
            v *= 2
            d = mc.make_desc(N, v, v, v, ch[l], ch[l + 1], 2, 2, 0, dtype)  # the convolution whose dgrad is the up-sampling
            a.last_fwd = len(self.ops)
            # the up-sampling writes straight into its half of the concatenated tensor, and its backward passes read
            # their half of that tensor's gradient in place, where the library has the kernels for it
            in_place = all(mc.kernel_name(d, p) == "mfma_k2s2_panel_gemm" for p in range(3))
            # Virtual concatenation: where the library's kernels take the two halves as separate tensors, the
            # concatenated tensor and its gradient never exist; the up-sampled map is a saved tensor of its own and the
            # skip tensor is read a second time by the decoder (forward and weight gradient).
            d1 = mc.make_desc(N, v, v, v, 2 * ch[l], ch[l], 3, 1, 1, dtype)
            virtual = virtual_cat and all(mc.pair_supported(d1, p) for p in range(3))
            in_place = in_place and not virtual
            u = new_saved((N, v, v, v, ch[l]), sw.TAG_DECODER) if virtual else None
            self.ops.append(dict(kind="up", name=f"dec{l}.up", desc=d, src=a, w=wi, shape=(N, v, v, v, ch[l]), in_place=in_place,
                                 virtual=virtual, out=u)); wi += 1
            self.flops += 3 * 2.0 * N * (v // 2) ** 3 * 8 * ch[l] * ch[l + 1]
            if virtual:
                self.ops.append(dict(kind="cat", name=f"dec{l}.cat", skip=skips[l], up=u, c=ch[l], virtual=True))
                a, _ = conv_op(f"dec{l}.conv1", u, v, 2 * ch[l], ch[l], 1, wi, sw.TAG_DECODER, src2=skips[l]); wi += 1
                a, _ = conv_op(f"dec{l}.conv2", a, v, ch[l], ch[l], 1, wi, sw.TAG_DECODER); wi += 1
                continue
            cat = new_saved((N, v, v, v, 2 * ch[l]), sw.TAG_DECODER)
            if in_place:
                cat.produce = len(self.ops) - 1      # allocated and half filled by the up-sampling, completed by the next op
            skips[l].last_fwd = len(self.ops)
            self.ops.append(dict(kind="cat", name=f"dec{l}.cat", skip=skips[l], out=cat, c=ch[l], virtual=False))
            a, _ = conv_op(f"dec{l}.conv1", cat, v, 2 * ch[l], ch[l], 1, wi, sw.TAG_DECODER); wi += 1
            a, _ = conv_op(f"dec{l}.conv2", a, v, ch[l], ch[l], 1, wi, sw.TAG_DECODER); wi += 1
        d = mc.make_desc(N, v, v, v, ch[0], classes, 1, 1, 0, dtype)
        logits = new_saved((N, v, v, v, classes), sw.TAG_HEAD)
        a.last_fwd = len(self.ops)
        self.ops.append(dict(kind="head", name="head", desc=d, src=a, out=logits, w=wi))
        self.flops += 3 * 2.0 * N * v ** 3 * ch[0] * classes
        logits.last_fwd = len(self.ops)
        self.ops.append(dict(kind="loss", name="loss", src=logits))
        self.n_fwd = len(self.ops)
        self.n_ops = 2 * self.n_fwd
        # a convolution whose input is the activation of the convolution right before it, read by nobody else
        skip_ids = {s.id for s in skips}
        for f, op in enumerate(self.ops):
            if op["kind"] == "head":
                # the head reads the last normalised convolution's activation (nobody else does): its data gradient
                # streams that tensor's gradient once, so the sums ride along (data gradient + backward pass 1.19 -> 1.01 ms at 192^3, N = 2)
                op["through_norm"] = bool(self.norm and fused_bwd_sums and self.ops[f - 1]["kind"] == "conv"
                                          and self.ops[f - 1]["out"] is op["src"] and mc.dgrad_insums_supported(op["desc"]))
            if op["kind"] == "conv":
                prev = self.ops[f - 1]
                alone = prev["kind"] == "conv" and prev["out"] is op["src"] and op["src"].id not in skip_ids
                op["through_act"] = not self.norm and alone
                # with the normalisation in between, the data gradient can still take the two sums of that
                # normalisation's backward pass on its way out
                # (measured at N = 2, data gradient + backward pass: 1.79 -> 1.49 ms at 192^3 with 32 channels, where the
                # tensors come from memory; 0.575 -> 0.555 at 96^3 with 64, 0.268 -> 0.260 at 48^3 with 128: small gains
                # where the reduction it saves runs from the caches)
                op["through_norm"] = bool(self.norm and alone and fused_bwd_sums and mc.dgrad_insums_supported(op["desc"]))
                # the stride-2 data gradient that adds the skip connection's second gradient (virtual concatenation):
                # the gradient of the skip tensor is complete there, so the sums of its producer's normalisation can
                # be taken there as well (the producer is the convolution right before this one)
                op["skip_sums"] = bool(self.norm and fused_bwd_sums and virtual_cat and op["src"].id in skip_ids
                                       and prev["kind"] == "conv" and prev["out"] is op["src"]
                                       and mc.dgrad_insums_supported(op["desc"], with_add=True))
        # backward readers: conv f reads its input (weight gradient; LeakyReLU derivative of the layer below where the
        # data gradient applies it) and, unless the layer above has applied it already, its output (LeakyReLU
        # derivative); up and head read their input (weight gradient); the loss reads the logits
        for f, op in enumerate(self.ops):
            b = self.bwd_op(f)
            if op["kind"] == "conv":
                op["src"].bwd_ops.append(b)
                if op["src2"] is not None:
                    op["src2"].bwd_ops.append(b)
                nxt = self.ops[f + 1]
                if not (nxt["kind"] == "conv" and nxt["through_act"]):
                    op["out"].bwd_ops.append(b)
            elif op["kind"] in ("up", "head"):
                op["src"].bwd_ops.append(b)
            elif op["kind"] == "loss":
                op["src"].bwd_ops.append(b)
        # the backward op of the encoder convolution that reads a skip tensor (conv1 of the next level down) is the
        # one that consumes the skip half of the concatenated tensor's gradient
        for op in self.ops:
            if op["kind"] == "cat":
                op["enc_reader"] = next(self.bwd_op(f) for f, o in enumerate(self.ops)
                                        if o["kind"] == "conv" and o["src"] is op["skip"])
        # ---- workspaces and small buffers
        ws_bytes = 256
        for op in self.ops:
            if "desc" in op:
                ws_bytes = max(ws_bytes, max(mc.workspace_bytes(op["desc"], p) for p in range(3)) + 256)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        self.dice_ws = glue.dice_workspace(classes)
        if self.norm:     # statistics of every normalised convolution output (kept for the backward pass) and the reduction scratch
            self.in_ws = glue.instnorm_workspace(N, max(ch))
            for op in self.ops:
                if op["kind"] == "conv":
                    op["stats"] = torch.zeros((N, op["out"].shape[-1], 2), dtype=torch.float32, device="cuda")
                    op["bwd_sums"] = torch.zeros((N, op["out"].shape[-1], 2), dtype=torch.float32, device="cuda")
                    op["fused_stats"] = fused_stats and mc.fwd_stats_supported(op["desc"])
        self.sums = torch.zeros(3 * classes, dtype=torch.float32, device="cuda")
        self.loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        # ---- swap engine
        self.engine = None
        if swap:
            budget = (1 << 62) if budget_bytes is None else int(budget_bytes)
            sizes = [s.bytes for s in self.saved]
            pool = sum((b + 4095) // 4096 * 4096 for b in sizes) + 4096
            # the arena is sized by the plan's static placement of the saved tensors (see _read_plan): what the step
            # holds on the device is then fixed by the plan, not by how an allocator happened to fill a large pool
            self.arena, self.budget = None, budget
            self.engine = e = sw.SwapEngine(budget_bytes=budget, host_pool_bytes=pool, arena=None, lookahead=lookahead,
                                            policy=policy, n_tensors=n_tensors, exclude_tags=exclude_tags)
            e.set_timeline(self.n_fwd, self.n_ops)
            e.set_eviction(eviction)
            for s in self.saved:
                e.register(s.id, s.bytes, s.produce, s.last_fwd, min(s.bwd_ops), max(s.bwd_ops), s.tag)
            # outputs of convolutions can be produced again from their input; cost until measured: the forward
            # pass at 800 TFLOP/s or 4 TB/s, whichever is slower
            for op in self.ops:
                if op["kind"] in ("conv", "head"):
                    d = op["desc"]
                    fl = 2.0 * _numel(op["out"].shape) * d.kD * d.kH * d.kW * d.Cin
                    ms = max(fl / 8e14, (op["src"].bytes + op["out"].bytes) / 4e12) * 1e3
                    if op.get("src2") is not None:
                        e.set_recompute(op["out"].id, ms, op["src"].id, op["src2"].id)
                    else:
                        e.set_recompute(op["out"].id, ms, op["src"].id)
            for op in range(self.n_ops):
                e.set_transient(op, self._transient(op))
            self._read_plan(e.plan(allow_over_budget=True))
        else:
            self.planned = [False] * len(self.saved)
            self.recomputed = [False] * len(self.saved)
            self.prefetch = [-1] * len(self.saved)
            self.plan_status = 0
        self.producer = {op["out"].id: op for op in self.ops if op["kind"] in ("conv", "head")}

    def _read_plan(self, status):
        e = self.engine
        self.plan_status = status
        self.planned = [e.is_planned(s.id) for s in self.saved]
        self.recomputed = [e.is_recomputed(s.id) for s in self.saved]
        self.prefetch = [e.prefetch_op(s.id) for s in self.saved]
        need = e.static_arena_bytes() + 256
        if self.arena is None or self.arena.numel() != need:
            e.set_arena(None)
            self.arena = None
            torch.cuda.empty_cache()
            self.arena = torch.empty(need, dtype=torch.uint8, device="cuda")
            e.set_arena(self.arena)

    def bwd_op(self, f):
        return self.n_fwd + (self.n_fwd - 1 - f)

    def _transient(self, op):
        """Device bytes an op holds besides saved tensors: parameters, workspace, labels, and the gradient tensors
        alive during it (the gradient pair of the layer, plus the skip gradients waiting for the encoder)."""
        fixed = self.w32.numel() * ((16 if self.optimizer == "adam" else 8) + (2 if self.w16 is not None else 0)) + self.ws.numel() + self.labels.numel()
        if self.norm:
            fixed += self.in_ws.numel()
        if op < self.n_fwd:
            o = self.ops[op]
            return fixed + (_numel(o["shape"]) * self.esize if o["kind"] == "up" and not o["in_place"] and not o["virtual"] else 0)
        f = self.n_fwd - 1 - (op - self.n_fwd)
        o = self.ops[f]
        live = 0
        if o.get("out") is not None:
            live += o["out"].bytes
        if o.get("src") is not None:
            live += o["src"].bytes
        if o.get("src2") is not None:
            live += o["src2"].bytes
        # gradients of concatenated tensors (their skip halves) of decoder levels already walked back and not yet
        # consumed by the encoder
        for g, oo in enumerate(self.ops):
            if oo["kind"] == "cat" and g >= f:
                if oo["enc_reader"] >= op:       # (virtual concatenation: only the skip half of the gradient exists)
                    live += oo["skip"].bytes if oo["virtual"] else oo["out"].bytes
        return fixed + live

    # ---- storage of saved tensors
    def _view(self, ptr, shape):
        off = ptr - self.arena.data_ptr()
        return self.arena[off:off + _numel(shape) * self.esize].view(self.dtype).view(shape)

    def _timed_wait(self, call):
        """Runs an engine call that may make the compute stream wait for a swap-in; while a calibration records,
        brackets it with events so that the wait can be taken off the op's measured duration."""
        rec = getattr(self, "_wait_events", None)
        if rec is None:
            return call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        r = call()
        e1.record()
        rec.append((self._cur_op, e0, e1))
        return r

    def _produce(self, s):
        if self.engine is None:
            s.view = torch.empty(s.shape, dtype=self.dtype, device="cuda")
        else:
            s.ptr = self.engine.alloc_tensor(s.id)
            s.view = self._view(s.ptr, s.shape)
        return s.view

    def _after_fwd_op(self, f):
        """Swap-outs of tensors produced by op f, releases of tensors whose last forward reader was op f."""
        if self.engine is None:
            return
        for s in self.saved:
            if self.recomputed[s.id] and s.last_fwd == f:      # dropped; produced again at its first backward use
                self.engine.free(s.ptr)
                s.ptr, s.view = None, None
            if not self.planned[s.id]:
                continue
            if s.complete == f:
                self.engine.swap_out(s.id, s.ptr)
            if s.last_fwd == f:
                self.engine.release(s.id)
                s.ptr, s.view = None, None

    def _before_bwd_op(self, op):
        if self.engine is None:
            return
        # (swap-ins that fall on the same op go out in the order of their first use: they share one copy stream, and
        # under a link-bound plan most of them fall on the first backward op)
        for s in sorted(self.saved, key=lambda t: min(t.bwd_ops)):
            if self.planned[s.id] and self.prefetch[s.id] == op:
                s.ptr = self.engine.alloc_tensor(s.id)
                self.engine.swap_in(s.id, s.ptr)
                s.view = self._view(s.ptr, s.shape)

    def _need(self, s):
        if self.engine is not None and self.planned[s.id] and not getattr(s, "_waited", False):
            self._timed_wait(lambda: self.engine.wait_in(s.id))
            s._waited = True
        if s.view is None and self.recomputed[s.id]:
            op = self.producer[s.id]
            self._need(op["src"])
            if op.get("src2") is not None:
                self._need(op["src2"])
            self._forward_conv(op)
            self.n_recomputed += 1
        return s.view

    def _forward_conv(self, op):
        out = self._produce(op["out"])
        d, w = op["desc"], self.w[op["w"]]
        x, x_hi = op["src"].view, (op["src2"].view if op.get("src2") is not None else None)
        if op["kind"] == "conv" and self.norm:
            # convolution -> instance normalisation -> LeakyReLU; the statistics come out of the convolution kernel
            # where it can produce them, else from a pass of their own
            if op["fused_stats"]:
                mc.conv3d_fwd_stats(d, x, w, op["stats"], glue.IN_EPS, out, self.ws, x_hi=x_hi)
            else:
                if x_hi is not None:
                    mc.conv3d_fwd_pair(d, x, x_hi, w, 1.0, out, self.ws)
                else:
                    mc.conv3d_fwd(d, x, w, out, self.ws)
                glue.instnorm_stats(out, op["stats"], self.in_ws)
            if self._trace is not None:
                self._trace[op["name"] + ".z"] = out.clone()
                self._trace[op["name"] + ".stats"] = op["stats"].clone()
            glue.instnorm_lrelu_fwd(out, op["stats"], SLOPE)
        elif op["kind"] == "conv" and x_hi is not None:
            mc.conv3d_fwd_pair(d, x, x_hi, w, SLOPE, out, self.ws)
        elif op["kind"] == "conv":
            mc.conv3d_fwd_lrelu(d, x, w, SLOPE, out, self.ws)
        else:
            mc.conv3d_fwd(d, x, w, out, self.ws)
        return out

    def _after_bwd_op(self, op):
        for s in self.saved:
            if max(s.bwd_ops) == op:
                if self.engine is not None:
                    if self.planned[s.id]:
                        self.engine.done(s.id)
                    self.engine.free(s.ptr)
                s.ptr, s.view, s._waited = None, None, False

    # ---- the step
    def run(self, update=True, trace=None, timeline=None):
        """trace: optional dict that receives copies of intermediate tensors (tests); the step then takes the skip
        gradient in a pass of its own, so that the data gradient before it can be recorded, unless the dict has an
        attribute keep_fused = True (then `<conv>.skip_add` is recorded instead).  timeline: optional list that
        receives (op name, "fwd" | "bwd", event recorded on the compute stream after the op) for a per-op time line."""
        e = self.engine

        def mark(name, phase):
            if timeline is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record()
                timeline.append((name, phase, ev))

        mark("start", "fwd")
        self._trace = trace
        self.n_recomputed = 0
        if e is not None:
            e.reset_step()
        bf = self.dtype      # element type of activations and gradients
        # forward
        for f, op in enumerate(self.ops):
            k = op["kind"]
            self._cur_op = f
            if k == "input":
                self._produce(op["out"]).copy_(self.x_in)
                if trace is not None:
                    trace["input.a"] = op["out"].view.clone()
            elif k == "conv":
                out = self._forward_conv(op)
                if trace is not None:
                    trace[op["name"] + ".a"] = out.clone()
            elif k == "up":
                if op["virtual"]:
                    u = self._produce(op["out"])
                    mc.conv3d_dgrad(op["desc"], op["src"].view, self.w[op["w"]], u, self.ws)
                    if trace is not None:
                        trace[op["name"] + ".a"] = u.clone()
                elif op["in_place"]:
                    cat = self._produce(self.ops[f + 1]["out"])
                    mc.conv3d_dgrad_view(op["desc"], op["src"].view, self.w[op["w"]], cat, 0, self.ws)
                    if trace is not None:
                        trace[op["name"] + ".a"] = cat[..., :op["shape"][-1]].clone()
                else:
                    op["u"] = torch.empty(op["shape"], dtype=bf, device="cuda")
                    mc.conv3d_dgrad(op["desc"], op["src"].view, self.w[op["w"]], op["u"], self.ws)
                    if trace is not None:
                        trace[op["name"] + ".a"] = op["u"].clone()
            elif k == "cat":
                up = self.ops[f - 1]
                if op["virtual"]:
                    if trace is not None:
                        trace[op["name"] + ".a"] = torch.cat([op["up"].view, op["skip"].view], dim=-1)
                elif up["in_place"]:
                    glue.place_channels(op["skip"].view, op["out"].view, op["c"])
                else:
                    glue.concat_channels(up["u"], op["skip"].view, self._produce(op["out"]))
                    up["u"] = None
                if trace is not None and not op["virtual"]:
                    trace[op["name"] + ".a"] = op["out"].view.clone()
            elif k == "head":
                self._forward_conv(op)
                if trace is not None:
                    trace["head.a"] = op["out"].view.clone()
            elif k == "loss":
                glue.dice_loss(op["src"].view, self.labels, self.dice_ws, self.sums, self.loss)
            self._after_fwd_op(f)
            mark(op["name"], "fwd")
        # backward
        da = None              # gradient with respect to the output of the op being walked back
        premasked = False      # da already carries the LeakyReLU derivative of the op being walked back
        have_sums = False      # the sums of the normalisation's backward pass came with da (op["bwd_sums"])
        dskip = {}
        d_pair = None          # skip half of the gradient of a virtual concatenation, between its convolution and its cat op
        for f in range(self.n_fwd - 1, -1, -1):
            op, b = self.ops[f], self.bwd_op(f)
            self._cur_op = b
            self._before_bwd_op(b)
            k = op["kind"]
            if trace is not None and da is not None:
                trace[op["name"] + ".dout"] = da[..., :op["shape"][-1]].clone() if k == "up" else da.clone()
            if k == "loss":
                lg = self._need(op["src"])
                da = torch.empty(op["src"].shape, dtype=bf, device="cuda")
                glue.dice_grad(lg, self.labels, self.sums, da)
            elif k == "head":
                a = self._need(op["src"])
                mc.conv3d_wgrad(op["desc"], a, da, self.dw[op["w"]], self.ws)
                nxt = torch.empty(op["src"].shape, dtype=bf, device="cuda")
                if self.norm and op["through_norm"]:
                    # the data gradient also adds up what the backward pass of the normalisation below needs
                    mc.conv3d_dgrad_insums(op["desc"], da, self.w[op["w"]], a, SLOPE, self.ops[f - 1]["bwd_sums"], nxt, self.ws)
                    have_sums = True
                elif self.norm:
                    mc.conv3d_dgrad(op["desc"], da, self.w[op["w"]], nxt, self.ws)
                else:
                    # its input is the last convolution's activation: the data gradient applies that derivative as well
                    mc.conv3d_dgrad_lrelu(op["desc"], da, self.w[op["w"]], a, SLOPE, nxt, self.ws)
                    premasked = True
                da = nxt
            elif k == "conv":
                if self.norm and have_sums:
                    glue.instnorm_lrelu_bwd_sums(da, self._need(op["out"]), op["stats"], op["bwd_sums"], SLOPE)
                elif self.norm:    # through the LeakyReLU and the normalisation, in place
                    glue.instnorm_lrelu_bwd(da, self._need(op["out"]), op["stats"], self.in_ws, SLOPE)
                elif not premasked:
                    glue.leaky_relu_bwd(da, self._need(op["out"]), SLOPE)
                premasked = False
                have_sums = False
                if trace is not None:
                    trace[op["name"] + ".dz"] = da.clone()
                din_trace = None
                if op["src2"] is not None:
                    mc.conv3d_wgrad_pair(op["desc"], self._need(op["src"]), self._need(op["src2"]), da, self.dw[op["w"]], self.ws)
                else:
                    mc.conv3d_wgrad(op["desc"], self._need(op["src"]), da, self.dw[op["w"]], self.ws)
                if op["first"]:
                    da = None      # the network input needs no gradient
                elif op["src2"] is not None:
                    # the two halves of the gradient go where they are needed: the up-sampling layer's and the skip's
                    d_lo = torch.empty(op["src"].shape, dtype=bf, device="cuda")
                    d_hi = torch.empty(op["src2"].shape, dtype=bf, device="cuda")
                    mc.conv3d_dgrad_pair(op["desc"], da, self.w[op["w"]], d_lo, d_hi, self.ws)
                    da, d_pair = d_lo, d_hi
                    if trace is not None:
                        din_trace = torch.cat([d_lo, d_hi], dim=-1)
                else:
                    nxt = torch.empty(op["src"].shape, dtype=bf, device="cuda")
                    if op["through_act"]:
                        # the input is the previous convolution's activation and nothing else feeds its gradient:
                        # the data gradient applies that LeakyReLU's derivative as well
                        mc.conv3d_dgrad_lrelu(op["desc"], da, self.w[op["w"]], self._need(op["src"]), SLOPE, nxt, self.ws)
                        premasked = True
                    elif op["through_norm"]:
                        # the same situation with a normalisation in between: the data gradient also adds up what
                        # that normalisation's backward pass needs
                        mc.conv3d_dgrad_insums(op["desc"], da, self.w[op["w"]], self._need(op["src"]), SLOPE,
                                               self.ops[f - 1]["bwd_sums"], nxt, self.ws)
                        have_sums = True
                    elif op["src"].id in dskip and dskip[op["src"].id][1] == 0 and (trace is None or getattr(trace, "keep_fused", False) or self.dtype == torch.float32):
                        # the input is also a skip connection whose second gradient is a tensor of its own: the
                        # data gradient adds it and applies the derivative of the producing layer in the same call
                        # (with normalisation the derivative is not a factor: the call only adds, slope 1)
                        d_skip, _ = dskip.pop(op["src"].id)
                        if trace is not None:
                            trace[op["name"] + ".skip_add"] = d_skip.clone()
                        if op["skip_sums"]:
                            # ... and the sums of the backward pass of the normalisation that produced the skip tensor
                            mc.conv3d_dgrad_insums(op["desc"], da, self.w[op["w"]], self._need(op["src"]), SLOPE,
                                                   self.ops[f - 1]["bwd_sums"], nxt, self.ws, add=d_skip)
                            have_sums = True
                        else:
                            mc.conv3d_dgrad_skip(op["desc"], da, self.w[op["w"]], d_skip, self._need(op["src"]),
                                                 1.0 if self.norm else SLOPE, nxt, self.ws)
                        premasked = not self.norm
                    else:
                        mc.conv3d_dgrad(op["desc"], da, self.w[op["w"]], nxt, self.ws)
                    da = nxt
                    if op["src"].id in dskip:
                        # the input is also a skip connection: its second gradient is the skip half of the gradient of
                        # the concatenated tensor; one pass adds it and applies the derivative of the producing layer
                        if trace is not None:
                            trace[op["name"] + ".dgrad"] = da.clone()
                        dcat, c_off = dskip.pop(op["src"].id)
                        # (with normalisation the derivative is not a factor: the pass only adds, slope 1)
                        glue.skip_grad(da, dcat, c_off, self._need(op["src"]), 1.0 if self.norm else SLOPE)
                        premasked = not self.norm
            elif k == "cat" and op["virtual"]:
                dskip[op["skip"].id] = (d_pair, 0)  # da is the up-sampling layer's half already
                if trace is not None:
                    trace[op["name"] + ".dout"] = torch.cat([da, d_pair], dim=-1)
                    trace[op["name"] + ".dskip"] = d_pair.clone()
                d_pair = None
            elif k == "cat":
                c = op["c"]
                dskip[op["skip"].id] = (da, c)      # the skip half stays where it is until the encoder reads it
                if trace is not None:
                    trace[op["name"] + ".dskip"] = da[..., c:].clone()
                if not self.ops[f - 1]["in_place"]:  # otherwise the up-sampling layer reads its half in place
                    d_up = torch.empty(op["out"].shape[:-1] + (c,), dtype=bf, device="cuda")
                    glue.slice_channels(da, 0, d_up)
                    da = d_up
            elif k == "up":
                a = self._need(op["src"])
                # roles: x := gradient of the up-sampled map, dy := the small input
                nxt = torch.empty(op["src"].shape, dtype=bf, device="cuda")
                if op["in_place"]:   # da is the gradient of the concatenated tensor; the first half is this layer's
                    mc.conv3d_wgrad_view(op["desc"], da, 0, a, self.dw[op["w"]], self.ws)
                    mc.conv3d_fwd_view(op["desc"], da, 0, self.w[op["w"]], nxt, self.ws)
                else:
                    mc.conv3d_wgrad(op["desc"], da, a, self.dw[op["w"]], self.ws)
                    mc.conv3d_fwd(op["desc"], da, self.w[op["w"]], nxt, self.ws)
                da = nxt
            if trace is not None and da is not None:
                if k == "conv" and din_trace is not None:
                    trace[op["name"] + ".din"] = din_trace
                else:
                    trace[op["name"] + ".din"] = da[..., :op["c"]].clone() if k == "cat" else da.clone()
            self._after_bwd_op(b)
            mark(op["name"], "bwd")
        if update:
            self.opt_step += 1
            if self.optimizer == "adam":
                glue.adam_update(self.w32, self.dw32, self.m32, self.v32, self.w16, self.lr, self.opt_step)
            else:
                glue.sgd_update(self.w32, self.dw32, self.w16, self.lr)

    def calibrate(self, link_gbs=55.0, passes=1):
        """Runs one step with per-op events, hands the measured op durations and the host-link rate to the
        planner and plans again: the swap-ins are then scheduled by time instead of by op count.  What the compute
        stream spent waiting for swap-ins under the plan it was measured with (issued a fixed number of ops ahead) is
        taken off the backward ops' durations: left in, the time line looks longer than it will be and the timed
        swap-ins come late (fp32, 192^3, 16 GB: a 28 ms wait for a level-0 tensor, 13 % of the step).  The forward
        ops keep their waits for places in the arena that are still being copied out: the placement model counts on
        them (taken off as well, the link-bound bf16 plans got 12 % slower)."""
        if self.engine is None:
            return
        self.link_gbs = link_gbs
        for _ in range(max(1, int(passes))):
            self._calibrate_once(link_gbs)

    def _calibrate_once(self, link_gbs):
        self.run(update=False)
        tl = []
        self._wait_events = []
        try:
            self.run(update=False, timeline=tl)
        finally:
            waits, self._wait_events = self._wait_events, None
        torch.cuda.synchronize()
        t = [tl[0][2].elapsed_time(ev) for _, _, ev in tl]
        ms = [max(t[i + 1] - t[i], 0.0) for i in range(len(t) - 1)]     # forward ops, then backward ops in timeline order
        assert len(ms) == self.n_ops
        for op_index, e0, e1 in waits:
            ms[op_index] = max(ms[op_index] - e0.elapsed_time(e1), 0.0)
        e = self.engine
        # a re-computation costs what the forward op took; the backward ops that ran one under the current plan are
        # charged without it (the planner adds the cost of the re-computations it chooses itself)
        for s in self.saved:
            if self.recomputed[s.id]:
                b = e.first_use_op(s.id)
                ms[b] = max(ms[b] - ms[s.produce], 0.0)
        e.set_op_times(ms, link_gbs)
        for f, op in enumerate(self.ops):
            if op["kind"] in ("conv", "head"):
                if op.get("src2") is not None:
                    e.set_recompute(op["out"].id, ms[f], op["src"].id, op["src2"].id)
                else:
                    e.set_recompute(op["out"].id, ms[f], op["src"].id)
        self._read_plan(e.plan(allow_over_budget=True))
        self.op_ms = ms

    def fit_budget(self, rounds=6):
        """Makes the step's measured device footprint meet its budget: runs a step, reads the peak of the torch
        allocator (arena, gradients, weights, workspaces, labels: every device byte this process holds) and, where
        that exceeds the budget, takes the excess off the planner's budget and plans again.  Returns the measured
        peak of the last step (bytes)."""
        if self.engine is None:
            return None
        internal = self.budget
        peak = None
        self.fit_log = []     # per round: planner budget, plan status, tensors swapped, re-computed, measured peak
        for r in range(rounds + 4):
            torch.cuda.synchronize()
            torch.cuda.reset_peak_memory_stats()
            self.run(update=False)
            torch.cuda.synchronize()
            peak = torch.cuda.max_memory_allocated()
            self.fit_log.append((internal, self.plan_status, sum(self.planned), sum(self.recomputed), peak))
            if peak <= self.budget or self.budget >= (1 << 60):
                break
            # the planner's model has to come down by what the measurement exceeds the budget (the model knows nothing
            # of what else the process holds, so the correction is relative to the model's own peak)
            modelled = self.engine.stats()["planned_peak_bytes"]
            internal = min(internal, modelled) - (peak - self.budget) - (4 << 20)
            if internal <= 0:
                break
            self.engine.set_budget(internal)
            self._read_plan(self.engine.plan(allow_over_budget=True))
            # op durations under the new plan (other tensors wait now); the last rounds keep the op durations they
            # have, so that the plan only moves with the budget (a re-measured time line can move a swap-in by an op
            # and the footprint by some MB, which kept one run from settling within 0.1 % of its budget)
            if getattr(self, "link_gbs", None) and r < rounds:
                self._calibrate_once(self.link_gbs)
        self.measured_peak_bytes = peak
        return peak

    def close(self):
        if self.engine is not None:
            self.engine.close()
            self.engine = None
