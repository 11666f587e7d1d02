"""One training step of a chain of Conv3D layers with data swapping.

Host-side orchestration only: every arithmetic step is a call into
libmi3d.so (conv3d_fwd / dgrad / wgrad) and every copy a call into its swap
engine.  The chain is the first level of the 3D U-Net at full resolution
(two 3x3x3 convolutions and the stride-2 convolution that leaves the level);
saved inputs of the layers are the feature maps of Section 3.1 of the paper:
produced in the forward pass, needed again by the weight gradient of the same
layer in the backward pass, and moved to pinned host memory in between when
the device budget asks for it.

Op timeline (planner indices): forward op i = layer i; backward, for
i = L-1 .. 0: op L + 2 (L-1-i) = dgrad of layer i, the next op = wgrad of
layer i.
"""
import torch

from . import conv3d as mc
from . import swap as sw


class Layer:
    def __init__(self, Cin, Cout, k=3, s=1, p=1):
        self.Cin, self.Cout, self.k, self.s, self.p = Cin, Cout, k, s, p


def _nbytes(shape, dtype=torch.bfloat16):
    n = 1
    for v in shape:
        n *= v
    return n * (2 if dtype == torch.bfloat16 else 4)


class ChainStep:
    def __init__(self, N, vol, layers, weights, x0, dy_last, budget_bytes=None, lookahead=1,
                 policy=sw.POLICY_BUDGET, n_tensors=-1, exclude_tags=0, swap=True, arena_slack=1.0):
        """weights: list of bf16 CUDA tensors [Cout,k,k,k,Cin]; x0: bf16 input
        [N,vol,vol,vol,Cin0]; dy_last: gradient w.r.t. the last layer's output.
        budget_bytes=None means no limit (nothing is swapped)."""
        self.N, self.layers, self.w = N, layers, weights
        self.L = L = len(layers)
        self.descs, self.shapes = [], [tuple(x0.shape)]
        v = vol
        for ly in layers:
            d = mc.make_desc(N, v, v, v, ly.Cin, ly.Cout, ly.k, ly.s, ly.p, torch.bfloat16)
            self.descs.append(d)
            v = mc.out_dims(d)[0]
            self.shapes.append((N, v, v, v, ly.Cout))
        assert tuple(dy_last.shape) == self.shapes[-1]
        self.x0, self.dy_last = x0, dy_last
        self.n_fwd, self.n_ops = L, 3 * L
        # algorithmic count: 2 * N*Do*Ho*Wo * k^3 * Cin * Cout per pass, three passes per layer
        self.flops_per_layer = [2.0 * (_nbytes(self.shapes[i + 1]) // (2 * ly.Cout)) * ly.k ** 3 * ly.Cin * ly.Cout
                                for i, ly in enumerate(layers)]
        self.flops_per_step = 3.0 * sum(self.flops_per_layer)
        ws_bytes = max(mc.workspace_bytes(d, p) for d in self.descs for p in range(3)) + 256
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        self.dw = [torch.empty(w.shape, dtype=torch.float32, device="cuda") for w in weights]
        # gradient buffers (transients): grad[i] is d(loss)/d(act[i])
        self.grad = [torch.empty(s, dtype=torch.bfloat16, device="cuda") for s in self.shapes[:-1]] + [dy_last]
        self.y_last = torch.empty(self.shapes[-1], dtype=torch.bfloat16, device="cuda")
        # saved tensors: act[i] = input of layer i, i = 0..L-1
        self.saved_bytes = [_nbytes(s) for s in self.shapes[:-1]]
        self.swap = swap
        sizes = self.saved_bytes
        self.engine = None
        if swap:
            budget = (1 << 62) if budget_bytes is None else int(budget_bytes)
            pool = sum((b + 4095) // 4096 * 4096 for b in sizes) + 4096
            arena_bytes = int(sum((b + 255) // 256 * 256 for b in sizes) * arena_slack) + 4096
            self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
            self.engine = e = sw.SwapEngine(budget_bytes=budget, host_pool_bytes=pool, arena=self.arena,
                                            lookahead=lookahead, policy=policy, n_tensors=n_tensors,
                                            exclude_tags=exclude_tags)
            e.set_timeline(self.n_fwd, self.n_ops)
            for i in range(L):
                tag = sw.TAG_INPUT if i == 0 else sw.TAG_ENCODER
                e.register(i, sizes[i], max(i - 1, 0), i, self.op_wgrad(i), self.op_wgrad(i), tag)
            for op in range(self.n_ops):
                e.set_transient(op, self._transient(op))
            self.plan_status = e.plan(allow_over_budget=True)
            self.planned = [e.is_planned(i) for i in range(L)]
            self.prefetch = [e.prefetch_op(i) for i in range(L)]
        else:
            self.planned = [False] * L
            self.acts = [x0] + [torch.empty(s, dtype=torch.bfloat16, device="cuda") for s in self.shapes[1:-1]]

    def op_dgrad(self, i):
        return self.L + 2 * (self.L - 1 - i)

    def op_wgrad(self, i):
        return self.op_dgrad(i) + 1

    def _transient(self, op):
        """Device bytes an op holds besides saved tensors: weights, weight
        gradients, workspace, the last output, and the gradient pair in use."""
        fixed = sum(w.numel() * 2 for w in self.w) + sum(d.numel() * 4 for d in self.dw) + self.ws.numel()
        fixed += _nbytes(self.shapes[-1]) * 2          # y_last and dy_last
        if op < self.n_fwd:
            return fixed
        i = self.L - 1 - (op - self.n_fwd) // 2
        return fixed + _nbytes(self.shapes[i]) + (_nbytes(self.shapes[i + 1]) if i + 1 < self.L else 0)

    def _view(self, ptr, shape):
        off = ptr - self.arena.data_ptr()
        return self.arena[off:off + _nbytes(shape)].view(torch.bfloat16).view(shape)

    def run(self):
        """One forward + backward pass; returns nothing (results stay on the device)."""
        L, e = self.L, self.engine
        if not self.swap:
            acts = self.acts
            for i in range(L):
                out = acts[i + 1] if i + 1 < L else self.y_last
                mc.conv3d_fwd(self.descs[i], acts[i], self.w[i], out, self.ws)
            for i in reversed(range(L)):
                mc.conv3d_dgrad(self.descs[i], self.grad[i + 1], self.w[i], self.grad[i], self.ws)
                mc.conv3d_wgrad(self.descs[i], acts[i], self.grad[i + 1], self.dw[i], self.ws)
            return
        e.reset_step()
        ptr = [None] * L
        acts = [None] * L
        # the network input is copied into the arena like a produced feature map
        ptr[0] = e.alloc(self.saved_bytes[0])
        acts[0] = self._view(ptr[0], self.shapes[0])
        acts[0].copy_(self.x0)
        if self.planned[0]:
            e.swap_out(0, ptr[0])
        for i in range(L):
            if i + 1 < L:
                ptr[i + 1] = e.alloc(self.saved_bytes[i + 1])
                acts[i + 1] = self._view(ptr[i + 1], self.shapes[i + 1])
                out = acts[i + 1]
            else:
                out = self.y_last
            mc.conv3d_fwd(self.descs[i], acts[i], self.w[i], out, self.ws)
            if i + 1 < L and self.planned[i + 1]:
                e.swap_out(i + 1, ptr[i + 1])          # copy starts once the producer has finished
            if self.planned[i]:
                e.release(i)                            # last forward reader of act[i] is enqueued
                ptr[i], acts[i] = None, None
        for op in range(self.n_fwd, self.n_ops):
            for t in range(L):                          # swap-ins due at this op (the lookahead knob)
                if self.planned[t] and self.prefetch[t] == op:
                    ptr[t] = e.alloc(self.saved_bytes[t])
                    e.swap_in(t, ptr[t])
                    acts[t] = self._view(ptr[t], self.shapes[t])
            i = L - 1 - (op - self.n_fwd) // 2
            if (op - self.n_fwd) % 2 == 0:
                mc.conv3d_dgrad(self.descs[i], self.grad[i + 1], self.w[i], self.grad[i], self.ws)
            else:
                if self.planned[i]:
                    e.wait_in(i)
                mc.conv3d_wgrad(self.descs[i], acts[i], self.grad[i + 1], self.dw[i], self.ws)
                if self.planned[i]:
                    e.done(i)
                e.free(ptr[i])
                ptr[i], acts[i] = None, None

    def close(self):
        if self.engine is not None:
            self.engine.close()
            self.engine = None
