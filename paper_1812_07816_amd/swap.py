"""Thin binding of the data-swapping engine (marshalling only)."""
import ctypes

import torch

from ._lib import SwapConfig, SwapStats, check, lib

POLICY_BUDGET, POLICY_ALL, POLICY_FIRST_N = 0, 1, 2
EVICT_SWAP, EVICT_RECOMPUTE, EVICT_HYBRID = 0, 1, 2
TAG_ENCODER, TAG_DECODER, TAG_INPUT, TAG_HEAD = 1, 2, 4, 8


def _stream(stream=None):
    if stream is None:
        if not torch.cuda.is_available():
            return ctypes.c_void_p(None)  # host-only use (planner); the library rejects copies itself
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class SwapEngine:
    def __init__(self, budget_bytes, host_pool_bytes=0, arena=None, lookahead=1, policy=POLICY_BUDGET,
                 n_tensors=-1, exclude_tags=0, include_tags=0):
        self.arena = arena  # keeps the torch buffer alive
        ap = arena.data_ptr() if arena is not None else None
        an = arena.numel() * arena.element_size() if arena is not None else 0
        cfg = SwapConfig(int(budget_bytes), ap, an, int(host_pool_bytes), int(lookahead), int(policy),
                         int(n_tensors), int(exclude_tags), int(include_tags))
        h = ctypes.c_void_p()
        check(lib().mi3d_swap_create(ctypes.byref(cfg), ctypes.byref(h)), "swap_create")
        self._h = h

    def close(self):
        if self._h is not None:
            h, self._h = self._h, None
            check(lib().mi3d_swap_destroy(h), "swap_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_timeline(self, n_fwd_ops, n_ops):
        check(lib().mi3d_swap_set_timeline(self._h, n_fwd_ops, n_ops), "swap_set_timeline")

    def register(self, id, bytes, produce_op, last_fwd_use_op, bwd_first_use_op, bwd_last_use_op, tags=0):
        check(lib().mi3d_swap_register(self._h, id, bytes, produce_op, last_fwd_use_op, bwd_first_use_op,
                                       bwd_last_use_op, tags), "swap_register")

    def set_op_times(self, ms, link_gbs):
        arr = (ctypes.c_float * len(ms))(*[float(v) for v in ms])
        check(lib().mi3d_swap_set_op_times(self._h, arr, len(ms), float(link_gbs)), "swap_set_op_times")

    def set_eviction(self, eviction):
        check(lib().mi3d_swap_set_eviction(self._h, int(eviction)), "swap_set_eviction")

    def set_recompute(self, id, cost_ms, dep0=-1, dep1=-1):
        check(lib().mi3d_swap_set_recompute(self._h, id, float(cost_ms), dep0, dep1), "swap_set_recompute")

    def is_recomputed(self, id):
        r = lib().mi3d_swap_is_recomputed(self._h, id)
        if r < 0:
            check(r, "swap_is_recomputed")
        return bool(r)

    def first_use_op(self, id):
        r = lib().mi3d_swap_first_use_op(self._h, id)
        if r < 0:
            check(r, "swap_first_use_op")
        return r

    def set_transient(self, op, bytes):
        check(lib().mi3d_swap_set_transient(self._h, op, bytes), "swap_set_transient")

    def plan(self, allow_over_budget=False):
        st = lib().mi3d_swap_plan(self._h)
        if st == -6 and allow_over_budget:
            return st
        check(st, "swap_plan")
        return st

    def is_planned(self, id):
        r = lib().mi3d_swap_is_planned(self._h, id)
        if r < 0:
            check(r, "swap_is_planned")
        return bool(r)

    def prefetch_op(self, id):
        r = lib().mi3d_swap_prefetch_op(self._h, id)
        if r < 0:
            check(r, "swap_prefetch_op")
        return r

    def planned_bytes_at(self, op):
        b = ctypes.c_uint64()
        check(lib().mi3d_swap_planned_bytes_at(self._h, op, ctypes.byref(b)), "swap_planned_bytes_at")
        return b.value

    def alloc(self, bytes, stream=None):
        p = ctypes.c_void_p()
        check(lib().mi3d_swap_alloc(self._h, bytes, _stream(stream), ctypes.byref(p)), "swap_alloc")
        return p.value

    def set_arena(self, arena):
        """Replaces the device arena (a torch uint8 CUDA tensor, or None); no block may be handed out."""
        check(lib().mi3d_swap_set_arena(self._h, None if arena is None else arena.data_ptr(),
                                        0 if arena is None else arena.numel() * arena.element_size()), "swap_set_arena")
        self.arena = arena

    def set_budget(self, budget_bytes):
        check(lib().mi3d_swap_set_budget(self._h, int(budget_bytes)), "swap_set_budget")

    def static_arena_bytes(self):
        b = ctypes.c_uint64()
        check(lib().mi3d_swap_static_arena_bytes(self._h, ctypes.byref(b)), "swap_static_arena_bytes")
        return b.value

    def planned_offset(self, id, stay=0):
        b = ctypes.c_uint64()
        check(lib().mi3d_swap_planned_offset(self._h, id, stay, ctypes.byref(b)), "swap_planned_offset")
        return b.value

    def alloc_tensor(self, id, stream=None):
        """The planned place of saved tensor `id` in the arena (its first or second stay, in call order)."""
        p = ctypes.c_void_p()
        check(lib().mi3d_swap_alloc_tensor(self._h, id, _stream(stream), ctypes.byref(p)), "swap_alloc_tensor")
        return p.value

    def free(self, ptr, stream=None):
        check(lib().mi3d_swap_free(self._h, ptr, _stream(stream)), "swap_free")

    def swap_out(self, id, dev_src, stream=None):
        check(lib().mi3d_swap_out(self._h, id, dev_src, _stream(stream)), "swap_out")

    def release(self, id, stream=None):
        check(lib().mi3d_swap_release(self._h, id, _stream(stream)), "swap_release")

    def swap_in(self, id, dev_dst, stream=None):
        check(lib().mi3d_swap_in(self._h, id, dev_dst, _stream(stream)), "swap_in")

    def wait_in(self, id, stream=None):
        check(lib().mi3d_swap_wait_in(self._h, id, _stream(stream)), "swap_wait_in")

    def done(self, id):
        check(lib().mi3d_swap_done(self._h, id), "swap_done")

    def set_verify(self, on=True):
        """Checksum mode: every swapped tensor is summed before it leaves and after it is back; see stats()."""
        check(lib().mi3d_swap_set_verify(self._h, int(bool(on))), "swap_set_verify")

    def sync(self):
        check(lib().mi3d_swap_sync(self._h), "swap_sync")

    def reset_step(self):
        check(lib().mi3d_swap_reset_step(self._h), "swap_reset_step")

    def stats(self):
        s = SwapStats()
        check(lib().mi3d_swap_stats(self._h, ctypes.byref(s)), "swap_stats")
        return {k: getattr(s, k) for k, _ in SwapStats._fields_}


def checksum64(t, stream=None):
    """64-bit checksum of a CUDA tensor's bytes (the function of the engine's checksum mode)."""
    v = ctypes.c_uint64()
    check(lib().mi3d_checksum64(t.data_ptr(), t.numel() * t.element_size(), ctypes.byref(v), _stream(stream)), "checksum64")
    return v.value
