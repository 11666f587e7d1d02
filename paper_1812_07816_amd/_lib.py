"""Loads libmi3d.so and declares its C ABI (include/mi3d.h) for ctypes."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmi3d.so")


class ConvDesc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "D", "H", "W", "Cin", "Cout", "kD", "kH", "kW",
                 "sD", "sH", "sW", "pD", "pH", "pW", "dtype")]


class View(ctypes.Structure):
    _fields_ = [("pitch", ctypes.c_int), ("offset", ctypes.c_int)]


class SwapConfig(ctypes.Structure):
    _fields_ = [("budget_bytes", ctypes.c_size_t), ("dev_arena", ctypes.c_void_p),
                ("arena_bytes", ctypes.c_size_t), ("host_pool_bytes", ctypes.c_size_t),
                ("lookahead", ctypes.c_int), ("policy", ctypes.c_int), ("n_tensors", ctypes.c_int),
                ("exclude_tags", ctypes.c_uint), ("include_tags", ctypes.c_uint)]


class SwapStats(ctypes.Structure):
    _fields_ = [("bytes_out", ctypes.c_uint64), ("bytes_in", ctypes.c_uint64),
                ("copy_ms_out", ctypes.c_double), ("copy_ms_in", ctypes.c_double),
                ("busy_ms", ctypes.c_double),
                ("peak_arena_bytes", ctypes.c_uint64), ("arena_high_water_bytes", ctypes.c_uint64),
                ("planned_arena_bytes", ctypes.c_uint64), ("static_arena_bytes", ctypes.c_uint64), ("n_arena_overflow", ctypes.c_int),
                ("planned_peak_bytes", ctypes.c_uint64),
                ("unswapped_peak_bytes", ctypes.c_uint64),
                ("n_registered", ctypes.c_int), ("n_planned", ctypes.c_int),
                ("n_swapped_out", ctypes.c_int), ("n_swapped_in", ctypes.c_int),
                ("n_recompute", ctypes.c_int), ("recompute_ms", ctypes.c_double),
                ("n_checksummed", ctypes.c_int), ("n_checksum_mismatch", ctypes.c_int)]


_vp, _sz, _i, _u = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint
_pd = ctypes.POINTER(ConvDesc)
_pi = ctypes.POINTER(ctypes.c_int)

# name -> (restype, argtypes); one entry per declaration in include/mi3d.h
SIGNATURES = {
    "mi3d_status_string": (ctypes.c_char_p, [_i]),
    "mi3d_last_hip_error": (_i, []),
    "mi3d_conv3d_out_dims": (_i, [_pd, _pi, _pi, _pi]),
    "mi3d_leaky_relu_fwd": (_i, [_vp, _sz, ctypes.c_float, _vp]),
    "mi3d_leaky_relu_bwd": (_i, [_vp, _vp, _sz, ctypes.c_float, _vp]),
    "mi3d_leaky_relu_bwd_f32": (_i, [_vp, _vp, _sz, ctypes.c_float, _vp]),
    "mi3d_dice_loss_f32": (_i, [_vp, _vp, _sz, _i, ctypes.c_float, _vp, _sz, _vp, _vp, _vp]),
    "mi3d_dice_grad_f32": (_i, [_vp, _vp, _sz, _i, ctypes.c_float, _vp, _vp, _vp]),
    "mi3d_concat_channels": (_i, [_vp, _i, _vp, _i, _vp, _sz, _vp]),
    "mi3d_split_channels": (_i, [_vp, _i, _i, _vp, _vp, _sz, _vp]),
    "mi3d_add_inplace": (_i, [_vp, _vp, _sz, _vp]),
    "mi3d_slice_channels": (_i, [_vp, _i, _i, _i, _vp, _sz, _vp]),
    "mi3d_place_channels": (_i, [_vp, _i, _vp, _i, _i, _sz, _vp]),
    "mi3d_skip_grad": (_i, [_vp, _vp, _i, _i, _vp, _i, _sz, ctypes.c_float, _vp]),
    "mi3d_dice_workspace_bytes": (_sz, [_i]),
    "mi3d_dice_loss": (_i, [_vp, _vp, _sz, _i, ctypes.c_float, _vp, _sz, _vp, _vp, _vp]),
    "mi3d_dice_grad": (_i, [_vp, _vp, _sz, _i, ctypes.c_float, _vp, _vp, _vp]),
    "mi3d_sgd_update": (_i, [_vp, _vp, _vp, _sz, ctypes.c_float, _vp]),
    "mi3d_instnorm_workspace_bytes": (_sz, [_i, _i]),
    "mi3d_instnorm_stats": (_i, [_vp, _i, _sz, _i, ctypes.c_float, _vp, _vp, _sz, _vp]),
    "mi3d_instnorm_lrelu_fwd": (_i, [_vp, _vp, _i, _sz, _i, ctypes.c_float, _vp]),
    "mi3d_instnorm_lrelu_bwd": (_i, [_vp, _vp, _vp, _i, _sz, _i, ctypes.c_float, _vp, _sz, _vp]),
    "mi3d_instnorm_stats_f32": (_i, [_vp, _i, _sz, _i, ctypes.c_float, _vp, _vp, _sz, _vp]),
    "mi3d_instnorm_lrelu_fwd_f32": (_i, [_vp, _vp, _i, _sz, _i, ctypes.c_float, _vp]),
    "mi3d_instnorm_lrelu_bwd_f32": (_i, [_vp, _vp, _vp, _i, _sz, _i, ctypes.c_float, _vp, _sz, _vp]),
    "mi3d_adam_update": (_i, [_vp, _vp, _vp, _vp, _vp, _sz, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float, _i, _vp]),
    "mi3d_conv3d_workspace_bytes": (_sz, [_pd, _i]),
    "mi3d_conv3d_fwd": (_i, [_pd, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_dgrad": (_i, [_pd, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_wgrad": (_i, [_pd, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mi3d_static_scratch_bytes": (_sz, []),
    "mi3d_conv3d_wgrad_static": (_i, [_pd, _vp, _vp, _vp, _vp]),
    "mi3d_conv3d_fwd_view": (_i, [_pd, _vp, ctypes.POINTER(View), _vp, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_dgrad_view": (_i, [_pd, _vp, _vp, _vp, ctypes.POINTER(View), _vp, _sz, _vp]),
    "mi3d_conv3d_wgrad_view": (_i, [_pd, _vp, ctypes.POINTER(View), _vp, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_dgrad_skip": (_i, [_pd, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_dgrad_insums_supported": (_i, [_pd, _i]),
    "mi3d_conv3d_dgrad_insums": (_i, [_pd, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _sz, _vp]),
    "mi3d_instnorm_lrelu_bwd_sums": (_i, [_vp, _vp, _vp, _vp, _i, _sz, _i, ctypes.c_float, _vp]),
    "mi3d_conv3d_fwd_stats_supported": (_i, [_pd]),
    "mi3d_conv3d_fwd_stats": (_i, [_pd, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_pair_supported": (_i, [_pd, _i]),
    "mi3d_conv3d_fwd_pair": (_i, [_pd, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _sz, _vp]),
    "mi3d_conv3d_dgrad_pair": (_i, [_pd, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_wgrad_pair": (_i, [_pd, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_fwd_lrelu": (_i, [_pd, _vp, _vp, _vp, ctypes.c_float, _vp, _sz, _vp]),
    "mi3d_conv3d_dgrad_lrelu": (_i, [_pd, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _sz, _vp]),
    "mi3d_conv3d_kernel_name": (_i, [_pd, _i, ctypes.c_char_p, _sz]),
    "mi3d_swap_create": (_i, [ctypes.POINTER(SwapConfig), ctypes.POINTER(_vp)]),
    "mi3d_swap_destroy": (_i, [_vp]),
    "mi3d_swap_set_timeline": (_i, [_vp, _i, _i]),
    "mi3d_swap_register": (_i, [_vp, _i, _sz, _i, _i, _i, _i, _u]),
    "mi3d_swap_set_eviction": (_i, [_vp, _i]),
    "mi3d_swap_set_recompute": (_i, [_vp, _i, ctypes.c_float, _i, _i]),
    "mi3d_swap_is_recomputed": (_i, [_vp, _i]),
    "mi3d_swap_first_use_op": (_i, [_vp, _i]),
    "mi3d_swap_set_op_times": (_i, [_vp, ctypes.POINTER(ctypes.c_float), _i, ctypes.c_float]),
    "mi3d_swap_set_transient": (_i, [_vp, _i, _sz]),
    "mi3d_swap_plan": (_i, [_vp]),
    "mi3d_swap_is_planned": (_i, [_vp, _i]),
    "mi3d_swap_prefetch_op": (_i, [_vp, _i]),
    "mi3d_swap_planned_bytes_at": (_i, [_vp, _i, ctypes.POINTER(ctypes.c_uint64)]),
    "mi3d_swap_alloc": (_i, [_vp, _sz, _vp, ctypes.POINTER(_vp)]),
    "mi3d_swap_free": (_i, [_vp, _vp, _vp]),
    "mi3d_swap_set_arena": (_i, [_vp, _vp, _sz]),
    "mi3d_swap_set_budget": (_i, [_vp, _sz]),
    "mi3d_swap_planned_offset": (_i, [_vp, _i, _i, ctypes.POINTER(ctypes.c_uint64)]),
    "mi3d_swap_static_arena_bytes": (_i, [_vp, ctypes.POINTER(ctypes.c_uint64)]),
    "mi3d_swap_alloc_tensor": (_i, [_vp, _i, _vp, ctypes.POINTER(_vp)]),
    "mi3d_swap_out": (_i, [_vp, _i, _vp, _vp]),
    "mi3d_swap_release": (_i, [_vp, _i, _vp]),
    "mi3d_swap_in": (_i, [_vp, _i, _vp, _vp]),
    "mi3d_swap_wait_in": (_i, [_vp, _i, _vp]),
    "mi3d_swap_done": (_i, [_vp, _i]),
    "mi3d_swap_set_verify": (_i, [_vp, _i]),
    "mi3d_checksum64": (_i, [_vp, _sz, ctypes.POINTER(ctypes.c_uint64), _vp]),
    "mi3d_swap_sync": (_i, [_vp]),
    "mi3d_swap_reset_step": (_i, [_vp]),
    "mi3d_swap_stats": (_i, [_vp, ctypes.POINTER(SwapStats)]),
}

_lib = None


class Mi3dError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = lib().mi3d_status_string(status).decode()
        if status == -4:
            msg += f" (hipError {lib().mi3d_last_hip_error()})"
        super().__init__(f"{what}: {msg} [{status}]")


def lib():
    """The loaded library.  There is no fallback: if the HIP extension has not
    been built this raises."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or paper_1812_07816_amd/build.py) first")
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def check(status, what):
    if status != 0:
        raise Mi3dError(status, what)
