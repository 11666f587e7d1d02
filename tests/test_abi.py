"""The C-ABI library loads and exports every symbol include/mi3d.h declares
(no compute calls; runs without a GPU)."""
import ctypes
import os
import re

from paper_1812_07816_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "mi3d.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mi3d_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_hot_path_calls():
    names = _declared()
    for n in ("mi3d_conv3d_fwd", "mi3d_conv3d_dgrad", "mi3d_conv3d_wgrad", "mi3d_swap_out", "mi3d_swap_in", "mi3d_swap_plan"):
        assert n in names


def test_library_exports_every_declared_symbol():
    l = ctypes.CDLL(_lib.LIB_PATH)
    for n in _declared():
        assert hasattr(l, n), n


def test_binding_covers_every_declared_symbol():
    assert sorted(_lib.SIGNATURES) == _declared()


def test_status_strings():
    l = _lib.lib()
    seen = set()
    for s in range(0, -8, -1):
        msg = l.mi3d_status_string(s)
        assert msg and msg not in seen
        seen.add(msg)
    assert l.mi3d_status_string(-99) == b"unknown status"


def test_descriptor_validation_needs_no_gpu():
    from paper_1812_07816_amd import conv3d as mc
    d = mc.make_desc(1, 192, 192, 192, 32, 64, 3, 2, 1, 1)
    assert mc.out_dims(d) == (96, 96, 96)
    a = ctypes.c_int()
    bad = mc.make_desc(1, 1, 4, 4, 1, 1, 3, 1, 0, 0)
    assert _lib.lib().mi3d_conv3d_out_dims(ctypes.byref(bad), ctypes.byref(a), ctypes.byref(a), ctypes.byref(a)) == -1
    bad = mc.make_desc(1, 4, 4, 4, 1, 1, 3, 1, 1, 7)
    assert _lib.lib().mi3d_conv3d_out_dims(ctypes.byref(bad), ctypes.byref(a), ctypes.byref(a), ctypes.byref(a)) == -2
    # null pointers are rejected before anything is launched
    assert _lib.lib().mi3d_conv3d_fwd(ctypes.byref(d), None, None, None, None, 0, None) == -1
    assert _lib.lib().mi3d_conv3d_fwd(None, None, None, None, None, 0, None) == -1


def test_largest_sizes_are_routed_by_their_plane_size_or_refused():
    """The tiled kernels address inside a D-plane with 32-bit offsets: a descriptor whose planes reach 2 GiB must go to
    the kernels with 64-bit indices, whatever its channel counts; one beyond 2^40 elements is refused outright.
    (Host logic only: nothing is launched.)"""
    import torch
    from paper_1812_07816_amd import conv3d as mc
    bf = torch.bfloat16
    # 64 GiB tensors with 64 MiB planes: still the tiled kernels
    d = mc.make_desc(1, 1024, 1024, 1024, 32, 32, 3, 1, 1, bf)
    assert [mc.kernel_name(d, q) for q in range(3)] == ["mfma_plane_stream", "mfma_plane_stream", "mfma_wgrad_plane_stream"]
    # the last plane size below the limit, and the first one at it
    d = mc.make_desc(1, 4, 4096, 4096, 32, 32, 3, 1, 1, bf)          # 1 GiB planes
    assert mc.kernel_name(d, 0) == "mfma_plane_stream"
    for args in ((1, 4, 8192, 8192, 32, 32, 3, 1, 1),     # stride 1, 4 GiB planes
                 (1, 4, 4096, 4096, 64, 64, 3, 1, 1),     # exactly 2 GiB
                 (1, 4, 8192, 4096, 32, 32, 3, 2, 1),     # stride 2: the input plane decides
                 (1, 4, 16384, 16384, 4, 32, 3, 1, 1)):   # first layer: the output plane decides
        d = mc.make_desc(*args, bf)
        assert [mc.kernel_name(d, q) for q in range(3)] == ["direct"] * 3, args
    a = ctypes.c_int()
    huge = mc.make_desc(64, 4096, 4096, 4096, 32, 32, 3, 1, 1, bf)   # 2^47 elements
    assert _lib.lib().mi3d_conv3d_out_dims(ctypes.byref(huge), ctypes.byref(a), ctypes.byref(a), ctypes.byref(a)) == -2
