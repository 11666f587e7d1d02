"""MI355X-native hot path of full-resolution 3D U-Net training with data
swapping: Conv3D forward / data-gradient / weight-gradient HIP kernels and a
swap engine, behind the C ABI of include/mi3d.h.  This package is only the
ctypes binding; there is no CPU fallback."""
from . import conv3d, swap  # noqa: F401
from ._lib import Mi3dError, lib  # noqa: F401
