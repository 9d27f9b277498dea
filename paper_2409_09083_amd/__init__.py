"""MI355X-native fused tile partitioning of early CNN layers (forward + back-propagation).

`binding` mirrors the C ABI of libftp.so one to one; `harness.Session` holds the device buffers
(PyTorch is used for device memory and streams only).
"""
from . import binding  # noqa: F401  (raises if libftp.so is not built)
from .binding import *  # noqa: F401,F403
