"""MI355X-native local step of auxiliary-variable, module-parallel ResNet training.

`binding` exposes the C ABI of include/lp.h one to one (ctypes, argument marshalling only);
`runtime.LocalStep` holds the device buffers (PyTorch is used for device memory and streams only).
Every step of the path runs in the HIP library; there is no CPU fallback: if liblp.so is missing the
first call raises.
"""
from . import binding  # noqa: F401
from .runtime import LocalStep  # noqa: F401
