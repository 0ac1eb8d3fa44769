"""MI355X-native single-launch decode step (persistent megakernel with an
offline-synthesised static schedule).  The product is ``libmk.so`` (HIP kernels
+ C ABI, see ``include/mk.h``); this package is its thin ctypes binding.
PyTorch is used only for device memory and streams."""
from .binding import *  # noqa: F401,F403
