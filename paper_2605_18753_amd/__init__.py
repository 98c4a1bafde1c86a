"""MI355X-native DashAttention forward path: HIP kernels behind a C ABI
(include/dash_attn.h) plus a thin ctypes binding.  Importing the package does
not load the shared library; the first call does, and fails loudly if it is
missing."""
from . import binding, inputs  # noqa: F401
