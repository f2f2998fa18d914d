"""MI355X-native SwiftKV prefill: HIP kernels behind a C ABI (libswiftkv.so)
and a thin ctypes binding.  Nothing here computes on the CPU."""
from . import binding  # noqa: F401
