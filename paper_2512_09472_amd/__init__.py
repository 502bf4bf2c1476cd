"""warmkv: MI355X-native KV-cache reclaim (plan, compact, remap) and weight
materialisation behind a C ABI (include/warmkv.h, libwarmkv.so).

The package namespace is the binding's: one Python function per exported C
function (binding.EXPORTS), the status codes, and the small helpers that build
argument structures."""
from . import binding
from .binding import *  # noqa: F401,F403

__all__ = list(binding.__all__)
