"""MI355X-native G-KV decode/evict hot path: HIP kernels behind a C ABI (libgkv.so)
and a thin ctypes binding.  See include/gkv.h for the contract of every call."""
from .binding import (Context, GkvConfig, GkvError, EXPORTS, LIB_PATH, cache_bytes, k_offset,
                      load_library, make_config)

__all__ = ["Context", "GkvConfig", "GkvError", "EXPORTS", "LIB_PATH", "cache_bytes", "k_offset",
           "load_library", "make_config"]
