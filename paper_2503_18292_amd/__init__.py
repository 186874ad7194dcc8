"""MI355X-native paged decode attention + KV append over a two-level (LCM) KV page pool.

The work is done by libjenga.so (csrc/, C ABI in include/jenga.h); this package is the
thin Python binding: same names, argument marshalling only.
"""
from .api import (BF16, CROSS, F32, FULL, OPAQUE, WINDOW, JengaError, KindDesc, Pool, lcm_page_bytes,
                  stream_copy, stream_read, version)

__all__ = ["Pool", "KindDesc", "JengaError", "lcm_page_bytes", "stream_copy", "stream_read",
           "version", "F32", "BF16", "FULL", "WINDOW", "CROSS", "OPAQUE"]
