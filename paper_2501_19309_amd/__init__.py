"""MI355X-native batched verification head of Judge Decoding (arXiv 2501.19309).

The product is the C-ABI library ``libjdverify.so`` (include/jd_verify.h); this
package holds its HIP sources (``csrc/``), the build step and a thin ctypes binding.
"""

from . import binding
from .binding import JDVerify, JDError, make_config, load_library

__all__ = ["binding", "JDVerify", "JDError", "make_config", "load_library"]
