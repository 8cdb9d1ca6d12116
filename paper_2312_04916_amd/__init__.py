"""MI355X-native early-exit decode with KV recomputation: thin Python binding of the C ABI in include/ee.h.

The work is done by hand-written HIP kernels in ``libee.so`` (built in-tree by ``build.py``); this
package only marshals arguments and uses PyTorch for device memory and streams.  There is no CPU
fallback: importing :mod:`binding` fails loudly when the library has not been built.
"""
from .binding import *  # noqa: F401,F403
