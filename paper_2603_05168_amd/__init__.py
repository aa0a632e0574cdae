"""MI355X-native N:M-sparse ternary linear layer (Sparse-BitNet, arxiv 2603.05168).

The work is done by hand-written HIP kernels in libsbn.so behind the C ABI of include/sbn.h; this
package is the thin ctypes binding with the same entry-point names.  PyTorch appears only as the
owner of device memory and streams.  There is no CPU fallback: if the library is missing the import
of `binding` fails with an error that says how to build it.
"""
from .binding import *  # noqa: F401,F403
