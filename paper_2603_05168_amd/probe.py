"""ctypes binding of libsbn_probe.so (include/sbn_probe.h): the ceiling probes the benchmark runs next to the
layer's kernels.  Measurement support, apart from the layer's library; argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsbn_probe.so")

SBN_CEIL_SMFMAC_I8, SBN_CEIL_MFMA_I8, SBN_CEIL_MFMA_BF16, SBN_CEIL_HBM_READ, SBN_CEIL_HBM_WRITE, SBN_CEIL_LDS_READ = range(6)


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.sbn_ceiling_probe.restype = ctypes.c_int
    lib.sbn_ceiling_probe.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    return lib


_lib = _load()


def lib_path() -> str:
    return _LIB_PATH


def sbn_ceiling_probe(kind: int, buf, iters: int = 1) -> float:
    """Enqueue one ceiling-probe kernel on the current torch stream; returns the operations or bytes it performs."""
    work = ctypes.c_double(0.0)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None
    rc = _lib.sbn_ceiling_probe(kind, ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), iters,
                                ctypes.byref(work), stream)
    if rc != 0:
        raise RuntimeError(f"sbn_ceiling_probe: status {rc}")
    return work.value
