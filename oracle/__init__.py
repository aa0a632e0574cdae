"""CPU oracle of the N:M-sparse ternary linear layer (Sparse-BitNet, arxiv 2603.05168).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports it and it imports nothing from the product.
The arithmetic lives in sbn_oracle.c (plain C loops, each function citing the passage it follows);
this module only marshals numpy arrays into it and chains the steps in the paper's order.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from .build import build as _build

_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build())
        i64, f32, cint = ctypes.c_int64, ctypes.c_float, ctypes.c_int
        vp = ctypes.c_void_p
        lib.sbn_oracle_absmean.restype = f32
        lib.sbn_oracle_absmean.argtypes = [vp, i64, i64]
        lib.sbn_oracle_nm_mask.restype = None
        lib.sbn_oracle_nm_mask.argtypes = [vp, i64, i64, cint, cint, vp]
        lib.sbn_oracle_ternary.restype = None
        lib.sbn_oracle_ternary.argtypes = [vp, i64, f32, vp]
        lib.sbn_oracle_apply_mask.restype = None
        lib.sbn_oracle_apply_mask.argtypes = [vp, vp, i64, vp]
        lib.sbn_oracle_act_quant.restype = None
        lib.sbn_oracle_act_quant.argtypes = [vp, i64, i64, vp, vp]
        lib.sbn_oracle_acc.restype = None
        lib.sbn_oracle_rmsnorm.argtypes = [vp, vp, f32, i64, i64, vp]
        lib.sbn_oracle_rmsnorm.restype = None
        lib.sbn_oracle_acc.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.sbn_oracle_rescale.restype = None
        lib.sbn_oracle_rescale.argtypes = [vp, f32, vp, vp, i64, i64, vp]
        lib.sbn_oracle_backward_dx.restype = None
        lib.sbn_oracle_backward_dx.argtypes = [vp, vp, f32, i64, i64, i64, vp]
        lib.sbn_oracle_backward_dw.restype = None
        lib.sbn_oracle_backward_dw.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        lib.sbn_oracle_chunk_bytes.restype = i64
        lib.sbn_oracle_chunk_bytes.argtypes = [cint, cint]
        lib.sbn_oracle_packed_bytes.restype = i64
        lib.sbn_oracle_packed_bytes.argtypes = [i64, i64, cint, cint]
        lib.sbn_oracle_pack.restype = cint
        lib.sbn_oracle_pack.argtypes = [vp, vp, i64, i64, cint, cint, vp]
        lib.sbn_oracle_unpack.restype = cint
        lib.sbn_oracle_unpack.argtypes = [vp, i64, i64, cint, cint, vp, vp]
        lib.sbn_oracle_flip_rate.restype = ctypes.c_double
        lib.sbn_oracle_flip_rate.argtypes = [vp, vp, i64]
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _f32(a) -> np.ndarray:
    """Inputs arrive as fp32 numpy arrays (bf16 tensors are up-converted exactly by the caller)."""
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs must be float32 (convert bf16 exactly before the call)")
    if not np.isfinite(a).all():
        raise ValueError("oracle inputs must be finite")
    return a


def absmean(W) -> np.float32:
    W = _f32(W)
    return np.float32(_L().sbn_oracle_absmean(_p(W), W.shape[0], W.shape[1]))


def nm_mask(W, N: int, M: int) -> np.ndarray:
    W = _f32(W)
    if W.shape[1] % M or not (1 <= N <= M):
        raise ValueError("d_in must be a multiple of M and 1 <= N <= M")
    mask = np.empty(W.shape, dtype=np.uint8)
    _L().sbn_oracle_nm_mask(_p(W), W.shape[0], W.shape[1], N, M, _p(mask))
    return mask


def ternary(W, gamma) -> np.ndarray:
    W = _f32(W)
    Wq = np.empty(W.shape, dtype=np.int8)
    _L().sbn_oracle_ternary(_p(W), W.size, ctypes.c_float(float(gamma)), _p(Wq))
    return Wq


def apply_mask(Wq: np.ndarray, mask: np.ndarray) -> np.ndarray:
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.empty(Wq.shape, dtype=np.int8)
    _L().sbn_oracle_apply_mask(_p(Wq), _p(mask), Wq.size, _p(out))
    return out


def quantize_mask(W, N: int, M: int):
    """Steps of the weight side in the paper's order: mask from latent W, gamma from the full W,
    ternary quantization, then W_eff = W_q * mask.  Returns (W_eff int8, mask uint8, gamma fp32)."""
    mask = nm_mask(W, N, M)
    gamma = absmean(W)
    Wq = ternary(W, gamma)
    return apply_mask(Wq, mask), mask, gamma


def chunk_bytes(N: int, M: int) -> int:
    return int(_L().sbn_oracle_chunk_bytes(N, M))


def packed_bytes(d_out: int, d_in: int, N: int, M: int) -> int:
    return int(_L().sbn_oracle_packed_bytes(d_out, d_in, N, M))


def pack(Weff: np.ndarray, mask: np.ndarray, N: int, M: int) -> np.ndarray:
    Weff = np.ascontiguousarray(Weff, dtype=np.int8)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    nb = packed_bytes(Weff.shape[0], Weff.shape[1], N, M)
    if nb < 0:
        raise ValueError("unsupported pattern or shape")
    out = np.empty(nb, dtype=np.uint8)
    rc = _L().sbn_oracle_pack(_p(Weff), _p(mask), Weff.shape[0], Weff.shape[1], N, M, _p(out))
    if rc:
        raise ValueError(f"pack failed ({rc}): mask does not hold exactly N ones per group")
    return out


def unpack(packed: np.ndarray, d_out: int, d_in: int, N: int, M: int):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    if packed.size != packed_bytes(d_out, d_in, N, M):
        raise ValueError("packed buffer has the wrong size")
    Weff = np.empty((d_out, d_in), dtype=np.int8)
    mask = np.empty((d_out, d_in), dtype=np.uint8)
    rc = _L().sbn_oracle_unpack(_p(packed), d_out, d_in, N, M, _p(Weff), _p(mask))
    if rc:
        raise ValueError(f"unpack failed ({rc})")
    return Weff, mask


def quantize_mask_pack(W, N: int, M: int):
    """Returns (packed bytes, gamma) for a latent matrix W [d_out, d_in] (fp32 numpy)."""
    Weff, mask, gamma = quantize_mask(W, N, M)
    return pack(Weff, mask, N, M), gamma


def act_quant(X):
    X = _f32(X)
    xq = np.empty(X.shape, dtype=np.int8)
    sx = np.empty(X.shape[0], dtype=np.float32)
    _L().sbn_oracle_act_quant(_p(X), X.shape[0], X.shape[1], _p(xq), _p(sx))
    return xq, sx


def rmsnorm(X, gain=None, eps: float = 1e-6) -> np.ndarray:
    """Algorithm 1's Norm(x), read as RMS normalisation with gain; values are bf16-representable floats."""
    X = _f32(X)
    g = None if gain is None else _f32(gain)
    Xn = np.empty(X.shape, dtype=np.float32)
    _L().sbn_oracle_rmsnorm(_p(X), None if g is None else _p(g), np.float32(eps), X.shape[0], X.shape[1], _p(Xn))
    return Xn


def rmsnorm_act_quant(X, gain=None, eps: float = 1e-6):
    """x~, s_x = Q_a(Norm(x)) (Algorithm 1); also returns the normalised activations."""
    Xn = rmsnorm(X, gain, eps)
    xq, sx = act_quant(Xn)
    return xq, sx, Xn


def acc(Weff: np.ndarray, xq: np.ndarray) -> np.ndarray:
    Weff = np.ascontiguousarray(Weff, dtype=np.int8)
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    T, K = xq.shape
    d_out = Weff.shape[0]
    assert Weff.shape[1] == K
    out = np.empty((T, d_out), dtype=np.int32)
    _L().sbn_oracle_acc(_p(Weff), _p(xq), T, K, d_out, _p(out))
    return out


def rescale(acc_: np.ndarray, gamma, sx: np.ndarray, bias=None) -> np.ndarray:
    acc_ = np.ascontiguousarray(acc_, dtype=np.int32)
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    T, d_out = acc_.shape
    y = np.empty((T, d_out), dtype=np.float64)
    b = None
    if bias is not None:
        b = np.ascontiguousarray(bias, dtype=np.float32)
    _L().sbn_oracle_rescale(_p(acc_), ctypes.c_float(float(gamma)), _p(sx),
                            _p(b) if b is not None else None, T, d_out, _p(y))
    return y


def sparse_ternary_linear(X, Weff: np.ndarray, gamma, bias=None):
    """Forward of the layer from dense W_eff: returns (y fp64, acc int32, xq int8, sx fp32)."""
    xq, sx = act_quant(X)
    a = acc(Weff, xq)
    return rescale(a, gamma, sx, bias), a, xq, sx


def backward_dx(dY, Weff: np.ndarray, gamma) -> np.ndarray:
    dY = _f32(dY)
    Weff = np.ascontiguousarray(Weff, dtype=np.int8)
    T, d_out = dY.shape
    K = Weff.shape[1]
    assert Weff.shape[0] == d_out
    dX = np.empty((T, K), dtype=np.float64)
    _L().sbn_oracle_backward_dx(_p(dY), _p(Weff), ctypes.c_float(float(gamma)), T, K, d_out, _p(dX))
    return dX


def backward_dw(dY, xq: np.ndarray, sx: np.ndarray) -> np.ndarray:
    dY = _f32(dY)
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    T, d_out = dY.shape
    K = xq.shape[1]
    assert xq.shape[0] == T and sx.shape[0] == T
    dW = np.empty((d_out, K), dtype=np.float64)
    _L().sbn_oracle_backward_dw(_p(dY), _p(xq), _p(sx), T, K, d_out, _p(dW))
    return dW


def backward_dw_gradient_masked(dY, xq: np.ndarray, sx: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """The ablation study's "gradient masking" variant (Section 2.3 names it as what other N:M methods
    do): dL/dW ~ M (.) dL/dW_eff, i.e. the dense gradient with the entries of masked-out weights
    blocked.  Same forward pass; only the weights of the current mask receive an update."""
    dW = backward_dw(dY, xq, sx)
    mask = np.ascontiguousarray(mask)
    assert mask.shape == dW.shape
    out = np.zeros_like(dW)
    for o in range(dW.shape[0]):
        for k in range(dW.shape[1]):
            if mask[o, k]:
                out[o, k] = dW[o, k]
    return out


def flip_rate(mask_a: np.ndarray, mask_b: np.ndarray) -> float:
    a = np.ascontiguousarray(mask_a, dtype=np.uint8)
    b = np.ascontiguousarray(mask_b, dtype=np.uint8)
    assert a.shape == b.shape
    return float(_L().sbn_oracle_flip_rate(_p(a), _p(b), a.size))


def threads() -> int:
    """Threads the OpenMP loops of the oracle use (for the cpu_baseline report)."""
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
