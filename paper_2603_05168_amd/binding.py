"""ctypes binding of libsbn.so: argument marshalling only (see include/sbn.h for semantics).

Every function takes torch tensors (or raw integers) for device buffers, passes their data
pointers and sizes straight to the C ABI on the current torch stream, and raises SbnError on a
non-zero status.  No step of the method runs here.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsbn.so")

SBN_OK, SBN_EINVAL, SBN_EUNSUPPORTED, SBN_ESIZE, SBN_EALIGN, SBN_EHIP = 0, -1, -2, -3, -4, -5
SBN_F32, SBN_BF16 = 0, 1
SBN_PATH_AUTO, SBN_PATH_GEMV, SBN_PATH_SMFMAC, SBN_PATH_DENSE_MFMA, SBN_PATH_GENERIC = 0, 1, 2, 3, 4
SBN_OP_QUANTIZE_MASK_PACK, SBN_OP_LINEAR, SBN_OP_BACKWARD, SBN_OP_MASK_FLIPS = 0, 1, 2, 3

_STATUS_NAMES = {0: "SBN_OK", -1: "SBN_EINVAL", -2: "SBN_EUNSUPPORTED", -3: "SBN_ESIZE", -4: "SBN_EALIGN", -5: "SBN_EHIP"}


class SbnError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: {_STATUS_NAMES.get(status, status)} {detail}".strip())


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc, gfx950).  There is no fallback path.")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, cint, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    pp = ctypes.POINTER(ctypes.c_void_p)
    pi64 = ctypes.POINTER(ctypes.c_int64)
    lib.sbn_last_error.restype = ctypes.c_char_p
    lib.sbn_last_error.argtypes = []
    lib.sbn_packed_bytes.restype = cint
    lib.sbn_packed_bytes.argtypes = [i64, i64, cint, cint, ctypes.POINTER(sz)]
    lib.sbn_workspace_bytes.restype = cint
    lib.sbn_workspace_bytes.argtypes = [cint, i64, i64, i64, cint, cint, ctypes.POINTER(sz)]
    lib.sbn_quantize_mask_pack.restype = cint
    lib.sbn_quantize_mask_pack.argtypes = [vp, cint, i64, i64, i64, cint, cint, vp, vp, vp, sz, vp]
    lib.sbn_quantize_mask_pack_batched.restype = cint
    lib.sbn_quantize_mask_pack_batched.argtypes = [cint, pp, cint, pi64, pi64, cint, cint, pp, pp, vp, sz, vp]
    lib.sbn_quantize_mask_pack_flips_batched.restype = cint
    lib.sbn_quantize_mask_pack_flips_batched.argtypes = [cint, pp, cint, pi64, pi64, cint, cint, pp, pp, vp, vp, sz, vp]
    lib.sbn_act_quant.restype = cint
    lib.sbn_act_quant.argtypes = [vp, i64, i64, vp, vp, vp]
    lib.sbn_sparse_ternary_linear.restype = cint
    lib.sbn_sparse_ternary_linear.argtypes = [vp, i64, i64, i64, cint, cint, vp, vp, vp, vp, vp, vp, vp, cint, vp, sz, vp]
    lib.sbn_sparse_ternary_linear_static.restype = cint
    lib.sbn_sparse_ternary_linear_static.argtypes = [vp, i64, i64, i64, cint, cint, vp, vp, vp, vp, vp, vp, vp, cint, vp]
    lib.sbn_sparse_ternary_linear_grouped.restype = cint
    lib.sbn_sparse_ternary_linear_grouped.argtypes = [cint, pp, pi64, pi64, pi64, cint, cint, pp, pp, pp, cint, vp, sz, vp]
    lib.sbn_sparse_ternary_linear_backward.restype = cint
    lib.sbn_sparse_ternary_linear_backward.argtypes = [vp, i64, i64, i64, cint, cint, vp, vp, vp, vp, vp, vp, cint, vp, sz, vp]
    lib.sbn_sparse_ternary_linear_backward_grouped.restype = cint
    lib.sbn_sparse_ternary_linear_backward_grouped.argtypes = [cint, pp, pi64, pi64, pi64, cint, cint, pp, pp, pp, pp, pp, pp, cint,
                                                               vp, sz, vp]
    lib.sbn_dense_ternary_linear.restype = cint
    lib.sbn_dense_ternary_linear.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    lib.sbn_unpack.restype = cint
    lib.sbn_unpack.argtypes = [vp, i64, i64, cint, cint, vp, vp, vp]
    lib.sbn_convert_packed.restype = cint
    lib.sbn_convert_packed.argtypes = [vp, i64, i64, cint, cint, cint, cint, vp, vp]
    lib.sbn_rmsnorm_act_quant.restype = cint
    lib.sbn_rmsnorm_act_quant.argtypes = [vp, i64, i64, vp, ctypes.c_float, vp, vp, vp, vp]
    lib.sbn_test_set_spin_limits.restype = None
    lib.sbn_test_set_spin_limits.argtypes = [cint, cint]
    lib.sbn_mask_flips.restype = cint
    lib.sbn_mask_flips.argtypes = [vp, vp, i64, i64, cint, cint, vp, vp, sz, vp]
    return lib


_lib = _load()


def lib_path() -> str:
    return _LIB_PATH


def _ptr(t):
    """Device (or host) address of a tensor, an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None


def _check(status: int, where: str):
    if status != SBN_OK:
        detail = _lib.sbn_last_error().decode() if status == SBN_EHIP else ""
        raise SbnError(status, where, detail)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SBN_BF16
    if t.dtype == torch.float32:
        return SBN_F32
    raise TypeError("latent weights must be bf16 or fp32")


def sbn_last_error() -> str:
    return _lib.sbn_last_error().decode()


def sbn_packed_bytes(d_out: int, d_in: int, N: int, M: int) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib.sbn_packed_bytes(d_out, d_in, N, M, ctypes.byref(out)), "sbn_packed_bytes")
    return out.value


def sbn_workspace_bytes(op: int, tokens: int, d_out: int, d_in: int, N: int, M: int) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib.sbn_workspace_bytes(op, tokens, d_out, d_in, N, M, ctypes.byref(out)), "sbn_workspace_bytes")
    return out.value


def sbn_quantize_mask_pack(W_latent, N: int, M: int, packed, gamma, workspace, ld_w: int | None = None):
    d_out, d_in = W_latent.shape
    ld = W_latent.stride(0) if ld_w is None else ld_w
    _check(_lib.sbn_quantize_mask_pack(_ptr(W_latent), _dtype_code(W_latent), d_out, d_in, ld, N, M, _ptr(packed),
                                       _ptr(gamma), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _stream()), "sbn_quantize_mask_pack")


def _ptr_array(tensors):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else (t.data_ptr() if not isinstance(t, int) else t)
    return arr


def _i64_array(values):
    arr = (ctypes.c_int64 * len(values))()
    for i, v in enumerate(values):
        arr[i] = int(v)
    return arr


class PackBatch:
    """Host-side argument arrays of sbn_quantize_mask_pack_batched, marshalled once and reusable."""

    def __init__(self, W_list, N, M, packed_list, gamma_list, workspace, flips_out=None):
        self.flips_out = flips_out   # int64 device tensor of len(W_list): pack in place over the old forms and count flips
        self.count = len(W_list)
        self.dtype = _dtype_code(W_list[0])
        self.W = _ptr_array(W_list)
        self.d_out = _i64_array([w.shape[0] for w in W_list])
        self.d_in = _i64_array([w.shape[1] for w in W_list])
        self.packed = _ptr_array(packed_list)
        self.gamma = _ptr_array(gamma_list)
        self.N, self.M = N, M
        self.workspace = workspace
        self.keep = (W_list, packed_list, gamma_list)

    def run(self):
        ws = self.workspace
        if self.flips_out is not None:
            _check(_lib.sbn_quantize_mask_pack_flips_batched(self.count, self.W, self.dtype, self.d_out, self.d_in, self.N,
                                                             self.M, self.packed, self.gamma, _ptr(self.flips_out), _ptr(ws),
                                                             ws.numel() * ws.element_size(), _stream()),
                   "sbn_quantize_mask_pack_flips_batched")
            return
        _check(_lib.sbn_quantize_mask_pack_batched(self.count, self.W, self.dtype, self.d_out, self.d_in, self.N,
                                                   self.M, self.packed, self.gamma, _ptr(ws),
                                                   ws.numel() * ws.element_size(), _stream()),
               "sbn_quantize_mask_pack_batched")


def sbn_quantize_mask_pack_batched(W_list, N: int, M: int, packed_list, gamma_list, workspace):
    PackBatch(W_list, N, M, packed_list, gamma_list, workspace).run()


def sbn_quantize_mask_pack_flips_batched(W_list, N: int, M: int, packed_list, gamma_list, flips_out, workspace):
    """Packs in place over the previous packed forms; flips_out (int64 device tensor, one per matrix) gets the mask flips."""
    PackBatch(W_list, N, M, packed_list, gamma_list, workspace, flips_out).run()


def sbn_act_quant(X, xq, sx):
    tokens, d_in = X.shape
    if X.dtype != torch.bfloat16:
        raise TypeError("X must be bf16")
    _check(_lib.sbn_act_quant(_ptr(X), tokens, d_in, _ptr(xq), _ptr(sx), _stream()), "sbn_act_quant")


def sbn_sparse_ternary_linear(X, packed, gamma, Y, N: int, M: int, workspace, bias=None, xq_out=None, sx_out=None,
                              acc_out=None, path: int = SBN_PATH_AUTO):
    """X = None runs on activations already quantized into xq_out / sx_out (then inputs)."""
    tokens, d_in = X.shape if X is not None else xq_out.shape
    d_out = Y.shape[1]
    if (X is not None and X.dtype != torch.bfloat16) or Y.dtype != torch.float32:
        raise TypeError("X must be bf16 and Y fp32")
    _check(_lib.sbn_sparse_ternary_linear(_ptr(X), tokens, d_in, d_out, N, M, _ptr(packed), _ptr(gamma), _ptr(bias),
                                          _ptr(Y), _ptr(xq_out), _ptr(sx_out), _ptr(acc_out), path, _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()),
           "sbn_sparse_ternary_linear")


SBN_STATIC_SCRATCH_MIB = 16


def sbn_sparse_ternary_linear_static(X, packed, gamma, Y, N: int, M: int, bias=None, xq_out=None, sx_out=None, acc_out=None,
                                     path: int = SBN_PATH_AUTO):
    """sbn_sparse_ternary_linear on the library's own scratch: no workspace argument, nothing allocated."""
    tokens, d_in = X.shape if X is not None else xq_out.shape
    d_out = Y.shape[1]
    if (X is not None and X.dtype != torch.bfloat16) or Y.dtype != torch.float32:
        raise TypeError("X must be bf16 and Y fp32")
    status = _lib.sbn_sparse_ternary_linear_static(_ptr(X), tokens, d_in, d_out, N, M, _ptr(packed), _ptr(gamma), _ptr(bias),
                                                   _ptr(Y), _ptr(xq_out), _ptr(sx_out), _ptr(acc_out), path, _stream())
    if status != SBN_OK:
        raise SbnError(status, "sbn_sparse_ternary_linear_static", _lib.sbn_last_error().decode() if status in (SBN_EHIP, SBN_ESIZE) else "")


class LinearGroup:
    """Host-side argument arrays of sbn_sparse_ternary_linear_grouped, marshalled once and reusable."""

    def __init__(self, X_list, packed_list, gamma_list, Y_list, N, M, workspace, path=SBN_PATH_AUTO):
        self.count = len(X_list)
        self.X = _ptr_array(X_list)
        self.tokens = _i64_array([x.shape[0] for x in X_list])
        self.d_in = _i64_array([x.shape[1] for x in X_list])
        self.d_out = _i64_array([y.shape[1] for y in Y_list])
        self.packed = _ptr_array(packed_list)
        self.gamma = _ptr_array(gamma_list)
        self.Y = _ptr_array(Y_list)
        self.N, self.M, self.path, self.workspace = N, M, path, workspace
        self.keep = (X_list, packed_list, gamma_list, Y_list)

    def run(self):
        ws = self.workspace
        _check(_lib.sbn_sparse_ternary_linear_grouped(self.count, self.X, self.tokens, self.d_in, self.d_out, self.N,
                                                      self.M, self.packed, self.gamma, self.Y, self.path, _ptr(ws),
                                                      ws.numel() * ws.element_size(), _stream()),
               "sbn_sparse_ternary_linear_grouped")


def sbn_sparse_ternary_linear_grouped(X_list, packed_list, gamma_list, Y_list, N, M, workspace, path=SBN_PATH_AUTO):
    LinearGroup(X_list, packed_list, gamma_list, Y_list, N, M, workspace, path).run()


SBN_BWD_ACCUMULATE, SBN_BWD_MASK_DW = 1, 2


def sbn_sparse_ternary_linear_backward(dY, packed, gamma, xq, sx, N: int, M: int, workspace, d_in: int, dX=None, dW=None,
                                       accumulate: bool = False, mask_dw: bool = False):
    tokens, d_out = dY.shape
    if dY.dtype != torch.bfloat16:
        raise TypeError("dY must be bf16")
    _check(_lib.sbn_sparse_ternary_linear_backward(_ptr(dY), tokens, d_in, d_out, N, M, _ptr(packed), _ptr(gamma),
                                                   _ptr(xq), _ptr(sx), _ptr(dX), _ptr(dW),
                                                   (SBN_BWD_ACCUMULATE if accumulate else 0) | (SBN_BWD_MASK_DW if mask_dw else 0),
                                                   _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                   _stream()), "sbn_sparse_ternary_linear_backward")


class BackwardGroup:
    """Host-side argument arrays of sbn_sparse_ternary_linear_backward_grouped, marshalled once and reusable.
    Lists hold one entry per layer; entries of dX_list / dW_list may be None."""

    def __init__(self, dY_list, packed_list, gamma_list, xq_list, sx_list, N, M, workspace, d_in_list, dX_list, dW_list,
                 accumulate=False, mask_dw=False):
        for dY in dY_list:
            if dY.dtype != torch.bfloat16:
                raise TypeError("dY must be bf16")
        self.count = len(dY_list)
        self.dY = _ptr_array(dY_list)
        self.tokens = _i64_array([d.shape[0] for d in dY_list])
        self.d_out = _i64_array([d.shape[1] for d in dY_list])
        self.d_in = _i64_array(list(d_in_list))
        self.packed, self.gamma = _ptr_array(packed_list), _ptr_array(gamma_list)
        self.xq, self.sx = _ptr_array(xq_list), _ptr_array(sx_list)
        self.dX, self.dW = _ptr_array(dX_list), _ptr_array(dW_list)
        self.flags = (SBN_BWD_ACCUMULATE if accumulate else 0) | (SBN_BWD_MASK_DW if mask_dw else 0)
        self.N, self.M, self.workspace = N, M, workspace
        self.keep = (dY_list, packed_list, gamma_list, xq_list, sx_list, dX_list, dW_list)

    def run(self):
        ws = self.workspace
        _check(_lib.sbn_sparse_ternary_linear_backward_grouped(self.count, self.dY, self.tokens, self.d_in, self.d_out, self.N,
                                                               self.M, self.packed, self.gamma, self.xq, self.sx, self.dX,
                                                               self.dW, self.flags, _ptr(ws), ws.numel() * ws.element_size(),
                                                               _stream()),
               "sbn_sparse_ternary_linear_backward_grouped")


def sbn_sparse_ternary_linear_backward_grouped(dY_list, packed_list, gamma_list, xq_list, sx_list, N, M, workspace, d_in_list,
                                               dX_list, dW_list, accumulate=False, mask_dw=False):
    BackwardGroup(dY_list, packed_list, gamma_list, xq_list, sx_list, N, M, workspace, d_in_list, dX_list, dW_list, accumulate,
                  mask_dw).run()


def sbn_unpack(packed, d_out: int, d_in: int, N: int, M: int, W_eff=None, mask=None):
    _check(_lib.sbn_unpack(_ptr(packed), d_out, d_in, N, M, _ptr(W_eff), _ptr(mask), _stream()), "sbn_unpack")


def sbn_rmsnorm_act_quant(X, xq, sx, gain=None, eps: float = 1e-6, xn_out=None):
    """x~, s_x = Q_a(Norm(x)); X bf16 [tokens, d_in]; gain fp32 [d_in] or None; xn_out bf16 or None."""
    tokens, d_in = X.shape
    _check(_lib.sbn_rmsnorm_act_quant(_ptr(X), tokens, d_in, _ptr(gain), eps, _ptr(xq), _ptr(sx), _ptr(xn_out), _stream()),
           "sbn_rmsnorm_act_quant")


def sbn_convert_packed(packed, d_out: int, d_in: int, N: int, M: int, to_N: int, to_M: int, out):
    """Rewrite a packed N:M matrix into the packed form of to_N:to_M (2:4 or M:M) for decode."""
    _check(_lib.sbn_convert_packed(_ptr(packed), d_out, d_in, N, M, to_N, to_M, _ptr(out), _stream()), "sbn_convert_packed")


def sbn_dense_ternary_linear(xq, sx, W_eff, gamma, Y, bias=None, acc_out=None):
    """The dense comparison kernel alone: Y = (xq @ W_eff^T) * gamma / s_x (+ bias) with W_eff int8 [d_out, d_in]."""
    tokens, d_in = xq.shape
    _check(_lib.sbn_dense_ternary_linear(_ptr(xq), _ptr(sx), tokens, d_in, W_eff.shape[0], _ptr(W_eff), _ptr(gamma), _ptr(bias),
                                         _ptr(Y), _ptr(acc_out), _stream()), "sbn_dense_ternary_linear")


SBN_SPIN_DEFAULT = -2 ** 31


def sbn_test_set_spin_limits(gemv_polls: int = SBN_SPIN_DEFAULT, pack_polls: int = SBN_SPIN_DEFAULT):
    """Test hook: polls of the two bounded inter-block waits (negative: never wait; SBN_SPIN_DEFAULT restores)."""
    _lib.sbn_test_set_spin_limits(gemv_polls, pack_polls)


def sbn_mask_flips(packed_a, packed_b, d_out: int, d_in: int, N: int, M: int, flips_out, workspace):
    """flips_out: int64 device tensor of one element (the count is non-negative and below 2**63)."""
    _check(_lib.sbn_mask_flips(_ptr(packed_a), _ptr(packed_b), d_out, d_in, N, M, _ptr(flips_out), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream()), "sbn_mask_flips")


def new_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch of at least nbytes (torch's allocator returns 512-byte aligned blocks)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
