"""The forward entry point that allocates nothing (sbn_sparse_ternary_linear_static: the library's own scratch
instead of a workspace argument), through the C ABI, against sbn_sparse_ternary_linear on the same inputs:
int8 activations, scales, int32 accumulators and Y bit for bit, and against the CPU oracle to the forward's
bar (integers exact, Y within 1e-3).  Two calls in a row on the shared scratch, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import sbn_synth
from gpu_util import DEV, assert_rel, hip_linear, hip_pack, oracle_pack, sbn

pytestmark = pytest.mark.gpu


def static_linear_raw(lib, X, packed, gamma, d_out, N, M, path, bias=None):
    """Calls the raw C symbol (no Python binding in between) on the current torch stream."""
    T, K = X.shape
    Xd = X.to(DEV)
    Y = torch.full((T, d_out), float("nan"), dtype=torch.float32, device=DEV)
    acc = torch.full((T, d_out), -7, dtype=torch.int32, device=DEV)
    xq = torch.zeros((T, K), dtype=torch.int8, device=DEV)
    sx = torch.zeros(T, dtype=torch.float32, device=DEV)
    b = None if bias is None else bias.to(DEV)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    rc = lib.sbn_sparse_ternary_linear_static(vp(Xd.data_ptr()), i64(T), i64(K), i64(d_out), ci(N), ci(M), vp(packed.data_ptr()),
                                              vp(gamma.data_ptr()), vp(b.data_ptr()) if b is not None else None,
                                              vp(Y.data_ptr()), vp(xq.data_ptr()), vp(sx.data_ptr()), vp(acc.data_ptr()), ci(path),
                                              vp(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, f"sbn_sparse_ternary_linear_static returned {rc}"
    torch.cuda.synchronize()
    return Y.cpu().numpy(), acc.cpu().numpy(), xq.cpu().numpy(), sx.cpu().numpy()


@pytest.mark.parametrize("path_name", ["SBN_PATH_SMFMAC", "SBN_PATH_GEMV", "SBN_PATH_AUTO"])
def test_static_scratch_entry_matches_workspace_entry_two_calls(path_name):
    s = sbn()
    lib = ctypes.CDLL(s.lib_path())
    lib.sbn_sparse_ternary_linear_static.restype = ctypes.c_int
    path = getattr(s, path_name)
    decode = path_name == "SBN_PATH_GEMV"
    # first a larger input, then a smaller one: the second call finds the first call's bytes in the scratch
    cases = [((16, (520, 1280)), (3, (250, 640))), ((700, (520, 1280)), (130, (300, 384)))][0 if decode else 1]
    bias = None
    for call, (tokens, shape) in enumerate(cases):
        W = sbn_synth.latent_weight(shape[0], shape[1], 3000 + call)
        X = sbn_synth.activations(tokens, shape[1], 3010 + call)
        packed, gamma = hip_pack(W, 2, 4)
        got = static_linear_raw(lib, X, packed, gamma, shape[0], 2, 4, path, bias)
        want = hip_linear(X, packed, gamma, shape[0], 2, 4, path, bias)
        for g, w, what in zip(got, want, ("Y", "acc", "xq", "sx")):
            assert np.array_equal(g, w), f"call {call}: {what} differs from the workspace entry point"
        _, ref_gamma, Weff, _ = oracle_pack(W, 2, 4)
        y, acc, xq, sx = oracle.sparse_ternary_linear(X.float().numpy(), Weff, ref_gamma)
        assert np.array_equal(got[1], acc) and np.array_equal(got[2], xq) and np.array_equal(got[3], sx)
        assert_rel(got[0], y, 1e-3, f"call {call}: Y against the oracle")


def test_static_scratch_entry_limits_and_refusals():
    s = sbn()
    W = sbn_synth.latent_weight(64, 128, 3020)
    packed, gamma = hip_pack(W, 2, 4)
    # beyond the buffer: 16 MiB hold fewer than 20000 x 1024 int8 activations
    X = torch.zeros(20000, 1024, dtype=torch.bfloat16, device=DEV)
    Y = torch.zeros(20000, 64, dtype=torch.float32, device=DEV)
    W2 = sbn_synth.latent_weight(64, 1024, 3021)
    p2, g2 = hip_pack(W2, 2, 4)
    with pytest.raises(s.SbnError) as e:
        s.sbn_sparse_ternary_linear_static(X, p2, g2, Y, 2, 4)
    assert e.value.status == s.SBN_ESIZE and "scratch" in str(e.value)
    # a path that would expand the weights into a workspace is refused
    X = sbn_synth.activations(40, 128, 3022).to(DEV)
    Y = torch.zeros(40, 64, dtype=torch.float32, device=DEV)
    with pytest.raises(s.SbnError) as e:
        s.sbn_sparse_ternary_linear_static(X, packed, gamma, Y, 2, 4, path=s.SBN_PATH_DENSE_MFMA)
    assert e.value.status == s.SBN_EUNSUPPORTED
    # the binding of the same name gives the same Y as the workspace call
    s.sbn_sparse_ternary_linear_static(X, packed, gamma, Y, 2, 4)
    torch.cuda.synchronize()
    Y1, *_ = hip_linear(X.cpu(), packed, gamma, 64, 2, 4, s.SBN_PATH_AUTO, want_acc=False)
    assert np.array_equal(Y.cpu().numpy(), Y1)
    # 1:4 at a decode size: the kernel reads that packed form as stored, so it needs no expansion region either
    p14, g14 = hip_pack(W, 1, 4)
    X = sbn_synth.activations(8, 128, 3023).to(DEV)
    Y = torch.zeros(8, 64, dtype=torch.float32, device=DEV)
    s.sbn_sparse_ternary_linear_static(X, p14, g14, Y, 1, 4)
    torch.cuda.synchronize()
    Y1, *_ = hip_linear(X.cpu(), p14, g14, 64, 1, 4, s.SBN_PATH_AUTO, want_acc=False)
    assert np.array_equal(Y.cpu().numpy(), Y1)
