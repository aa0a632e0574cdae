"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding and the CPU oracle
on the same seeded tensors."""
import numpy as np
import torch

import oracle

DEV = "cuda"


def sbn():
    import paper_2603_05168_amd as m
    return m


def hip_pack(W: torch.Tensor, N: int, M: int):
    """W on the host (bf16 or fp32) -> (packed uint8 device tensor, gamma device tensor)."""
    s = sbn()
    Wd = W.to(DEV)
    d_out, d_in = W.shape
    packed = torch.full((s.sbn_packed_bytes(d_out, d_in, N, M),), 0xAA, dtype=torch.uint8, device=DEV)
    gamma = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, 1, d_out, d_in, N, M))
    s.sbn_quantize_mask_pack(Wd, N, M, packed, gamma, ws)
    torch.cuda.synchronize()
    return packed, gamma


def oracle_pack(W: torch.Tensor, N: int, M: int):
    Wf = W.float().numpy()
    Weff, mask, gamma = oracle.quantize_mask(Wf, N, M)
    return oracle.pack(Weff, mask, N, M), gamma, Weff, mask


def hip_linear(X: torch.Tensor, packed, gamma, d_out: int, N: int, M: int, path: int, bias=None, want_acc=True):
    s = sbn()
    Xd = X.to(DEV)
    T, K = X.shape
    Y = torch.full((T, d_out), float("nan"), dtype=torch.float32, device=DEV)
    acc = torch.full((T, d_out), -7, dtype=torch.int32, device=DEV)
    xq = torch.zeros((T, K), dtype=torch.int8, device=DEV)
    sx = torch.zeros(T, dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, d_out, K, N, M))
    s.sbn_sparse_ternary_linear(Xd, packed, gamma, Y, N, M, ws, bias=None if bias is None else bias.to(DEV),
                                xq_out=xq, sx_out=sx, acc_out=acc if want_acc else None, path=path)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), acc.cpu().numpy(), xq.cpu().numpy(), sx.cpu().numpy()


def assert_rel(got: np.ndarray, ref: np.ndarray, tol: float, what: str):
    """Elementwise |got - ref| <= tol * |ref| (the forward tolerance: the accumulator is exact, so
    ref == 0 implies got == 0)."""
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > tol * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond {tol} relative; worst {err.max()}"


def assert_rel_rms(got: np.ndarray, ref: np.ndarray, tol: float, what: str):
    """|got - ref| <= tol * max(|ref|, rms(ref)): the backward tolerance (cancelling sums)."""
    err = np.abs(got.astype(np.float64) - ref)
    rms = np.sqrt(np.mean(ref ** 2))
    bad = err > tol * np.maximum(np.abs(ref), rms)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond {tol}; worst {err.max()} rms {rms}"
