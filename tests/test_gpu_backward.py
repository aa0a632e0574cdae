"""GPU parity of the backward products against the CPU oracle (Section 2.3, dual straight-through
estimator): dX through the transposed ternary weights, dense unmasked dW; bf16 outputs within
2e-2 of the fp64 oracle, measured against max(|ref|, rms(ref)) because the sums cancel."""
import numpy as np
import pytest
import torch

import oracle
import sbn_synth
from gpu_util import DEV, assert_rel_rms, hip_pack, oracle_pack, sbn

pytestmark = pytest.mark.gpu
BWD_TOL = 2e-2


def hip_forward_backward(W, X, dY, N, M, want_dx=True, want_dw=True, accumulate_into=None, mask_dw=False):
    s = sbn()
    d_out, d_in = W.shape
    T = X.shape[0]
    packed, gamma = hip_pack(W, N, M)
    Xd, dYd = X.to(DEV), dY.to(DEV)
    Y = torch.empty(T, d_out, dtype=torch.float32, device=DEV)
    xq = torch.empty(T, d_in, dtype=torch.int8, device=DEV)
    sx = torch.empty(T, dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, d_out, d_in, N, M))
    s.sbn_sparse_ternary_linear(Xd, packed, gamma, Y, N, M, ws, xq_out=xq, sx_out=sx)
    dX = torch.full((T, d_in), float("nan"), dtype=torch.bfloat16, device=DEV) if want_dx else None
    if accumulate_into is not None:
        dW = accumulate_into.to(DEV)
    else:
        dW = torch.full((d_out, d_in), float("nan"), dtype=torch.bfloat16, device=DEV) if want_dw else None
    wsb = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, T, d_out, d_in, N, M))
    s.sbn_sparse_ternary_linear_backward(dYd, packed, gamma, xq, sx, N, M, wsb, d_in, dX=dX, dW=dW,
                                         accumulate=accumulate_into is not None, mask_dw=mask_dw)
    torch.cuda.synchronize()
    return (None if dX is None else dX.float().cpu().numpy(), None if dW is None else dW.float().cpu().numpy(),
            xq.cpu().numpy(), sx.cpu().numpy())


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8)])
@pytest.mark.parametrize("tokens,shape", [(16, (256, 256)), (200, (136, 384)), (77, (520, 128)), (50, (104, 136))])
def test_backward_small(N, M, tokens, shape):
    W = sbn_synth.latent_weight(shape[0], shape[1], 900 + shape[0])
    X = sbn_synth.activations(tokens, shape[1], 910 + tokens)
    dY = sbn_synth.grad_output(tokens, shape[0], 920)
    dX, dW, xq, sx = hip_forward_backward(W, X, dY, N, M)
    _, gamma, Weff, mask = oracle_pack(W, N, M)
    r_dx = oracle.backward_dx(dY.float().numpy(), Weff, gamma)
    r_dw = oracle.backward_dw(dY.float().numpy(), xq, sx)
    assert_rel_rms(dX, r_dx, BWD_TOL, "dX")
    assert_rel_rms(dW, r_dw, BWD_TOL, "dW")
    assert (dW[mask == 0] != 0).mean() > 0.95        # masked-out weights receive gradient


def test_backward_accumulate_and_partial_outputs():
    W = sbn_synth.latent_weight(256, 256, 930)
    X = sbn_synth.activations(64, 256, 931)
    dY = sbn_synth.grad_output(64, 256, 932)
    base = (torch.randn(256, 256, generator=torch.Generator().manual_seed(5)) * 0.1).to(torch.bfloat16)
    dX, dW, xq, sx = hip_forward_backward(W, X, dY, 2, 4, want_dx=False, accumulate_into=base.clone())
    assert dX is None
    r_dw = oracle.backward_dw(dY.float().numpy(), xq, sx) + base.float().numpy().astype(np.float64)
    assert_rel_rms(dW, r_dw, BWD_TOL, "dW accumulate")
    dX, dW, *_ = hip_forward_backward(W, X, dY, 2, 4, want_dw=False)
    assert dW is None and np.isfinite(dX).all()


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8), (4, 4)])
@pytest.mark.parametrize("tokens,shape", [(64, (256, 256)), (77, (104, 136)), (130, (520, 392))])
def test_backward_gradient_masked_variant(N, M, tokens, shape):
    # ablation study, "gradient masking": dW = M (.) dense dW; entries outside the mask are exactly zero
    # (or, when accumulating, exactly what the buffer held), dX is unaffected
    W = sbn_synth.latent_weight(shape[0], shape[1], 940 + shape[0])
    X = sbn_synth.activations(tokens, shape[1], 941 + tokens)
    dY = sbn_synth.grad_output(tokens, shape[0], 942)
    _, gamma, Weff, mask = oracle_pack(W, N, M)
    dX, dW, xq, sx = hip_forward_backward(W, X, dY, N, M, mask_dw=True)
    r_dw = oracle.backward_dw_gradient_masked(dY.float().numpy(), xq, sx, mask)
    assert (dW[mask == 0] == 0).all()
    assert_rel_rms(dW, r_dw, BWD_TOL, "masked dW")
    assert_rel_rms(dX, oracle.backward_dx(dY.float().numpy(), Weff, gamma), BWD_TOL, "dX")
    base = (torch.randn(*shape, generator=torch.Generator().manual_seed(6)) * 0.1).to(torch.bfloat16)
    _, dWa, *_ = hip_forward_backward(W, X, dY, N, M, want_dx=False, accumulate_into=base.clone(), mask_dw=True)
    basef = base.float().numpy()
    assert np.array_equal(dWa[mask == 0], basef[mask == 0])
    assert_rel_rms(dWa, r_dw + basef.astype(np.float64), BWD_TOL, "masked dW accumulate")


def test_config5_training_step_block_matrices():
    # configs[4]: batch 8 x seq 2048 = 16384 tokens through the block's three matrix shapes.
    # dX is checked on sampled token rows, dW on sampled weight rows (each entry an exact fp64 sum).
    rng = np.random.default_rng(5)
    T = 16384
    for d_out, d_in in ((2560, 2560), (6912, 2560), (2560, 6912)):
        W = sbn_synth.latent_weight(d_out, d_in, sbn_synth.seed_for(5, d_out + 1))
        X = sbn_synth.activations(T, d_in, sbn_synth.seed_for(5, d_in))
        dY = sbn_synth.grad_output(T, d_out, sbn_synth.seed_for(5, 7))
        dX, dW, xq, sx = hip_forward_backward(W, X, dY, 2, 4)
        _, gamma, Weff, _ = oracle_pack(W, 2, 4)
        trow = np.unique(np.concatenate([[0, T - 1], rng.choice(T, 24, replace=False)]))
        r_dx = oracle.backward_dx(dY[trow].float().numpy(), Weff, gamma)
        assert_rel_rms(dX[trow], r_dx, BWD_TOL, f"dX {d_out}x{d_in}")
        orow = np.unique(np.concatenate([[0, d_out - 1], rng.choice(d_out, 6, replace=False)]))
        r_xq, r_sx = oracle.act_quant(X.float().numpy())
        assert np.array_equal(r_xq, xq) and np.array_equal(r_sx, sx)
        r_dw = oracle.backward_dw(np.ascontiguousarray(dY[:, orow].float().numpy()), r_xq, r_sx)
        assert_rel_rms(dW[orow], r_dw, BWD_TOL, f"dW {d_out}x{d_in}")
