"""GPU parity of the fused RMS normalisation + activation quantizer (Algorithm 1: x~ <- Q_a(Norm(x)))
against the CPU oracle: normalised bf16 activations, int8 codes and scales bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import sbn_synth
from gpu_util import DEV, assert_rel, hip_pack, oracle_pack, sbn

pytestmark = pytest.mark.gpu


def run(X, gain, eps, want_xn=True):
    s = sbn()
    T, K = X.shape
    xq = torch.full((T, K), 77, dtype=torch.int8, device=DEV)
    sx = torch.full((T,), -1.0, dtype=torch.float32, device=DEV)
    xn = torch.full((T, K), 9.0, dtype=torch.bfloat16, device=DEV) if want_xn else None
    s.sbn_rmsnorm_act_quant(X.to(DEV), xq, sx, None if gain is None else gain.to(DEV), eps, xn)
    torch.cuda.synchronize()
    return xq.cpu().numpy(), sx.cpu().numpy(), None if xn is None else xn.float().cpu().numpy()


@pytest.mark.parametrize("tokens,d_in", [(1, 128), (5, 2560), (64, 6912), (65, 2560), (300, 640), (70, 8200), (3, 16384),
                                         (130, 8192), (7, 8)])
@pytest.mark.parametrize("with_gain", [False, True])
def test_rmsnorm_act_quant_all_kernel_variants(tokens, d_in, with_gain):
    X = sbn_synth.activations(tokens, d_in, 1700 + tokens) * 2.5
    gain = (1.0 + 0.25 * torch.randn(d_in, generator=torch.Generator().manual_seed(d_in))) if with_gain else None
    xq, sx, xn = run(X, gain, 1e-6)
    r_xq, r_sx, r_xn = oracle.rmsnorm_act_quant(X.float().numpy(), None if gain is None else gain.numpy(), 1e-6)
    assert np.array_equal(xn, r_xn), f"{(xn != r_xn).sum()} normalised activations differ"
    assert np.array_equal(sx, r_sx)
    assert np.array_equal(xq, r_xq), f"{(xq != r_xq).sum()} int8 activations differ"


def test_rmsnorm_act_quant_edge_rows_and_eps():
    X = sbn_synth.adversarial_activations(8, 256, 1710)     # a zero row, ties, extremes
    for eps in (0.0, 1e-6, 0.5):
        if eps == 0.0:
            Xe = X.clone()
            Xe[1] = 1.0          # eps = 0 on an all-zero row would divide by zero; the oracle wants finite values
        else:
            Xe = X
        xq, sx, xn = run(Xe, None, eps, want_xn=(eps != 0.5))
        r_xq, r_sx, r_xn = oracle.rmsnorm_act_quant(Xe.float().numpy(), None, eps)
        assert np.array_equal(sx, r_sx) and np.array_equal(xq, r_xq)
        if xn is not None:
            assert np.array_equal(xn, r_xn)


def test_norm_then_layer_end_to_end():
    # Algorithm 1 in one piece: Norm + Q_a on the GPU, then the layer in its pre-quantized mode
    s = sbn()
    T, K, d_out = 24, 640, 200
    X = sbn_synth.activations(T, K, 1720) * 3.0
    W = sbn_synth.latent_weight(d_out, K, 1721)
    gain = 1.0 + 0.25 * torch.randn(K, generator=torch.Generator().manual_seed(5))
    packed, gamma = hip_pack(W, 2, 4)
    xq = torch.empty(T, K, dtype=torch.int8, device=DEV)
    sx = torch.empty(T, dtype=torch.float32, device=DEV)
    s.sbn_rmsnorm_act_quant(X.to(DEV), xq, sx, gain.to(DEV), 1e-5)
    Y = torch.full((T, d_out), float("nan"), dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, d_out, K, 2, 4))
    s.sbn_sparse_ternary_linear(None, packed, gamma, Y, 2, 4, ws, xq_out=xq, sx_out=sx)
    torch.cuda.synchronize()
    _, g, Weff, _ = oracle_pack(W, 2, 4)
    r_xq, r_sx, _ = oracle.rmsnorm_act_quant(X.float().numpy(), gain.numpy(), 1e-5)
    r_y = oracle.rescale(oracle.acc(Weff, r_xq), g, r_sx, None)
    assert_rel(Y.cpu().numpy(), r_y, 1e-3, "Y")


def test_rmsnorm_act_quant_full_size_as_timed():
    # the shape and launch configuration the benchmark times: 4096 tokens x 2560, gain, eps 1e-6
    X = sbn_synth.activations(4096, 2560, sbn_synth.seed_for(3, 10))
    gain = 1.0 + 0.25 * torch.randn(2560, generator=torch.Generator().manual_seed(3))
    xq, sx, xn = run(X, gain, 1e-6)
    r_xq, r_sx, r_xn = oracle.rmsnorm_act_quant(X.float().numpy(), gain.numpy(), 1e-6)
    assert np.array_equal(xn, r_xn) and np.array_equal(sx, r_sx) and np.array_equal(xq, r_xq)
