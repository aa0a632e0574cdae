"""Pins for the activation quantizer, the integer accumulation, the rescale and the backward
products of the CPU oracle.

Pins: numpy's IEEE fp32 arithmetic and int64 matmul, a brute-force fp64 product of the de-quantized
operands, the N = M reduction to the plain BitLinear layer, and the layer written as an fp64 graph
(Sections 2.1 - 2.3, both quantizers straight-through) whose gradients torch autograd derives.
"""
import numpy as np
import pytest
import torch

import oracle
import sbn_synth


def gaussian(shape, seed, sigma=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * sigma).astype(np.float32)


# ----------------------------------------------------------------------------- activation quantizer
def test_act_quant_against_numpy_fp32():
    X = sbn_synth.activations(64, 384, 1).float().numpy()
    xq, sx = oracle.act_quant(X)
    amax = np.maximum(np.abs(X).max(axis=1), np.float32(1e-5))
    s = (np.float32(127.0) / amax).astype(np.float32)
    prod = X * s[:, None]
    assert prod.dtype == np.float32
    assert np.array_equal(sx, s)
    assert np.array_equal(xq, np.clip(np.rint(prod), -128, 127).astype(np.int8))
    assert (np.abs(xq.astype(np.int32)).max(axis=1) == 127).all()     # every non-zero row reaches 127


def test_act_quant_edge_rows():
    X = sbn_synth.adversarial_activations(8, 256, 2).float().numpy()
    xq, sx = oracle.act_quant(X)
    assert (xq[1] == 0).all() and sx[1] == np.float32(127.0) / np.float32(1e-5)   # zero row
    assert sx[2] == np.float32(1.0)                                               # amax = 127
    assert np.array_equal(xq[2], np.rint(X[2]).astype(np.int8))                   # .5 ties go to even
    assert (np.rint(X[2]) != np.floor(X[2] + 0.5)).any()                          # the ties are really there
    # power-of-two scaling leaves the integers unchanged
    xq4, sx4 = oracle.act_quant(X * np.float32(4.0))
    assert np.array_equal(xq4, xq) and np.array_equal(sx4[[0, 2, 3]], (sx / np.float32(4.0))[[0, 2, 3]])


# ----------------------------------------------------------------------------- accumulate and rescale
@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8), (4, 4)])
def test_acc_is_integer_matmul_and_linear(N, M):
    W = gaussian((96, 256), 3, 0.02)
    Weff, _, _ = oracle.quantize_mask(W, N, M)
    rng = np.random.default_rng(4)
    xa = rng.integers(-128, 128, size=(12, 256)).astype(np.int8)
    xb = rng.integers(-60, 60, size=(12, 256)).astype(np.int8)
    a = oracle.acc(Weff, xa)
    assert np.array_equal(a, (xa.astype(np.int64) @ Weff.astype(np.int64).T).astype(np.int32))
    xs = (xa.astype(np.int32) // 2 + xb.astype(np.int32)).astype(np.int8)
    assert np.array_equal(oracle.acc(Weff, xs),
                          oracle.acc(Weff, (xa.astype(np.int32) // 2).astype(np.int8)) + oracle.acc(Weff, xb))


def test_forward_matches_fp64_product_of_dequantized_operands():
    W = sbn_synth.latent_weight(160, 256, 5).float().numpy()
    X = sbn_synth.activations(24, 256, 6).float().numpy()
    bias = gaussian((160,), 7, 0.1)
    Weff, _, gamma = oracle.quantize_mask(W, 2, 4)
    y, acc, xq, sx = oracle.sparse_ternary_linear(X, Weff, gamma, bias)
    xhat = xq.astype(np.float64) / sx.astype(np.float64)[:, None]
    ref = xhat @ (np.float64(gamma) * Weff.astype(np.float64)).T + bias.astype(np.float64)
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    assert np.abs(acc).max() <= 128 * 256 * 2 // 4


def test_n_equals_m_is_plain_bitlinear():
    # Section 2.1: y ~ gamma * matmul(W_q, x~) / s_x with no mask at all
    W = sbn_synth.latent_weight(64, 128, 8).float().numpy()
    X = sbn_synth.activations(8, 128, 9).float().numpy()
    Weff, _, gamma = oracle.quantize_mask(W, 8, 8)
    y, *_ = oracle.sparse_ternary_linear(X, Weff, gamma)
    g = np.float32(np.abs(W).astype(np.float64).mean())
    Wq = np.clip(np.rint(W / g), -1, 1).astype(np.float64)
    s = np.float32(127.0) / np.abs(X).max(axis=1)
    Xq = np.clip(np.rint(X * s[:, None]), -128, 127).astype(np.float64)
    ref = (Xq @ Wq.T) * np.float64(g) / s.astype(np.float64)[:, None]
    assert np.allclose(y, ref, rtol=1e-12, atol=0)


# ----------------------------------------------------------------------------- the layer as a differentiable graph
def _topn_mask(latent: np.ndarray, N: int, M: int) -> np.ndarray:
    """Section 2.2 mask: per group of M the N largest |w| of the latent weights, ties to the lower index;
    written with a stable sort (the oracle counts ranks instead)."""
    rows, cols = latent.shape
    mag = np.abs(latent).reshape(rows, cols // M, M)
    winners = np.argsort(-mag, axis=2, kind="stable")[:, :, :N]
    keep = np.zeros(mag.shape, dtype=np.float64)
    np.put_along_axis(keep, winners, 1.0, axis=2)
    return keep.reshape(rows, cols)


def _layer_graph(tokens_in: torch.Tensor, latent: torch.Tensor, N: int, M: int) -> torch.Tensor:
    """The layer of Sections 2.1 - 2.3 as an fp64 graph whose gradients an autograd engine derives:
    both quantizers contribute their VALUE but pass gradients through unchanged (value = input + constant),
    and the mask enters the value of the weight only, so the latent weight receives the dense gradient."""
    with torch.no_grad():
        t32 = tokens_in.float()
        peak = t32.abs().amax(dim=1, keepdim=True).clamp_min(1e-5)
        to_int = torch.full_like(peak, 127.0) / peak                         # IEEE fp32 division, per token
        levels = torch.clamp(torch.round(t32 * to_int), -128, 127)
        fake_quant_tokens = levels.double() / to_int.double()
        l32 = latent.float()
        absmean = l32.abs().double().mean().float().clamp_min(1e-5)
        ternary = torch.clamp(torch.round(l32 / absmean), -1, 1).double()
        effective = ternary * torch.from_numpy(_topn_mask(l32.numpy(), N, M)) * absmean.double()
    tokens_ste = tokens_in + (fake_quant_tokens - tokens_in).detach()
    weight_ste = latent + (effective - latent).detach()
    return tokens_ste @ weight_ste.t()


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8)])
def test_forward_backward_against_autograd_graph(N, M):
    W = sbn_synth.latent_weight(96, 256, 10 + N).float()
    X = sbn_synth.activations(32, 256, 20 + M).float()
    dY = sbn_synth.grad_output(32, 96, 30).float()
    latent = W.double().requires_grad_(True)
    tokens_in = X.double().requires_grad_(True)
    out = _layer_graph(tokens_in, latent, N, M)
    out.backward(dY.double())

    Weff, mask, gamma = oracle.quantize_mask(W.numpy(), N, M)
    y_o, _, xq, sx = oracle.sparse_ternary_linear(X.numpy(), Weff, gamma)
    dX = oracle.backward_dx(dY.numpy(), Weff, gamma)
    dW = oracle.backward_dw(dY.numpy(), xq, sx)

    def close(a, b, tol):
        scale = np.sqrt(np.mean(b ** 2))
        return np.abs(a - b).max() <= tol * scale

    # both sides are fp64 products of the same de-quantized operands: only the summation order differs
    assert close(y_o, out.detach().numpy(), 1e-12)
    assert close(dX, tokens_in.grad.numpy(), 1e-12)
    assert close(dW, latent.grad.numpy(), 1e-12)
    # dense gradient: masked-out weights receive gradient too
    assert (np.abs(dW[mask == 0]) > 0).mean() > 0.99


def test_dw_does_not_depend_on_weights_or_mask():
    X = sbn_synth.activations(16, 128, 40).float().numpy()
    dY = sbn_synth.grad_output(16, 32, 41).float().numpy()
    xq, sx = oracle.act_quant(X)
    dW = oracle.backward_dw(dY, xq, sx)
    ref = dY.astype(np.float64).T @ (xq.astype(np.float64) / sx.astype(np.float64)[:, None])
    assert np.allclose(dW, ref, rtol=1e-12, atol=1e-15)


def test_dx_brute_force():
    W = sbn_synth.latent_weight(48, 128, 42).float().numpy()
    dY = sbn_synth.grad_output(8, 48, 43).float().numpy()
    Weff, _, gamma = oracle.quantize_mask(W, 2, 4)
    dX = oracle.backward_dx(dY, Weff, gamma)
    ref = np.float64(gamma) * (dY.astype(np.float64) @ Weff.astype(np.float64))
    assert np.allclose(dX, ref, rtol=1e-12, atol=1e-15)


def test_gradient_masked_variant_against_autograd():
    # ablation study, "gradient masking": the gradient of the latent weight when the mask multiplies the
    # weight inside the graph (w_eff = w_q * m, straight-through for the quantizer only): autograd then
    # delivers m * dL/dw_eff.  Checked on a float transcription of the layer, exactly N entries per group survive.
    N, M = 2, 4
    W = sbn_synth.latent_weight(24, 64, 77).float()
    X = sbn_synth.activations(9, 64, 78).float()
    dY = sbn_synth.grad_output(9, 24, 79).float()
    Weff, mask, gamma = oracle.quantize_mask(W.numpy(), N, M)
    xq, sx = oracle.act_quant(X.numpy())
    w = W.clone().double().requires_grad_(True)
    m = torch.from_numpy(mask.astype(np.float64))
    wq = torch.from_numpy((Weff.astype(np.float64) * float(gamma)))
    w_ste = w + (wq - w).detach()                                    # value of the quantized weight, identity gradient
    w_eff = w_ste * m                                                # the mask gates value and gradient
    x_hat = torch.from_numpy(xq.astype(np.float64) / sx.astype(np.float64)[:, None])
    y = x_hat @ w_eff.t()
    y.backward(dY.double())
    got = oracle.backward_dw_gradient_masked(dY.numpy(), xq, sx, mask)
    assert np.allclose(got, w.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert ((got != 0).reshape(24, 16, 4).sum(axis=2) <= N).all() and (got[mask == 0] == 0).all()
    dense = oracle.backward_dw(dY.numpy(), xq, sx)
    assert np.array_equal(got[mask == 1], dense[mask == 1]) and (dense[mask == 0] != 0).any()
