"""Pins for the oracle's Norm(x) in front of the activation quantizer (Algorithm 1: x~ <- Q_a(Norm(x)),
read as RMS normalisation with gain): the library routine torch.nn.functional.rms_norm in fp64, closed
forms, exact invariances, and the composition with the activation quantizer."""
import numpy as np
import torch

import oracle
import sbn_synth


def bf16_ulp(y):
    """Spacing of bf16 numbers around y (8 bits of precision)."""
    return np.maximum(np.abs(y), 1e-30) * 2.0 ** -7


def is_bf16(a):
    return np.array_equal(a.view(np.uint32) & 0xffff, np.zeros(a.shape, dtype=np.uint32))


def test_rmsnorm_against_torch_rms_norm_fp64():
    X = sbn_synth.activations(48, 392, 11).float().numpy() * 3.0
    g = (1.0 + 0.25 * np.random.default_rng(12).standard_normal(392)).astype(np.float32)
    for eps in (1e-6, 1e-2):
        for gain in (None, g):
            y = oracle.rmsnorm(X, gain, eps)
            assert is_bf16(y)
            ref = torch.nn.functional.rms_norm(torch.from_numpy(X).double(), (392,),
                                               None if gain is None else torch.from_numpy(gain).double(), eps).numpy()
            # one rounding to bf16 (half a spacing) plus the fp32 roundings of r and the two multiplies
            assert (np.abs(y - ref) <= 0.5 * bf16_ulp(ref) * 1.02).all()


def test_rmsnorm_closed_forms():
    K = 256
    # a constant row has unit RMS: +-1 exactly without eps; eps = 3 c^2 halves it
    X = np.stack([np.full(K, 0.75, np.float32), np.full(K, -2.5, np.float32)])
    assert np.array_equal(oracle.rmsnorm(X, None, 0.0), np.sign(X))
    y = oracle.rmsnorm(X[:1], None, 3 * 0.75 ** 2)
    assert np.array_equal(y, np.full((1, K), 0.5, np.float32))
    # one non-zero element carries all the energy: sign(a) * sqrt(K) (= 16 for K = 256), the rest stay zero
    X = np.zeros((1, K), np.float32)
    X[0, 17] = -0.3
    y = oracle.rmsnorm(X, None, 0.0)
    assert y[0, 17] == -16.0 and np.count_nonzero(y) == 1
    # the mean runs over K, not a sum: two elements of equal size give sqrt(K / 2)
    X[0, 200] = 0.3
    y = oracle.rmsnorm(X, None, 0.0)
    assert abs(y[0, 200] - np.sqrt(K / 2)) <= 0.5 * bf16_ulp(np.sqrt(K / 2)) and y[0, 17] == -y[0, 200]
    # an all-zero row stays zero (eps keeps the root finite)
    assert (oracle.rmsnorm(np.zeros((1, K), np.float32), None, 1e-6) == 0).all()


def test_rmsnorm_exact_invariances():
    X = sbn_synth.activations(16, 384, 13).float().numpy()
    g = (1.0 + 0.25 * np.random.default_rng(14).standard_normal(384)).astype(np.float32)
    y = oracle.rmsnorm(X, g, 0.0)
    assert np.array_equal(oracle.rmsnorm(X * np.float32(8.0), g, 0.0), y)        # scale of x drops out (eps = 0)
    assert np.array_equal(oracle.rmsnorm(-X, g, 0.0), -y)
    assert np.array_equal(oracle.rmsnorm(X, g * np.float32(4.0), 0.0), y * 4.0)  # gain enters linearly, after the root
    assert np.array_equal(oracle.rmsnorm(X, np.ones(384, np.float32), 1e-5), oracle.rmsnorm(X, None, 1e-5))
    # rows are independent
    assert np.array_equal(oracle.rmsnorm(X[3:4], g, 1e-6), oracle.rmsnorm(X, g, 1e-6)[3:4])
    # unit mean square up to the bf16 rounding of the outputs
    y1 = oracle.rmsnorm(X, None, 0.0).astype(np.float64)
    assert np.allclose((y1 ** 2).mean(axis=1), 1.0, rtol=2e-3)


def test_rmsnorm_act_quant_is_the_composition():
    X = sbn_synth.activations(32, 640, 15).float().numpy()
    g = (1.0 + 0.25 * np.random.default_rng(16).standard_normal(640)).astype(np.float32)
    xq, sx, Xn = oracle.rmsnorm_act_quant(X, g, 1e-6)
    assert np.array_equal(Xn, oracle.rmsnorm(X, g, 1e-6))
    amax = np.abs(Xn).max(axis=1)
    assert np.array_equal(sx, (np.float32(127.0) / amax).astype(np.float32))
    assert np.array_equal(xq, np.clip(np.rint(Xn * sx[:, None]), -128, 127).astype(np.int8))
    assert (np.abs(xq.astype(np.int32)).max(axis=1) == 127).all()
