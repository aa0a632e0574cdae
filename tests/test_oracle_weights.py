"""Pins for the weight side of the CPU oracle (absmean scale, N:M mask, ternary values, W_eff).

Each check fixes the oracle to something other than itself: a closed form for Gaussian weights,
an exactly rounded sum, a library sort, invariances the definitions imply, or a hand-built case.
Citations: Section 2.1 (ternary quantizer, N:M definition), Section 2.2 (mask from latent weights,
quantize then mask), Section 3.4 (near-zero mass, per-block threshold).
"""
import math

import numpy as np
import pytest

import oracle

PATTERNS = [(2, 4), (1, 4), (2, 8), (6, 8), (4, 8), (1, 2), (3, 4), (8, 8), (4, 4)]
P_ZERO = math.erf(math.sqrt(2.0 / math.pi) / 2.0 / math.sqrt(2.0))   # P(|z| < sqrt(2/pi)/2) = 0.31006


def gaussian(shape, seed, sigma=0.02):
    return (np.random.default_rng(seed).standard_normal(shape) * sigma).astype(np.float32)


def to_bf16_grid(w):
    """Round fp32 values onto the bf16 grid (round-to-nearest-even on the upper 16 bits)."""
    u = w.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32)


# ----------------------------------------------------------------------------- gamma
def test_gamma_gaussian_closed_form():
    # E mean|w| = sigma * sqrt(2/pi); standard error for 2^20 samples is 1.2e-5
    W = gaussian((1024, 1024), 1)
    assert abs(float(oracle.absmean(W)) - 0.02 * math.sqrt(2 / math.pi)) < 5e-5


def test_gamma_is_exactly_rounded_mean():
    W = gaussian((300, 520), 2)
    exact = math.fsum(abs(float(v)) for v in W.ravel()) / W.size     # exactly rounded fp64 sum
    assert oracle.absmean(W) == np.float32(exact)


def test_gamma_power_of_two_scaling_and_clamp():
    W = gaussian((64, 256), 3)
    g = oracle.absmean(W)
    for k in (-3, 1, 5):
        assert oracle.absmean(W * np.float32(2.0 ** k)) == np.float32(g * np.float32(2.0 ** k))
    assert oracle.absmean(np.zeros((8, 16), np.float32)) == np.float32(1e-5)
    assert oracle.absmean(np.full((8, 16), 1e-7, np.float32)) == np.float32(1e-5)


def test_gamma_uses_whole_matrix_not_masked_subset():
    W = gaussian((128, 256), 4)
    _, mask, gamma = oracle.quantize_mask(W, 2, 4)
    masked_mean = np.abs(W[mask == 1]).mean()
    assert abs(float(gamma) - np.abs(W).mean()) < 1e-7
    assert abs(float(gamma) - masked_mean) > 1e-3          # the rejected "mask then quantize" scale differs


# ----------------------------------------------------------------------------- ternary
def test_ternary_values_and_half_threshold():
    W = gaussian((512, 512), 5)
    g = oracle.absmean(W)
    q = oracle.ternary(W, g)
    assert set(np.unique(q).tolist()) <= {-1, 0, 1}
    ratio = np.abs(W) / g                                   # numpy fp32 division, IEEE
    assert ratio.dtype == np.float32
    assert np.array_equal(q != 0, ratio > np.float32(0.5))
    assert np.array_equal(np.sign(q[q != 0]), np.sign(W[q != 0]).astype(np.int8))


def test_ternary_round_half_even_and_clip():
    g = np.float32(0.5)
    W = np.array([[0.25, -0.25, 0.2500001, 0.75, -0.75, 0.7500001, 1.25, 10.0, -10.0, 0.0, -0.0, 0.24999]],
                 dtype=np.float32)
    # w/g = .5 -> 0 (tie to even), 1.5 -> 2 -> clipped to 1, 2.5 -> 2 -> 1
    assert oracle.ternary(W, g).tolist() == [[0, 0, 1, 1, -1, 1, 1, 1, -1, 0, 0, 0]]


def test_dense_zero_fraction_is_near_zero_mass():
    # Section 3.4: near-zero mass P(|w|/mean|w| < 0.5) is the zero fraction of dense ternary weights
    W = gaussian((1024, 1024), 6)
    q = oracle.ternary(W, oracle.absmean(W))
    assert abs((q == 0).mean() - P_ZERO) < 2e-3
    assert abs((q == 1).mean() - (1 - P_ZERO) / 2) < 2e-3


def test_ternary_symmetry_and_scale_invariance():
    W = gaussian((64, 256), 7)
    g = oracle.absmean(W)
    q = oracle.ternary(W, g)
    assert np.array_equal(oracle.ternary(-W, g), -q)
    W8 = W * np.float32(8.0)
    assert np.array_equal(oracle.ternary(W8, oracle.absmean(W8)), q)


# ----------------------------------------------------------------------------- mask
def brute_force_mask(W, N, M):
    """Stable descending sort by magnitude per group; first N of the order are kept."""
    d_out, d_in = W.shape
    a = np.abs(W).reshape(d_out, d_in // M, M)
    order = np.argsort(-a, axis=-1, kind="stable")
    mask = np.zeros_like(a, dtype=np.uint8)
    np.put_along_axis(mask, order[..., :N], 1, axis=-1)
    return mask.reshape(d_out, d_in)


@pytest.mark.parametrize("N,M", PATTERNS)
def test_mask_matches_stable_sort(N, M):
    W = gaussian((96, 256), 10 + N * 16 + M)
    assert np.array_equal(oracle.nm_mask(W, N, M), brute_force_mask(W, N, M))


@pytest.mark.parametrize("N,M", PATTERNS)
def test_mask_with_ties_zeros_and_signs(N, M):
    rng = np.random.default_rng(100 + N * 16 + M)
    levels = np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0], dtype=np.float32)
    W = levels[rng.integers(0, len(levels), size=(64, 128))]
    m = oracle.nm_mask(W, N, M)
    assert np.array_equal(m, brute_force_mask(W, N, M))
    assert (m.reshape(64, -1, M).sum(-1) == N).all()        # exactly N ones per group
    # all-equal group keeps its first N positions
    E = np.full((2, 2 * M), -0.25, dtype=np.float32)
    assert oracle.nm_mask(E, N, M).reshape(-1, M).tolist() == [[1] * N + [0] * (M - N)] * 4


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8)])
def test_mask_threshold_property_and_invariances(N, M):
    W = to_bf16_grid(gaussian((128, 256), 200 + N * 16 + M))
    m = oracle.nm_mask(W, N, M).reshape(128, -1, M).astype(bool)
    a = np.abs(W).reshape(128, -1, M)
    t = np.sort(a, axis=-1)[..., M - N - 1]                 # |w|_(N+1): the (N+1)-th largest
    assert (np.where(m, a, np.inf).min(-1) >= t).all()      # kept >= threshold
    assert (np.where(~m, a, -np.inf).max(-1) <= t).all()    # dropped <= threshold
    flat = m.reshape(128, 256).astype(np.uint8)
    assert np.array_equal(oracle.nm_mask(-W, N, M), flat)
    assert np.array_equal(oracle.nm_mask(W * np.float32(4.0), N, M), flat)


def test_mask_comes_from_latent_not_quantized_weights():
    # |w| = (0.9, 1.0, 1.1, 3.0) * gamma-ish all quantize to +1; ranking must still follow the latent magnitudes
    W = np.tile(np.array([0.9, 1.0, 1.1, 3.0], dtype=np.float32), (4, 8))
    Weff, mask, _ = oracle.quantize_mask(W, 2, 4)
    assert mask.reshape(-1, 4).tolist() == [[0, 0, 1, 1]] * 32
    assert Weff.reshape(-1, 4).tolist() == [[0, 0, 1, 1]] * 32


# ----------------------------------------------------------------------------- W_eff statistics
def test_weff_structure_and_gaussian_closed_forms():
    W = gaussian((2048, 1024), 8)
    p = P_ZERO
    # 2:4 — a kept slot is zero when the largest (p^4) or the second largest (4p^3(1-p)+p^4) is below gamma/2
    Weff, mask, _ = oracle.quantize_mask(W, 2, 4)
    assert ((Weff != 0).reshape(2048, -1, 4).sum(-1) <= 2).all()
    assert (Weff[mask == 0] == 0).all()
    kept_zero = (Weff[mask == 1] == 0).mean()
    assert abs(kept_zero - (2 * p ** 4 + 4 * p ** 3 * (1 - p)) / 2) < 2e-3
    assert abs((Weff != 0).mean() - 0.5 * (1 - (2 * p ** 4 + 4 * p ** 3 * (1 - p)) / 2)) < 2e-3
    # 1:4 — the kept slot is the group maximum: zero with probability p^4
    Weff, mask, _ = oracle.quantize_mask(W, 1, 4)
    assert abs((Weff[mask == 1] == 0).mean() - p ** 4) < 1e-3
    assert abs((Weff != 0).mean() - 0.25 * (1 - p ** 4)) < 1e-3
    # 2:8 — largest of 8 (p^8) and second largest (8p^7(1-p)+p^8)
    Weff, mask, _ = oracle.quantize_mask(W, 2, 8)
    assert abs((Weff != 0).mean() - 0.25 * (1 - (2 * p ** 8 + 8 * p ** 7 * (1 - p)) / 2)) < 1e-3


def test_n_equals_m_is_plain_bitlinear_weights():
    W = gaussian((64, 128), 9)
    Weff, mask, gamma = oracle.quantize_mask(W, 4, 4)
    assert mask.all()
    expect = np.clip(np.rint(W / np.float32(np.abs(W).astype(np.float64).mean())), -1, 1).astype(np.int8)
    assert np.array_equal(Weff, expect)


def test_flip_rate():
    W = gaussian((64, 128), 11)
    m = oracle.nm_mask(W, 2, 4)
    assert oracle.flip_rate(m, m) == 0.0
    a = np.tile(np.array([1, 1, 0, 0], np.uint8), (4, 8))
    b = np.tile(np.array([0, 0, 1, 1], np.uint8), (4, 8))
    assert oracle.flip_rate(a, b) == 1.0                    # disjoint kept sets: 2N/M with N = 2, M = 4
