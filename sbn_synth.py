"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds shapes and random draws only: none of the layer's arithmetic lives here, so the CPU oracle
and the HIP path can both be fed from it without sharing any of the method.  The shapes are those
of a 30-layer ternary transformer with hidden size 2560 and FFN size 6912 (per layer: Q, K, V, O of
2560x2560, up and gate of 6912x2560, down of 2560x6912); latent weights are N(0, 0.02^2),
activations N(0, 1), output gradients N(0, (1e-2)^2), as stand-ins for the trained model's tensors.
"""
from __future__ import annotations

import torch

HIDDEN = 2560
FFN = 6912
LAYERS = 30

# (name, d_out, d_in) of the seven linear weights of one transformer block
BLOCK_MATRICES = (
    ("q_proj", HIDDEN, HIDDEN),
    ("k_proj", HIDDEN, HIDDEN),
    ("v_proj", HIDDEN, HIDDEN),
    ("o_proj", HIDDEN, HIDDEN),
    ("up_proj", FFN, HIDDEN),
    ("gate_proj", FFN, HIDDEN),
    ("down_proj", HIDDEN, FFN),
)


def seed_for(config: int, index: int) -> int:
    return 1000 * config + index


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def latent_weight(d_out: int, d_in: int, seed: int, dtype=torch.bfloat16, sigma: float = 0.02,
                  device="cpu") -> torch.Tensor:
    """Latent (master) weight ~ N(0, sigma^2), rounded once to `dtype`."""
    w = torch.randn(d_out, d_in, generator=_gen(seed, device), device=device, dtype=torch.float32)
    return (w * sigma).to(dtype)


def activations(tokens: int, d_in: int, seed: int, device="cpu") -> torch.Tensor:
    """Layer input ~ N(0, 1) in bf16."""
    x = torch.randn(tokens, d_in, generator=_gen(seed, device), device=device, dtype=torch.float32)
    return x.to(torch.bfloat16)


def grad_output(tokens: int, d_out: int, seed: int, device="cpu") -> torch.Tensor:
    """Gradient arriving at the layer output ~ N(0, (1e-2)^2) in bf16."""
    g = torch.randn(tokens, d_out, generator=_gen(seed, device), device=device, dtype=torch.float32)
    return (g * 1e-2).to(torch.bfloat16)


def adversarial_weight(d_out: int, d_in: int, seed: int, dtype=torch.bfloat16) -> torch.Tensor:
    """Latent weight full of the awkward cases: exact magnitude ties inside groups, signed zeros,
    all-zero groups, all-equal groups, values straddling half the mean magnitude, tiny values."""
    g = _gen(seed, "cpu")
    w = torch.randn(d_out, d_in, generator=g) * 0.02
    levels = torch.tensor([0.0, -0.0, 0.0078125, -0.0078125, 0.015625, -0.015625, 0.03125, 1e-6, -1e-6])
    pick = torch.randint(0, levels.numel(), (d_out, d_in), generator=g)
    use = torch.rand(d_out, d_in, generator=g) < 0.6
    w = torch.where(use, levels[pick], w)
    if d_out > 1:
        w[1] = 0.0                      # an all-zero row
    if d_out > 2:
        w[2] = 0.015625                 # every group all-equal
    if d_out > 3:
        w[3] = -w[3].abs()              # all negative
    return w.to(dtype)


def adversarial_activations(tokens: int, d_in: int, seed: int) -> torch.Tensor:
    """Activations with a zero row, a row whose products land on .5 ties, and large outliers."""
    g = _gen(seed, "cpu")
    x = torch.randn(tokens, d_in, generator=g)
    if tokens > 1:
        x[1] = 0.0
    if tokens > 2:
        # amax = 127 makes s_x = 1 exactly, so half-integers are exact rounding ties
        x[2] = (torch.randint(-253, 254, (d_in,), generator=g).float() * 0.5)
        x[2, 0] = 127.0
    if tokens > 3:
        x[3, ::97] *= 50.0
    return x.to(torch.bfloat16)
