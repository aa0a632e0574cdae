"""GPU parity of quantize_mask_pack (and the unpack hook) against the CPU oracle: packed bytes and
gamma bit-exact.  Section 2.1 / 2.2 define the arithmetic; the byte layout is include/sbn.h's."""
import numpy as np
import pytest
import torch

import oracle
import sbn_synth
from gpu_util import DEV, hip_pack, oracle_pack, sbn

pytestmark = pytest.mark.gpu

PATTERNS = [(2, 4), (1, 4), (2, 8), (6, 8), (4, 8), (1, 2), (3, 4), (8, 8), (4, 4), (1, 8), (7, 8), (2, 2), (3, 8), (5, 8)]


def check(W, N, M):
    packed, gamma = hip_pack(W, N, M)
    ref_packed, ref_gamma, Weff, mask = oracle_pack(W, N, M)
    assert gamma.cpu().numpy()[0] == ref_gamma, f"gamma {gamma.item()!r} vs {ref_gamma!r}"
    got = packed.cpu().numpy()
    assert got.size == ref_packed.size
    assert np.array_equal(got, ref_packed), f"{(got != ref_packed).sum()} packed bytes differ"
    return packed, Weff, mask


@pytest.mark.parametrize("N,M", PATTERNS)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_pack_small_shapes(N, M, dtype):
    # 100 x 384: several blocks of 16 chunks and a ragged last block
    check(sbn_synth.latent_weight(100, 384, 1 + N + 16 * M, dtype=dtype), N, M)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8)])
@pytest.mark.parametrize("shape", [(3, 8), (5, 136), (33, 200), (1, 128), (17, 1032)])
def test_pack_ragged_tails(N, M, shape):
    # d_in not a multiple of 128 (zero-padded last chunk) and not a multiple of 8 vectors
    check(sbn_synth.latent_weight(shape[0], shape[1], 50 + N + M, dtype=torch.bfloat16), N, M)
    check(sbn_synth.latent_weight(shape[0], shape[1], 60 + N + M, dtype=torch.float32), N, M)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8), (4, 4)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_pack_adversarial_ties_and_zeros(N, M, dtype):
    check(sbn_synth.adversarial_weight(64, 512, 70 + N, dtype=dtype), N, M)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8)])
def test_pack_wide_dynamic_range(N, M):
    # magnitudes from 2^-10 to 2^6 (bf16 exponent field with its top bit set and clear), both signs, many exact
    # ties: every bit of the magnitude takes part in the ranking; |w| sums stay exact in fp64 whatever their order
    g = torch.Generator().manual_seed(90 + N + M)
    e = torch.randint(-10, 7, (256, 384), generator=g).float()
    m = 1.0 + torch.randint(0, 4, (256, 384), generator=g).float() / 4.0
    sgn = torch.randint(0, 2, (256, 384), generator=g).float() * 2.0 - 1.0
    W = (sgn * m * torch.exp2(e)).to(torch.bfloat16)
    W[5] = 96.0
    W[6, ::3] = -0.0
    _, Weff, mask = check(W, N, M)
    assert (np.abs(Weff).sum(axis=1) > 0).any()


def test_pack_all_zero_matrix_clamps_gamma():
    packed, gamma = hip_pack(torch.zeros(16, 256, dtype=torch.bfloat16), 2, 4)
    assert gamma.item() == np.float32(1e-5)
    ref, g, *_ = oracle_pack(torch.zeros(16, 256, dtype=torch.bfloat16), 2, 4)
    assert np.array_equal(packed.cpu().numpy(), ref)


def test_pack_strided_rows():
    s = sbn()
    base = sbn_synth.latent_weight(40, 512, 80)
    view = base[:, 64:64 + 256]                      # ld = 512, d_in = 256
    Wd = base.to(DEV)[:, 64:64 + 256]
    packed = torch.zeros(s.sbn_packed_bytes(40, 256, 2, 4), dtype=torch.uint8, device=DEV)
    gamma = torch.zeros(1, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, 1, 40, 256, 2, 4))
    s.sbn_quantize_mask_pack(Wd, 2, 4, packed, gamma, ws)
    ref, g, *_ = oracle_pack(view.contiguous(), 2, 4)
    assert gamma.item() == g and np.array_equal(packed.cpu().numpy(), ref)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8), (8, 8)])
def test_unpack_hook_matches_oracle(N, M):
    s = sbn()
    W = sbn_synth.latent_weight(70, 392, 90 + N)
    packed, Weff, mask = check(W, N, M)
    We = torch.full((70, 392), 9, dtype=torch.int8, device=DEV)
    Mk = torch.full((70, 392), 9, dtype=torch.uint8, device=DEV)
    s.sbn_unpack(packed, 70, 392, N, M, We, Mk)
    assert np.array_equal(We.cpu().numpy(), Weff) and np.array_equal(Mk.cpu().numpy(), mask)


def test_pack_config1_fp32():
    # configs[0]: W 256x256 fp32 ~ N(0, 0.02), 2:4
    check(sbn_synth.latent_weight(256, 256, sbn_synth.seed_for(1, 0), dtype=torch.float32), 2, 4)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8)])
@pytest.mark.parametrize("shape", [(2560, 2560), (6912, 2560), (2560, 6912)])
def test_pack_full_size_matrices(N, M, shape):
    # the three matrix shapes of the 30-layer sweep, at the sweep's three patterns
    check(sbn_synth.latent_weight(shape[0], shape[1], sbn_synth.seed_for(4, shape[0] + N)), N, M)


def test_pack_batched_equals_single():
    s = sbn()
    shapes = [(256, 256), (100, 384), (33, 200), (640, 1280)] * 14       # 56 matrices: two launches
    Ws = [sbn_synth.latent_weight(a, b, 300 + i).to(DEV) for i, (a, b) in enumerate(shapes)]
    packed = [torch.zeros(s.sbn_packed_bytes(a, b, 2, 4), dtype=torch.uint8, device=DEV) for a, b in shapes]
    gammas = torch.zeros(len(shapes), dtype=torch.float32, device=DEV)
    glist = [gammas[i:i + 1] for i in range(len(shapes))]
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(shapes), 640, 1280, 2, 4))
    s.sbn_quantize_mask_pack_batched(Ws, 2, 4, packed, glist, ws)
    torch.cuda.synchronize()
    for i, W in enumerate(Ws):
        ref, g, *_ = oracle_pack(W.cpu(), 2, 4)
        assert gammas[i].item() == g
        assert np.array_equal(packed[i].cpu().numpy(), ref)


@pytest.fixture(scope="module")
def sweep_latents():
    """The 210 latent matrices of the 30-layer sweep, generated on the device exactly as the benchmark does
    (4.76 GB); freed when the module's tests are done."""
    Wl = []
    for layer in range(sbn_synth.LAYERS):
        for mi, (_, a, b) in enumerate(sbn_synth.BLOCK_MATRICES):
            Wl.append(sbn_synth.latent_weight(a, b, sbn_synth.seed_for(4, 10 * layer + mi), device=DEV))
    yield Wl
    del Wl
    torch.cuda.empty_cache()


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8)])
def test_config4_full_sweep_as_timed(N, M, sweep_latents):
    # configs[3] in the launch configuration the benchmark times: ONE batched call over all 210 matrices of the
    # 30-layer model (the library cuts it into three launches of 70), one workspace; every gamma and every
    # packed byte of every matrix against the oracle (the oracle's weight side runs on a few host threads,
    # matrix by matrix)
    from concurrent.futures import ThreadPoolExecutor
    s = sbn()
    Wl = sweep_latents
    assert len(Wl) == 210 and sum(w.numel() for w in Wl) == 2378956800
    packed = [torch.full((s.sbn_packed_bytes(w.shape[0], w.shape[1], N, M),), 0xAA, dtype=torch.uint8, device=DEV) for w in Wl]
    gammas = torch.zeros(len(Wl), dtype=torch.float32, device=DEV)
    glist = [gammas[i:i + 1] for i in range(len(Wl))]
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(Wl), sbn_synth.FFN, sbn_synth.HIDDEN, N, M))
    batch = s.PackBatch(Wl, N, M, packed, glist, ws)
    batch.run()
    batch.run()          # the timed loop calls it back to back on one workspace: counters and flags start clean
    torch.cuda.synchronize()
    got_gamma = gammas.cpu().numpy()

    def one(i):
        ref, g, *_ = oracle_pack(Wl[i].cpu(), N, M)
        return i, g == got_gamma[i], np.array_equal(packed[i].cpu().numpy(), ref)

    with ThreadPoolExecutor(4) as pool:
        for i, gamma_ok, bytes_ok in pool.map(one, range(len(Wl))):
            assert gamma_ok, f"gamma of matrix {i}"
            assert bytes_ok, f"packed bytes of matrix {i}"


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8), (3, 8), (1, 2), (4, 4)])
@pytest.mark.parametrize("shape", [(37, 392), (256, 1280)])
def test_mask_flips_between_two_steps(N, M, shape):
    # ablation study, mask flip rate equation: || m(W_t) - m(W_{t-1}) ||_1 from the packed index fields
    # of two steps, against the oracle's masks of the same two weight tensors (ragged last chunk included)
    s = sbn()
    W0 = sbn_synth.latent_weight(shape[0], shape[1], 900 + N + M)
    step = sbn_synth.latent_weight(shape[0], shape[1], 901 + N + M)
    W1 = (W0.float() + 0.25 * step.float()).to(torch.bfloat16)      # a noisy update: some masks flip, most stay
    p0, _ = hip_pack(W0, N, M)
    p1, _ = hip_pack(W1, N, M)
    flips = torch.full((1,), -5, dtype=torch.int64, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_MASK_FLIPS, 1, shape[0], shape[1], N, M))
    s.sbn_mask_flips(p0, p1, shape[0], shape[1], N, M, flips, ws)
    torch.cuda.synchronize()
    m0 = oracle.nm_mask(W0.float().numpy(), N, M)
    m1 = oracle.nm_mask(W1.float().numpy(), N, M)
    expected = int((m0 != m1).sum())
    assert flips.item() == expected
    assert oracle.flip_rate(m0, m1) == expected / m0.size
    if N < M:
        assert expected > 0
    s.sbn_mask_flips(p0, p0, shape[0], shape[1], N, M, flips, ws)
    torch.cuda.synchronize()
    assert flips.item() == 0


@pytest.fixture
def spin_limits():
    """Sets the bounds of the library's bounded waits for one test and restores the defaults afterwards."""
    s = sbn()
    yield s.sbn_test_set_spin_limits
    s.sbn_test_set_spin_limits()


@pytest.mark.parametrize("spin_limit", [-1, 0, 3])
@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8)])
def test_single_read_pack_when_blocks_do_not_wait(N, M, spin_limit, spin_limits):
    # the single-read form of the pack kernel with its wait cut short: -1 = no block waits for the matrix's
    # last block (each derives the threshold from HBM itself), 0 and 3 = a few polls, then the same;
    # bytes and gamma must not depend on which way a block took
    spin_limits(pack_polls=spin_limit)
    s = sbn()
    shapes = [(640, 1280), (100, 384), (256, 256), (1024, 2560)]
    Ws = [sbn_synth.latent_weight(a, b, 1800 + i) for i, (a, b) in enumerate(shapes)]
    Wd = [W.to(DEV) for W in Ws]
    packed = [torch.zeros(s.sbn_packed_bytes(a, b, N, M), dtype=torch.uint8, device=DEV) for a, b in shapes]
    gammas = torch.zeros(len(shapes), dtype=torch.float32, device=DEV)
    glist = [gammas[i:i + 1] for i in range(len(shapes))]
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(shapes), 1024, 2560, N, M))
    for _ in range(2):   # twice through the same workspace: counters and flags start clean every call
        s.sbn_quantize_mask_pack_batched(Wd, N, M, packed, glist, ws)
        torch.cuda.synchronize()
        for i, W in enumerate(Ws):
            ref, g, *_ = oracle_pack(W, N, M)
            assert gammas[i].item() == g
            assert np.array_equal(packed[i].cpu().numpy(), ref)
