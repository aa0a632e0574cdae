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


def noisy_step(W0, seed, scale=0.25):
    """The next step's latent weights: a noisy update under which some masks flip and most stay."""
    step = sbn_synth.latent_weight(W0.shape[0], W0.shape[1], seed, device=W0.device)
    return (W0.float() + scale * step.float()).to(torch.bfloat16)


def oracle_flips(W0, W1, N, M):
    m0 = oracle.nm_mask(W0.float().cpu().numpy(), N, M)
    m1 = oracle.nm_mask(W1.float().cpu().numpy(), N, M)
    return int((m0 != m1).sum())


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8)])
def test_pack_in_place_counts_mask_flips(N, M):
    # the per-step remask in place over the previous packed forms with the flip count as a by-product: a batch
    # of matrices whose last unit is partial (111, 1500 chunks) or whole, three steps in a row on one set of
    # buffers (the counters start from zero every call); bytes and gamma against the oracle's pack of the new
    # weights, flips against the oracle's masks of both steps and against the separate flip kernels
    s = sbn()
    shapes = [(37, 384), (256, 1280), (300, 640), (512, 4096), (16, 128)] * 3
    Ws = [sbn_synth.latent_weight(a, b, 2000 + i).to(DEV) for i, (a, b) in enumerate(shapes)]
    packed = [torch.zeros(s.sbn_packed_bytes(a, b, N, M), dtype=torch.uint8, device=DEV) for a, b in shapes]
    gammas = torch.zeros(len(shapes), dtype=torch.float32, device=DEV)
    glist = [gammas[i:i + 1] for i in range(len(shapes))]
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(shapes), 512, 4096, N, M))
    s.sbn_quantize_mask_pack_batched(Ws, N, M, packed, glist, ws)
    torch.cuda.synchronize()
    flips = torch.full((len(shapes),), -7, dtype=torch.int64, device=DEV)
    for step in range(3):
        Wn = [noisy_step(W, 2100 + 50 * step + i, scale=0.25 if step < 2 else 0.0) for i, W in enumerate(Ws)]
        old = [p.clone() for p in packed]
        s.sbn_quantize_mask_pack_flips_batched(Wn, N, M, packed, glist, flips, ws)
        torch.cuda.synchronize()
        got = flips.cpu().numpy()
        for i, (W0, W1) in enumerate(zip(Ws, Wn)):
            ref, g, *_ = oracle_pack(W1.cpu(), N, M)
            assert gammas[i].item() == g, f"step {step}, gamma of matrix {i}"
            assert np.array_equal(packed[i].cpu().numpy(), ref), f"step {step}, packed bytes of matrix {i}"
            expected = oracle_flips(W0, W1, N, M)
            assert got[i] == expected, f"step {step}, flips of matrix {i}: {got[i]} != {expected}"
            assert (expected > 0) == (step < 2)        # the third step repeats the second's weights: nothing flips
            one = torch.zeros(1, dtype=torch.int64, device=DEV)
            wsf = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_MASK_FLIPS, 1, shapes[i][0], shapes[i][1], N, M))
            s.sbn_mask_flips(old[i], packed[i], shapes[i][0], shapes[i][1], N, M, one, wsf)
            assert one.item() == expected
        Ws = Wn


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8)])
def test_pack_in_place_counts_mask_flips_three_pass_form(N, M):
    # a matrix of more units than the persistent grid holds blocks takes the three-pass form (sum, finalize, pack):
    # its pack kernel counts the flips the same way
    s = sbn()
    a, b = 6912, 4096
    W0 = sbn_synth.latent_weight(a, b, 2300 + N, device=DEV)
    W1 = noisy_step(W0, 2301 + N)
    packed = torch.zeros(s.sbn_packed_bytes(a, b, N, M), dtype=torch.uint8, device=DEV)
    gamma = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, 1, a, b, N, M))
    s.sbn_quantize_mask_pack(W0, N, M, packed, gamma, ws)
    flips = torch.full((1,), -7, dtype=torch.int64, device=DEV)
    s.sbn_quantize_mask_pack_flips_batched([W1], N, M, [packed], [gamma], flips, ws)
    torch.cuda.synchronize()
    ref, g, *_ = oracle_pack(W1.cpu(), N, M)
    assert gamma.item() == g
    assert np.array_equal(packed.cpu().numpy(), ref)
    assert flips.item() == oracle_flips(W0, W1, N, M)


def test_config4_sweep_in_place_with_flips_as_timed(sweep_latents):
    # the 210-matrix sweep of configs[3] at 2:4 as the benchmark times its flip-counting form: one batched call in
    # place over the previous step's packed forms; every packed byte, gamma and flip count against the oracle
    from concurrent.futures import ThreadPoolExecutor
    s = sbn()
    N, M = 2, 4
    Wl = sweep_latents
    W1 = [noisy_step(w, 2400 + i) for i, w in enumerate(Wl)]
    packed = [torch.zeros(s.sbn_packed_bytes(w.shape[0], w.shape[1], N, M), dtype=torch.uint8, device=DEV) for w in Wl]
    gammas = torch.zeros(len(Wl), dtype=torch.float32, device=DEV)
    glist = [gammas[i:i + 1] for i in range(len(Wl))]
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(Wl), sbn_synth.FFN, sbn_synth.HIDDEN, N, M))
    s.PackBatch(Wl, N, M, packed, glist, ws).run()
    flips = torch.full((len(Wl),), -7, dtype=torch.int64, device=DEV)
    s.PackBatch(W1, N, M, packed, glist, ws, flips).run()
    torch.cuda.synchronize()
    got_gamma, got_flips = gammas.cpu().numpy(), flips.cpu().numpy()

    def one(i):
        ref, g, *_ = oracle_pack(W1[i].cpu(), N, M)
        return i, g == got_gamma[i], np.array_equal(packed[i].cpu().numpy(), ref), got_flips[i] == oracle_flips(Wl[i], W1[i], N, M)

    with ThreadPoolExecutor(4) as pool:
        for i, gamma_ok, bytes_ok, flips_ok in pool.map(one, range(len(Wl))):
            assert gamma_ok, f"gamma of matrix {i}"
            assert bytes_ok, f"packed bytes of matrix {i}"
            assert flips_ok, f"flips of matrix {i}"
    del W1
    torch.cuda.empty_cache()


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
    # the flip-counting form on the same branches: in place over what the loop above left, with the next step's weights
    W1 = [noisy_step(W, 1850 + i) for i, W in enumerate(Wd)]
    flips = torch.full((len(shapes),), -7, dtype=torch.int64, device=DEV)
    s.sbn_quantize_mask_pack_flips_batched(W1, N, M, packed, glist, flips, ws)
    torch.cuda.synchronize()
    for i, (W0, Wn) in enumerate(zip(Wd, W1)):
        ref, g, *_ = oracle_pack(Wn.cpu(), N, M)
        assert gammas[i].item() == g
        assert np.array_equal(packed[i].cpu().numpy(), ref)
        assert flips[i].item() == oracle_flips(W0, Wn, N, M)
