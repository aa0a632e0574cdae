"""GPU parity of sparse_ternary_linear against the CPU oracle: int8 activations, per-token scales
and int32 accumulators bit-exact; Y within 1e-3 relative (Section 2.1 activation quantizer,
Section 2.2 forward-pass equation)."""
import numpy as np
import pytest
import torch

import oracle
import sbn_synth
from gpu_util import DEV, assert_rel, hip_linear, hip_pack, oracle_pack, sbn

pytestmark = pytest.mark.gpu
Y_TOL = 1e-3


def check_forward(W, X, N, M, path, bias=None, token_sample=None):
    packed, gamma = hip_pack(W, N, M)
    _, ref_gamma, Weff, _ = oracle_pack(W, N, M)
    Y, acc, xq, sx = hip_linear(X, packed, gamma, W.shape[0], N, M, path, bias)
    Xf = X.float().numpy()
    r_xq, r_sx = oracle.act_quant(Xf)
    assert np.array_equal(xq, r_xq), "int8 activations differ"
    assert np.array_equal(sx, r_sx), "activation scales differ"
    rows = np.arange(X.shape[0]) if token_sample is None else token_sample
    r_acc = oracle.acc(Weff, r_xq[rows])
    assert np.array_equal(acc[rows], r_acc), f"{(acc[rows] != r_acc).sum()} accumulators differ"
    r_y = oracle.rescale(r_acc, ref_gamma, r_sx[rows], None if bias is None else bias.numpy())
    if bias is None:
        assert_rel(Y[rows], r_y, Y_TOL, "Y")
    else:
        # acc * scale + bias can cancel: the rounding of the sum is relative to |acc * scale| + |bias|
        r_nb = oracle.rescale(r_acc, ref_gamma, r_sx[rows], None)
        err = np.abs(Y[rows].astype(np.float64) - r_y)
        bound = Y_TOL * (np.abs(r_nb) + np.abs(bias.numpy().astype(np.float64))[None, :])
        assert (err <= bound).all(), f"Y with bias: {(err > bound).sum()} beyond tolerance; worst {err.max()}"
    return Y


def test_config1_forward_all_paths():
    # configs[0]: X 16x256 bf16, W 256x256 fp32, 2:4
    s = sbn()
    W = sbn_synth.latent_weight(256, 256, sbn_synth.seed_for(1, 0), dtype=torch.float32)
    X = sbn_synth.activations(16, 256, sbn_synth.seed_for(1, 1))
    for path in (s.SBN_PATH_GENERIC, s.SBN_PATH_GEMV, s.SBN_PATH_AUTO):
        check_forward(W, X, 2, 4, path)


@pytest.mark.parametrize("tokens", [1, 3, 8, 16])
@pytest.mark.parametrize("shape", [(48, 128), (100, 640), (250, 1792), (16, 2560)])
def test_gemv_shapes(tokens, shape):
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 400 + shape[0])
    X = sbn_synth.activations(tokens, shape[1], 500 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(7))
    check_forward(W, X, 2, 4, s.SBN_PATH_GEMV, bias=bias)


def test_gemv_adversarial_inputs():
    s = sbn()
    W = sbn_synth.adversarial_weight(64, 512, 410)
    X = sbn_synth.adversarial_activations(8, 512, 411)
    check_forward(W, X, 2, 4, s.SBN_PATH_GEMV)


@pytest.mark.parametrize("tokens", [1, 8])
@pytest.mark.parametrize("shape", [(6912, 2560), (2560, 6912)])
def test_config2_decode_gemv_full_size(tokens, shape):
    # configs[1]: FFN up (6912x2560) and down (2560x6912) projections, batch 1 and 8
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], sbn_synth.seed_for(2, shape[0]))
    X = sbn_synth.activations(tokens, shape[1], sbn_synth.seed_for(2, 100 + tokens))
    check_forward(W, X, 2, 4, s.SBN_PATH_GEMV)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (6, 8), (4, 4), (1, 2), (3, 8)])
def test_generic_path_all_patterns(N, M):
    s = sbn()
    W = sbn_synth.latent_weight(130, 392, 420 + N + M)
    X = sbn_synth.activations(11, 392, 430)
    check_forward(W, X, N, M, s.SBN_PATH_GENERIC)


@pytest.mark.parametrize("N,M", [(6, 8), (2, 8), (1, 4), (4, 4), (3, 8), (7, 8)])
@pytest.mark.parametrize("tokens,shape", [(40, (130, 384)), (300, (520, 1280))])
def test_dense_mfma_path_other_patterns(N, M, tokens, shape):
    # the comparison path (weights expanded to int8 with explicit zeros, dense int8 matrix cores) takes every pattern
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 440 + N + M)
    X = sbn_synth.activations(tokens, shape[1], 450 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(9))
    check_forward(W, X, N, M, s.SBN_PATH_DENSE_MFMA, bias=bias)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 8), (1, 8), (1, 2)])
@pytest.mark.parametrize("tokens,shape", [(40, (130, 384)), (300, (520, 1280))])
def test_sparse_mfma_path_instances_of_2of4(N, M, tokens, shape):
    # patterns that never keep more than two of an aligned four are rewritten into the 2:4 operand form and
    # run on the sparse matrix instruction: same integers as the oracle, explicitly and through path selection
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 470 + N + M)
    X = sbn_synth.activations(tokens, shape[1], 480 + tokens)
    check_forward(W, X, N, M, s.SBN_PATH_SMFMAC)
    check_forward(W, X, N, M, s.SBN_PATH_AUTO)


@pytest.mark.parametrize("N,M", [(6, 8), (8, 8), (3, 4), (7, 8), (5, 8), (4, 4), (3, 8)])
@pytest.mark.parametrize("tokens,shape", [(40, (130, 384)), (300, (520, 1280)), (129, (1100, 128)), (97, (64, 2560))])
def test_sparse_mfma_path_dense_codes(N, M, tokens, shape):
    # patterns that keep more than two of an aligned four run beyond decode sizes as dense 2-bit codes (N = M as
    # stored, the rest converted first) through two sparse instructions per group of four: ragged edges in rows and
    # tokens, one chunk (128) and an odd number of chunks (384 = 3), bias; same integers as the oracle
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 2440 + 10 * N + M)
    X = sbn_synth.activations(tokens, shape[1], 2450 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(19))
    check_forward(W, X, N, M, s.SBN_PATH_SMFMAC, bias=bias)
    check_forward(W, X, N, M, s.SBN_PATH_AUTO)


def test_sparse_mfma_path_dense_codes_adversarial():
    s = sbn()
    W = sbn_synth.adversarial_weight(256, 512, 2460)
    X = sbn_synth.adversarial_activations(64, 512, 2461)
    for N, M in ((6, 8), (8, 8)):
        check_forward(W, X, N, M, s.SBN_PATH_SMFMAC)


@pytest.mark.parametrize("N,M", [(6, 8), (8, 8)])
def test_config3_prefill_dense_codes_full_size_as_timed(N, M):
    # configs[2] at the paper's main pattern: 4096 tokens against 6912x2560, as the benchmark times it (no accumulator
    # output); sampled token rows against the oracle, and the launch with accumulators bit for bit the same Y
    s = sbn()
    W = sbn_synth.latent_weight(6912, 2560, sbn_synth.seed_for(3, 6912))
    X = sbn_synth.activations(4096, 2560, sbn_synth.seed_for(3, 1))
    sample = np.unique(np.concatenate([np.arange(0, 4096, 97), [31, 32, 127, 128, 4095]]))
    Y = check_forward(W, X, N, M, s.SBN_PATH_SMFMAC, token_sample=sample)
    packed, gamma = hip_pack(W, N, M)
    Y2, *_ = hip_linear(X, packed, gamma, 6912, N, M, s.SBN_PATH_SMFMAC, want_acc=False)
    assert np.array_equal(Y, Y2)


@pytest.mark.parametrize("N,M", [(2, 4), (6, 8)])
def test_dense_comparison_kernel_alone(N, M):
    # the dense int8 kernel on weights expanded beforehand (sbn_unpack) gives what the comparison path gives with its
    # own expansion pass, bit for bit, with and without the accumulator output, and the oracle's integers
    s = sbn()
    W = sbn_synth.latent_weight(520, 640, 2490 + N)
    X = sbn_synth.activations(300, 640, 2491)
    bias = torch.randn(520, generator=torch.Generator().manual_seed(23))
    packed, gamma = hip_pack(W, N, M)
    Y1, acc1, xq, sx = hip_linear(X, packed, gamma, 520, N, M, s.SBN_PATH_DENSE_MFMA, bias)
    Weff = torch.empty(520, 640, dtype=torch.int8, device=DEV)
    s.sbn_unpack(packed, 520, 640, N, M, W_eff=Weff)
    _, _, ref_Weff, _ = oracle_pack(W, N, M)
    assert np.array_equal(Weff.cpu().numpy(), ref_Weff)
    for want_acc in (True, False):
        Y = torch.full((300, 520), float("nan"), dtype=torch.float32, device=DEV)
        acc = torch.full((300, 520), -7, dtype=torch.int32, device=DEV)
        s.sbn_dense_ternary_linear(torch.from_numpy(xq).to(DEV), torch.from_numpy(sx).to(DEV), Weff, gamma, Y,
                                   bias=bias.to(DEV), acc_out=acc if want_acc else None)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy(), Y1)
        if want_acc:
            assert np.array_equal(acc.cpu().numpy(), acc1)
            assert np.array_equal(acc1, oracle.acc(ref_Weff, xq))


def test_grouped_prefill_dense_codes_matches_single():
    # N = M problems of different shapes in one grouped launch of the GEMM kernel
    s = sbn()
    shapes = [(520, 384), (100, 128), (1030, 640)]
    tokens = [200, 40, 333]
    packs = [hip_pack(sbn_synth.latent_weight(a, b, 2470 + i), 8, 8) for i, (a, b) in enumerate(shapes)]
    Xs = [sbn_synth.activations(t, b, 2480 + i).to(DEV) for i, (t, (_, b)) in enumerate(zip(tokens, shapes))]
    Ys = [torch.zeros(t, a, dtype=torch.float32, device=DEV) for t, (a, _) in zip(tokens, shapes)]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, t, a, b, 8, 8) for t, (a, b) in zip(tokens, shapes))
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped(Xs, [p for p, _ in packs], [g for _, g in packs], Ys, 8, 8, ws, path=s.SBN_PATH_SMFMAC)
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(shapes):
        Y1, *_ = hip_linear(Xs[i].cpu(), packs[i][0], packs[i][1], a, 8, 8, s.SBN_PATH_SMFMAC, want_acc=False)
        assert np.array_equal(Ys[i].cpu().numpy(), Y1)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 8), (6, 8), (3, 8)])
@pytest.mark.parametrize("tokens", [1, 8, 16])
def test_decode_sizes_other_patterns_through_path_selection(N, M, tokens):
    # decode batches of other patterns: instances of 2:4 take the decode kernel after the rewrite into the
    # 2:4 operand form, the rest after the rewrite into dense 2-bit codes (dense matrix instruction)
    s = sbn()
    W = sbn_synth.latent_weight(200, 640, 490 + N + M)
    X = sbn_synth.activations(tokens, 640, 491 + tokens)
    check_forward(W, X, N, M, s.SBN_PATH_AUTO)
    check_forward(W, X, N, M, s.SBN_PATH_GEMV)


@pytest.mark.parametrize("tokens,shape", [(1, (48, 128)), (5, (100, 640)), (16, (250, 1792)), (8, (33, 2560)), (3, (16, 256))])
def test_decode_1of4_as_stored_shapes(tokens, shape):
    # the decode kernel reads the 1:4 packed form as stored (one bit per weight) and builds the sparse
    # instruction's operands in registers: ragged row counts, a partial last super-step, bias
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 1700 + shape[0])
    X = sbn_synth.activations(tokens, shape[1], 1701 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(13))
    check_forward(W, X, 1, 4, s.SBN_PATH_GEMV, bias=bias)


def test_decode_1of4_as_stored_adversarial_and_full_size():
    # ties inside groups, signed zeros, extreme magnitudes; then one kept position for the whole matrix (each of
    # the four in turn: both aligned pairs and both slots of the rewrite); then the decode shapes of configs[1]
    s = sbn()
    W = sbn_synth.adversarial_weight(64, 512, 1710)
    X = sbn_synth.adversarial_activations(8, 512, 1711)
    check_forward(W, X, 1, 4, s.SBN_PATH_GEMV)
    base = sbn_synth.latent_weight(48, 1024, 1712)
    for pos in range(4):
        W = base * 1e-3
        W[:, pos::4] = base[:, pos::4] + torch.sign(base[:, pos::4])   # the largest of every group by a wide margin
        _, _, _, mask = oracle_pack(W, 1, 4)
        assert mask.reshape(-1, 4)[:, pos].all()
        check_forward(W, sbn_synth.activations(5, 1024, 1713 + pos), 1, 4, s.SBN_PATH_GEMV)
    for shape, tokens in (((6912, 2560), 8), ((2560, 6912), 1)):
        W = sbn_synth.latent_weight(shape[0], shape[1], sbn_synth.seed_for(2, 14 + shape[0]))
        X = sbn_synth.activations(tokens, shape[1], sbn_synth.seed_for(2, 114 + tokens))
        check_forward(W, X, 1, 4, s.SBN_PATH_AUTO)


@pytest.mark.parametrize("tokens", [1, 8, 16])
def test_grouped_streaming_1of4_against_oracle(tokens):
    # 1:4 in one grouped call: the persistent streaming kernel on the packed form as stored (ragged row counts,
    # a partial last super-step at K = 768 and 640, three inputs quantized by the kernel)
    s = sbn()
    shapes = [(4100, 768), (4096, 256), (5000, 640)] * 14
    Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 1750 + sh[0]) for sh in set(shapes)}
    packs = {sh: hip_pack(W, 1, 4) for sh, W in Ws.items()}
    Xs = {k: sbn_synth.activations(tokens, k, 1760 + k) for k in (768, 256, 640)}
    Xd = {k: x.to(DEV) for k, x in Xs.items()}
    Y_list = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, 1, 4) for a, b in shapes)
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped([Xd[b] for _, b in shapes], [packs[sh][0] for sh in shapes],
                                        [packs[sh][1] for sh in shapes], Y_list, 1, 4, ws, path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    ref = {}
    for sh, W in Ws.items():
        _, g, Weff, _ = oracle_pack(W, 1, 4)
        y, *_ = oracle.sparse_ternary_linear(Xs[sh[1]].float().numpy(), Weff, g)
        ref[sh] = y
    for i, sh in enumerate(shapes):
        assert_rel(Y_list[i].cpu().numpy(), ref[sh], Y_TOL, f"Y of problem {i}")


@pytest.mark.parametrize("N,M", [(6, 8), (3, 8), (7, 8), (5, 8), (4, 8), (3, 4), (8, 8), (4, 4), (2, 2)])
@pytest.mark.parametrize("tokens,shape", [(1, (48, 128)), (5, (100, 640)), (16, (250, 1792)), (8, (33, 2560))])
def test_decode_dense_codes_shapes(N, M, tokens, shape):
    # the decode kernel on dense 2-bit codes: ragged row counts, a partial last super-step (640 = 5 chunks,
    # 1792 = 14), bias; N = M is stored as dense codes and needs no rewrite
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 1500 + 10 * N + M)
    X = sbn_synth.activations(tokens, shape[1], 1501 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(11))
    check_forward(W, X, N, M, s.SBN_PATH_GEMV, bias=bias)


def test_decode_dense_codes_adversarial_and_full_size():
    s = sbn()
    W = sbn_synth.adversarial_weight(64, 512, 1510)
    X = sbn_synth.adversarial_activations(8, 512, 1511)
    check_forward(W, X, 6, 8, s.SBN_PATH_GEMV)
    check_forward(W, X, 8, 8, s.SBN_PATH_GEMV)
    # the paper's main pattern at the decode shapes of configs[1]
    for shape, tokens in (((6912, 2560), 8), ((2560, 6912), 1)):
        W = sbn_synth.latent_weight(shape[0], shape[1], sbn_synth.seed_for(2, 68 + shape[0]))
        X = sbn_synth.activations(tokens, shape[1], sbn_synth.seed_for(2, 168 + tokens))
        check_forward(W, X, 6, 8, s.SBN_PATH_AUTO)


@pytest.mark.parametrize("tokens", [1, 8, 16])
def test_grouped_streaming_dense_codes_against_oracle(tokens):
    # N = M (plain ternary weights, no mask) in one grouped call: the persistent streaming kernel on dense codes
    s = sbn()
    shapes = [(4100, 768), (4096, 256), (5000, 640)] * 14
    Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 1550 + sh[0]) for sh in set(shapes)}
    packs = {sh: hip_pack(W, 8, 8) for sh, W in Ws.items()}
    Xs = {k: sbn_synth.activations(tokens, k, 1560 + k) for k in (768, 256, 640)}
    Xd = {k: x.to(DEV) for k, x in Xs.items()}
    Y_list = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, 8, 8) for a, b in shapes)
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped([Xd[b] for _, b in shapes], [packs[sh][0] for sh in shapes],
                                        [packs[sh][1] for sh in shapes], Y_list, 8, 8, ws, path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    ref = {}
    for sh, W in Ws.items():
        _, g, Weff, _ = oracle_pack(W, 8, 8)
        y, *_ = oracle.sparse_ternary_linear(Xs[sh[1]].float().numpy(), Weff, g)
        ref[sh] = y
    for i, sh in enumerate(shapes):
        assert_rel(Y_list[i].cpu().numpy(), ref[sh], Y_TOL, f"Y of problem {i}")


def test_sparse_mfma_path_adversarial_2of8():
    s = sbn()
    W = sbn_synth.adversarial_weight(64, 512, 472)
    X = sbn_synth.adversarial_activations(33, 512, 473)
    check_forward(W, X, 2, 8, s.SBN_PATH_SMFMAC)
    check_forward(W, X, 1, 4, s.SBN_PATH_SMFMAC)


def test_dense_mfma_path_ragged_2of4():
    # 2:4 with an input dimension that is not a whole number of 128-weight chunks: automatic selection
    # takes the dense matrix path (multiple of 64) or the generic kernel
    s = sbn()
    for d_in in (192, 200):
        W = sbn_synth.latent_weight(96, d_in, 460 + d_in)
        X = sbn_synth.activations(50, d_in, 461)
        check_forward(W, X, 2, 4, s.SBN_PATH_AUTO)


def test_grouped_gemv_matches_single():
    s = sbn()
    shapes = [(96, 640), (48, 128), (250, 1792)] * 20        # 60 problems: two launches
    Ws = [sbn_synth.latent_weight(a, b, 600 + i) for i, (a, b) in enumerate(shapes)]
    packs = [hip_pack(W, 2, 4) for W in Ws]
    Xs = {k: sbn_synth.activations(8, k, 700 + k).to(DEV) for k in (640, 128, 1792)}
    X_list = [Xs[b] for _, b in shapes]
    Y_list = [torch.zeros(8, a, dtype=torch.float32, device=DEV) for a, _ in shapes]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, 8, a, b, 2, 4) for a, b in shapes)
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped(X_list, [p for p, _ in packs], [g for _, g in packs], Y_list, 2, 4, ws)
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(shapes):
        Y1, *_ = hip_linear(X_list[i].cpu(), packs[i][0], packs[i][1], a, 2, 4, s.SBN_PATH_GEMV)
        assert np.array_equal(Y_list[i].cpu().numpy(), Y1)


@pytest.mark.parametrize("path_name", ["SBN_PATH_SMFMAC", "SBN_PATH_DENSE_MFMA"])
@pytest.mark.parametrize("tokens,shape", [(16, (256, 256)), (200, (300, 384)), (129, (64, 128)), (513, (520, 640))])
def test_gemm_paths_small(path_name, tokens, shape):
    # several block tiles plus ragged edges in both tokens and rows
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 800 + shape[0])
    X = sbn_synth.activations(tokens, shape[1], 810 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(8))
    check_forward(W, X, 2, 4, getattr(s, path_name), bias=bias)


@pytest.mark.parametrize("path_name", ["SBN_PATH_SMFMAC", "SBN_PATH_DENSE_MFMA"])
def test_gemm_adversarial_inputs(path_name):
    s = sbn()
    W = sbn_synth.adversarial_weight(256, 512, 820)
    X = sbn_synth.adversarial_activations(64, 512, 821)
    check_forward(W, X, 2, 4, getattr(s, path_name))


_CONFIG3_ORACLE = {}


def _config3_oracle(d_out):
    """Oracle forward of configs[2] for one matrix, all 4096 tokens (dense brute-force accumulate), computed once."""
    if d_out not in _CONFIG3_ORACLE:
        W = sbn_synth.latent_weight(d_out, 2560, sbn_synth.seed_for(3, d_out))
        X = sbn_synth.activations(4096, 2560, sbn_synth.seed_for(3, 1))
        _, g, Weff, _ = oracle_pack(W, 2, 4)
        y, acc, xq, sx = oracle.sparse_ternary_linear(X.float().numpy(), Weff, g)
        _CONFIG3_ORACLE[d_out] = (W, X, y, acc, xq, sx)
    return _CONFIG3_ORACLE[d_out]


@pytest.mark.parametrize("path_name", ["SBN_PATH_SMFMAC", "SBN_PATH_DENSE_MFMA"])
@pytest.mark.parametrize("d_out", [2560, 6912])
def test_config3_prefill_gemm_full_size(path_name, d_out):
    # configs[2]: X 4096x2560 against 2560x2560 and 6912x2560, both matrix paths: int8 activations, scales and
    # the int32 accumulators of ALL 4096 token rows bit-exact, every Y within 1e-3
    s = sbn()
    W, X, r_y, r_acc, r_xq, r_sx = _config3_oracle(d_out)
    packed, gamma = hip_pack(W, 2, 4)
    Y, acc, xq, sx = hip_linear(X, packed, gamma, d_out, 2, 4, getattr(s, path_name))
    assert np.array_equal(xq, r_xq) and np.array_equal(sx, r_sx)
    assert np.array_equal(acc, r_acc), f"{(acc != r_acc).sum()} accumulators differ"
    assert_rel(Y, r_y, Y_TOL, "Y")
    # the launch the benchmark times has no accumulator output (whole-row epilogue): same Y, bit for bit
    Y2, *_ = hip_linear(X, packed, gamma, d_out, 2, 4, getattr(s, path_name), want_acc=False)
    assert np.array_equal(Y2, Y)


def test_config3_grouped_step_full_size_as_timed():
    # the launch configuration the benchmark times: one grouped call for X 4096x2560 against 6912x2560 and
    # 2560x2560 (largest first), one quantization, one sparse GEMM launch, whole-row epilogue.
    # Every Y of both outputs against the oracle; Y of the grouped call equals the single calls bit for bit.
    s = sbn()
    shapes = [(6912, 2560), (2560, 2560)]
    refs = [_config3_oracle(a) for a, _ in shapes]
    X = refs[0][1]
    packs = [hip_pack(r[0], 2, 4) for r in refs]
    Xd = X.to(DEV)
    Ys = [torch.full((4096, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    ws = s.new_workspace(sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, 4096, a, b, 2, 4) for a, b in shapes))
    grp = s.LinearGroup([Xd, Xd], [p for p, _ in packs], [g for _, g in packs], Ys, 2, 4, ws, s.SBN_PATH_SMFMAC)
    grp.run()
    grp.run()            # the timed loop calls it back to back on one workspace
    torch.cuda.synchronize()
    for (a, b), ref, (packed, gamma), Y in zip(shapes, refs, packs, Ys):
        assert_rel(Y.cpu().numpy(), ref[2], Y_TOL, f"grouped Y {a}x{b}")
        Y1, *_ = hip_linear(X, packed, gamma, a, 2, 4, s.SBN_PATH_SMFMAC, want_acc=False)
        assert np.array_equal(Y.cpu().numpy(), Y1)


def test_prefill_longest_sequence_sampled_rows():
    # 65536 tokens (the longest prefill of the throughput table, Section 3.2) against 6912x2560: Y holds
    # 453 M values = 1.8 GB, so token offsets pass 2^31 bytes; the rows of the first, the last and 40 sampled
    # tokens are compared with the oracle (each an exact int32 dot product and one rescale)
    s = sbn()
    T, d_out, d_in = 65536, 6912, 2560
    W = sbn_synth.latent_weight(d_out, d_in, sbn_synth.seed_for(3, d_out))
    packed, gamma = hip_pack(W, 2, 4)
    Xd = sbn_synth.activations(T, d_in, sbn_synth.seed_for(3, 9), device=DEV)      # generated on the device: 335 MB
    Y = torch.empty(T, d_out, dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, d_out, d_in, 2, 4))
    s.sbn_sparse_ternary_linear(Xd, packed, gamma, Y, 2, 4, ws, path=s.SBN_PATH_SMFMAC)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 127, 128, T // 2 - 1, T // 2, T - 129, T - 1],
                                     np.random.default_rng(11).choice(T, size=40, replace=False)]))
    idx = torch.from_numpy(rows).to(DEV)
    Xs = Xd[idx].float().cpu().numpy()
    _, g, Weff, _ = oracle_pack(W, 2, 4)
    y, *_ = oracle.sparse_ternary_linear(Xs, Weff, g)
    assert_rel(Y[idx].cpu().numpy(), y, Y_TOL, "Y at 65536 tokens")
    del Y, Xd, ws
    torch.cuda.empty_cache()


def test_sparse_and_dense_paths_agree_bitwise_full_size():
    s = sbn()
    W = sbn_synth.latent_weight(2560, 2560, sbn_synth.seed_for(3, 7))
    X = sbn_synth.activations(4096, 2560, sbn_synth.seed_for(3, 8))
    packed, gamma = hip_pack(W, 2, 4)
    Ya, acca, *_ = hip_linear(X, packed, gamma, 2560, 2, 4, s.SBN_PATH_SMFMAC)
    Yb, accb, *_ = hip_linear(X, packed, gamma, 2560, 2, 4, s.SBN_PATH_DENSE_MFMA)
    assert np.array_equal(acca, accb) and np.array_equal(Ya, Yb)


@pytest.fixture
def spin_limits():
    """Sets the bounds of the library's bounded waits for one test and restores the defaults afterwards."""
    s = sbn()
    yield s.sbn_test_set_spin_limits
    s.sbn_test_set_spin_limits()


@pytest.mark.parametrize("spin_limit", [None, -1, 0])
@pytest.mark.parametrize("tokens", [1, 2, 3, 5, 8, 11, 16])   # a block's own quantizer splits a row over 8, 4, 2 or 1 wavefronts
def test_grouped_streaming_gemv_against_oracle(tokens, spin_limit, spin_limits):
    # enough rows in one grouped call to take the persistent streaming kernel; shapes with ragged
    # row counts and a partial last super-step (K = 768 = 6 chunks).  The kernel quantizes the three
    # inputs itself: its first blocks publish the rows, the others wait for them; spin limit -1 makes
    # every block quantize for itself without looking, 0 allows one look (either branch may run)
    s = sbn()
    if spin_limit is not None:
        spin_limits(gemv_polls=spin_limit)
    shapes = [(4100, 768), (4096, 256), (5000, 640)] * 14
    Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 650 + sh[0]) for sh in set(shapes)}
    packs = {sh: hip_pack(W, 2, 4) for sh, W in Ws.items()}
    Xs = {k: sbn_synth.activations(tokens, k, 750 + k) for k in (768, 256, 640)}
    Xd = {k: x.to(DEV) for k, x in Xs.items()}
    Y_list = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, 2, 4) for a, b in shapes)
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped([Xd[b] for _, b in shapes], [packs[sh][0] for sh in shapes],
                                        [packs[sh][1] for sh in shapes], Y_list, 2, 4, ws, path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    ref = {}
    for sh, W in Ws.items():
        _, g, Weff, _ = oracle_pack(W, 2, 4)
        y, *_ = oracle.sparse_ternary_linear(Xs[sh[1]].float().numpy(), Weff, g)
        ref[sh] = y
    for i, sh in enumerate(shapes):
        assert_rel(Y_list[i].cpu().numpy(), ref[sh], Y_TOL, f"Y of problem {i}")


@pytest.mark.parametrize("N,M", [(2, 4), (8, 8)])
@pytest.mark.parametrize("tokens", [1, 8, 13])
def test_grouped_streaming_rows_that_end_mid_line(tokens, N, M):
    # Input dimensions whose packed rows end 64 bytes past a cache line (22 and 54 chunks of 32 bytes: 2816 and 6912),
    # with more super-steps than the load queue holds (units handed out one at a time) and a partial last super-step;
    # row counts that are no multiple of 32, 16 or 4; every output against the oracle.
    s = sbn()
    shapes = [(2050, 2816), (1030, 6912)] * 32
    Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 2500 + sh[0]) for sh in set(shapes)}
    packs = {sh: hip_pack(W, N, M) for sh, W in Ws.items()}
    Xs = {k: sbn_synth.activations(tokens, k, 2600 + k) for k in (2816, 6912)}
    Xd = {k: x.to(DEV) for k, x in Xs.items()}
    Y_list = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    ws = s.new_workspace(sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, N, M) for a, b in shapes))
    s.sbn_sparse_ternary_linear_grouped([Xd[b] for _, b in shapes], [packs[sh][0] for sh in shapes],
                                        [packs[sh][1] for sh in shapes], Y_list, N, M, ws, path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    ref = {}
    for sh, W in Ws.items():
        _, g, Weff, _ = oracle_pack(W, N, M)
        ref[sh] = oracle.sparse_ternary_linear(Xs[sh[1]].float().numpy(), Weff, g)[0]
    for i, sh in enumerate(shapes):
        assert_rel(Y_list[i].cpu().numpy(), ref[sh], Y_TOL, f"Y of problem {i} {sh}")
        assert_rel(Y_list[i].cpu().numpy(), ref[sh], 2e-6, f"accumulators behind Y of problem {i} {sh}")


def test_streaming_gemv_workspace_reuse_and_many_inputs():
    # (a) the same workspace serves calls with different inputs one after the other: every call
    # must see its own quantized activations; (b) six distinct inputs interleaved over the problems
    # of one call on the streaming kernel, which restages its activations whenever the input changes
    s = sbn()
    tokens = 4
    shapes = [(8192, 512)] * 24
    Ws = [sbn_synth.latent_weight(a, b, 1300 + i) for i, (a, b) in enumerate(shapes)]
    packs = [hip_pack(W, 2, 4) for W in Ws]
    refs = [oracle_pack(W, 2, 4) for W in Ws]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, 2, 4) for a, b in shapes)
    ws = s.new_workspace(need)
    for call in range(3):
        X = sbn_synth.activations(tokens, 512, 1350 + call)
        Xd = X.to(DEV)
        Ys = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
        s.sbn_sparse_ternary_linear_grouped([Xd] * len(shapes), [p for p, _ in packs], [g for _, g in packs], Ys, 2, 4, ws,
                                            path=s.SBN_PATH_GEMV)
        torch.cuda.synchronize()
        for i in (0, 11, 23):
            y, *_ = oracle.sparse_ternary_linear(X.float().numpy(), refs[i][2], refs[i][1])
            assert_rel(Ys[i].cpu().numpy(), y, Y_TOL, f"call {call}, problem {i}")
    Xs = [sbn_synth.activations(tokens, 512, 1400 + i) for i in range(6)]
    Xd = [x.to(DEV) for x in Xs]
    Ys = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    s.sbn_sparse_ternary_linear_grouped([Xd[i % 6] for i in range(len(shapes))], [p for p, _ in packs],
                                        [g for _, g in packs], Ys, 2, 4, ws, path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        y, *_ = oracle.sparse_ternary_linear(Xs[i % 6].float().numpy(), refs[i][2], refs[i][1])
        assert_rel(Ys[i].cpu().numpy(), y, Y_TOL, f"six inputs, problem {i}")


def test_grouped_sparse_gemm_against_oracle():
    # prefill-sized grouped call: all problems take the sparse-MFMA path, their tiles share one launch
    # (ragged token and row counts, two problems sharing one input, more problems than one launch holds)
    s = sbn()
    shapes = [(300, 384), (512, 384), (130, 128), (700, 256), (256, 256), (64, 128), (257, 384), (96, 256), (160, 128), (40, 384)]
    tokens = {384: 200, 128: 33, 256: 130}
    Ws = [sbn_synth.latent_weight(a, b, 900 + i) for i, (a, b) in enumerate(shapes)]
    packs = [hip_pack(W, 2, 4) for W in Ws]
    Xs = {k: sbn_synth.activations(t, k, 950 + k) for k, t in tokens.items()}
    Xd = {k: x.to(DEV) for k, x in Xs.items()}
    Y_list = [torch.full((tokens[b], a), float("nan"), dtype=torch.float32, device=DEV) for a, b in shapes]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens[b], a, b, 2, 4) for a, b in shapes)
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped([Xd[b] for _, b in shapes], [p for p, _ in packs], [g for _, g in packs],
                                        Y_list, 2, 4, ws, path=s.SBN_PATH_SMFMAC)
    torch.cuda.synchronize()
    for i, ((a, b), W) in enumerate(zip(shapes, Ws)):
        _, g, Weff, _ = oracle_pack(W, 2, 4)
        y, *_ = oracle.sparse_ternary_linear(Xs[b].float().numpy(), Weff, g)
        assert_rel(Y_list[i].cpu().numpy(), y, Y_TOL, f"Y of problem {i}")


@pytest.mark.parametrize("N,M", [(2, 4), (8, 8)])
def test_grouped_decode_batches_on_the_gemm_kernel(N, M):
    # Decode batches of 17 .. 512 tokens (the batch sizes of the throughput table, Section 3.2): more problems than one
    # launch of the row-tile work split holds (32), token counts that are no multiple of a token unit, one and several
    # pieces per row tile, ragged last row tiles, one problem with enough tokens for the work-list split in between
    s = sbn()
    tokens_of = [17, 64, 100, 128, 200, 257, 512, 33, 40]
    shapes = [((1100, 256) if i % 3 == 0 else (520, 384) if i % 3 == 1 else (64, 128)) for i in range(38)]
    toks = [tokens_of[i % len(tokens_of)] for i in range(38)]
    toks[20] = 600   # breaks the run of small problems
    Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 2100 + sh[0]) for sh in set(shapes)}
    packs = {sh: hip_pack(W, N, M) for sh, W in Ws.items()}
    refs = {sh: oracle_pack(W, N, M) for sh, W in Ws.items()}
    Xs = {(t, k): sbn_synth.activations(t, k, 2200 + 7 * t + k) for t, (_, k) in set(zip(toks, shapes))}
    Xd = {key: x.to(DEV) for key, x in Xs.items()}
    Y_list = [torch.full((t, a), float("nan"), dtype=torch.float32, device=DEV) for t, (a, _) in zip(toks, shapes)]
    need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, t, a, b, N, M) for t, (a, b) in zip(toks, shapes))
    ws = s.new_workspace(need)
    s.sbn_sparse_ternary_linear_grouped([Xd[(t, sh[1])] for t, sh in zip(toks, shapes)], [packs[sh][0] for sh in shapes],
                                        [packs[sh][1] for sh in shapes], Y_list, N, M, ws, path=s.SBN_PATH_SMFMAC)
    torch.cuda.synchronize()
    done = {}
    for i, (t, sh) in enumerate(zip(toks, shapes)):
        if (t, sh) not in done:
            _, g, Weff, _ = refs[sh]
            done[(t, sh)] = oracle.sparse_ternary_linear(Xs[(t, sh[1])].float().numpy(), Weff, g)[0]
        assert_rel(Y_list[i].cpu().numpy(), done[(t, sh)], Y_TOL, f"Y of problem {i} ({t} tokens, {sh})")


@pytest.mark.parametrize("N,M", [(2, 4), (8, 8), (6, 8)])
def test_grouped_decode_batches_streaming_kernel(N, M):
    # Problems of at most 64 tokens with nothing but Y asked for take the streaming kernel for decode batches: 1 .. 64 tokens (two and four token tiles in separate launches), strips of 128 and of
    # 256 rows (second call: enough rows for the wide strips), ragged last strips, an input dimension that is no
    # multiple of a super-step (768 = 6 chunks), problems that share an input and problems that do not
    s = sbn()
    for reps in (1, 4):
        tokens_of = [17, 64, 33, 20, 48, 32, 1, 16]
        base = [(1100, 256), (520, 384), (4100, 768), (2052, 128)]
        shapes = [base[i % 4] for i in range(10 * reps)]
        toks = [tokens_of[i % len(tokens_of)] for i in range(len(shapes))]
        Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 2300 + sh[0]) for sh in set(shapes)}
        packs = {sh: hip_pack(W, N, M) for sh, W in Ws.items()}
        refs = {sh: oracle_pack(W, N, M) for sh, W in Ws.items()}
        Xs = {(t, k): sbn_synth.activations(t, k, 2400 + 7 * t + k) for t, (_, k) in set(zip(toks, shapes))}
        Xd = {key: x.to(DEV) for key, x in Xs.items()}
        Y_list = [torch.full((t, a), float("nan"), dtype=torch.float32, device=DEV) for t, (a, _) in zip(toks, shapes)]
        need = sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, t, a, b, N, M) for t, (a, b) in zip(toks, shapes))
        ws = s.new_workspace(need)
        s.sbn_sparse_ternary_linear_grouped([Xd[(t, sh[1])] for t, sh in zip(toks, shapes)], [packs[sh][0] for sh in shapes],
                                            [packs[sh][1] for sh in shapes], Y_list, N, M, ws, path=s.SBN_PATH_SMFMAC)
        torch.cuda.synchronize()
        done = {}
        for i, (t, sh) in enumerate(zip(toks, shapes)):
            if (t, sh) not in done:
                _, g, Weff, _ = refs[sh]
                done[(t, sh)] = oracle.sparse_ternary_linear(Xs[(t, sh[1])].float().numpy(), Weff, g)[0]
            assert_rel(Y_list[i].cpu().numpy(), done[(t, sh)], Y_TOL, f"Y of problem {i} ({t} tokens, {sh}), {reps}")
            # this kernel has no accumulator output; Y within 1e-6 relative says the same: one unit of an accumulator
            # is more than 2e-5 of |Y| at these input dimensions, the fp32 rescale errs by less than 2e-7
            assert_rel(Y_list[i].cpu().numpy(), done[(t, sh)], 1e-6, f"accumulators behind Y of problem {i} ({t} tokens, {sh}), {reps}")


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4)])
@pytest.mark.parametrize("tokens,shape", [(8, (6912, 2560)), (1, (2560, 6912))])
def test_config2_streaming_decode_full_size_as_timed(tokens, shape, N, M):
    # the launch configuration the benchmark times for decode: independently seeded copies of a full-size
    # matrix in one grouped call on the persistent streaming kernel (20 copies: enough rows to select it),
    # every output of every copy against the oracle; 2:4 and the 1:4 form the kernel reads as stored
    s = sbn()
    a, b = shape
    R = 20
    Ws = [sbn_synth.latent_weight(a, b, sbn_synth.seed_for(2, 100 * r + a % 7)) for r in range(R)]
    packs = [hip_pack(W, N, M) for W in Ws]
    X = sbn_synth.activations(tokens, b, sbn_synth.seed_for(2, tokens))
    Xd = X.to(DEV)
    Ys = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for _ in range(R)]
    ws = s.new_workspace(R * s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, N, M))
    s.sbn_sparse_ternary_linear_grouped([Xd] * R, [p for p, _ in packs], [g for _, g in packs], Ys, N, M, ws,
                                        path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    Xf = X.float().numpy()
    for r in range(R):
        _, g, Weff, _ = oracle_pack(Ws[r], N, M)
        y, *_ = oracle.sparse_ternary_linear(Xf, Weff, g)
        assert_rel(Ys[r].cpu().numpy(), y, Y_TOL, f"Y of copy {r}")


@pytest.mark.parametrize("tokens", [1, 5, 64, 65, 300])
@pytest.mark.parametrize("d_in", [8, 256, 2560, 6912, 8200, 16520])
def test_act_quant_entry_all_kernel_variants(tokens, d_in):
    # a block per token (1024 threads: decode; 256 threads with two or four vectors per thread: prefill) and the
    # two-pass kernel for very long rows
    s = sbn()
    X = sbn_synth.adversarial_activations(tokens, d_in, 840 + tokens) if d_in >= 256 else sbn_synth.activations(tokens, d_in, 841)
    xq = torch.full((tokens, d_in), 77, dtype=torch.int8, device=DEV)
    sx = torch.zeros(tokens, dtype=torch.float32, device=DEV)
    s.sbn_act_quant(X.to(DEV), xq, sx)
    torch.cuda.synchronize()
    r_xq, r_sx = oracle.act_quant(X.float().numpy())
    assert np.array_equal(xq.cpu().numpy(), r_xq) and np.array_equal(sx.cpu().numpy(), r_sx)


@pytest.mark.parametrize("tokens,shape", [(200, (512, 384)), (4096, (2560, 2560)), (130, (768, 128))])
def test_gemm_sparse_without_accumulator_output(tokens, shape):
    # without acc_out the sparse GEMM takes its LDS-transposed full-row epilogue: same Y, bias included
    s = sbn()
    W = sbn_synth.latent_weight(shape[0], shape[1], 860 + shape[0])
    X = sbn_synth.activations(tokens, shape[1], 861 + tokens)
    bias = torch.randn(shape[0], generator=torch.Generator().manual_seed(9))
    packed, gamma = hip_pack(W, 2, 4)
    Y_ref, *_ = hip_linear(X, packed, gamma, shape[0], 2, 4, s.SBN_PATH_SMFMAC, bias)
    Y, *_ = hip_linear(X, packed, gamma, shape[0], 2, 4, s.SBN_PATH_SMFMAC, bias, want_acc=False)
    assert np.array_equal(Y, Y_ref)
    _, g, Weff, _ = oracle_pack(W, 2, 4)
    rows = np.unique(np.random.default_rng(1).choice(tokens, size=min(tokens, 48), replace=False))
    # with a bias the sum can cancel, so the bound is taken relative to the two terms, not to their sum
    y_nb, *_ = oracle.sparse_ternary_linear(X.float().numpy(), Weff, g)
    ref = y_nb[rows] + bias.numpy().astype(np.float64)
    assert (np.abs(Y[rows] - ref) <= 1e-3 * (np.abs(y_nb[rows]) + np.abs(bias.numpy()))).all()


@pytest.mark.parametrize("N,M,to", [(6, 8, (8, 8)), (3, 8, (8, 8)), (3, 4, (4, 4)), (2, 8, (2, 4)), (1, 4, (2, 4)), (1, 8, (8, 8)), (2, 4, (4, 4))])
def test_convert_packed_once_then_decode(N, M, to):
    # weights rewritten once into a form the decode kernel streams as stored: the rewritten matrix unpacks to
    # the oracle's W_eff, and the layer on it (pattern = the target's) gives the oracle's integers and Y
    s = sbn()
    d_out, d_in, tokens = 200, 640, 8
    W = sbn_synth.latent_weight(d_out, d_in, 1600 + 10 * N + M)
    X = sbn_synth.activations(tokens, d_in, 1601)
    packed, gamma = hip_pack(W, N, M)
    _, ref_gamma, Weff, _ = oracle_pack(W, N, M)
    conv = torch.full((s.sbn_packed_bytes(d_out, d_in, *to),), 0xA5, dtype=torch.uint8, device=DEV)
    s.sbn_convert_packed(packed, d_out, d_in, N, M, to[0], to[1], conv)
    We = torch.full((d_out, d_in), 9, dtype=torch.int8, device=DEV)
    s.sbn_unpack(conv, d_out, d_in, to[0], to[1], We, None)
    assert np.array_equal(We.cpu().numpy(), Weff)
    Y, acc, xq, sx = hip_linear(X, conv, gamma, d_out, to[0], to[1], s.SBN_PATH_GEMV)
    r_xq, r_sx = oracle.act_quant(X.float().numpy())
    r_acc = oracle.acc(Weff, r_xq)
    assert np.array_equal(acc, r_acc)
    assert_rel(Y, oracle.rescale(r_acc, ref_gamma, r_sx, None), Y_TOL, "Y")


def test_convert_packed_6of8_full_size_streaming():
    # the paper's main pattern, decode shape of configs[1], converted once and streamed in one grouped call
    s = sbn()
    a, b, tokens, R = 6912, 2560, 8, 20
    Ws = [sbn_synth.latent_weight(a, b, sbn_synth.seed_for(2, 680 + r)) for r in range(R)]
    X = sbn_synth.activations(tokens, b, sbn_synth.seed_for(2, 688))
    convs, gammas = [], []
    for W in Ws:
        packed, gamma = hip_pack(W, 6, 8)
        conv = torch.empty(s.sbn_packed_bytes(a, b, 8, 8), dtype=torch.uint8, device=DEV)
        s.sbn_convert_packed(packed, a, b, 6, 8, 8, 8, conv)
        convs.append(conv)
        gammas.append(gamma)
    Ys = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for _ in range(R)]
    ws = s.new_workspace(R * s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, 8, 8))
    s.sbn_sparse_ternary_linear_grouped([X.to(DEV)] * R, convs, gammas, Ys, 8, 8, ws, path=s.SBN_PATH_GEMV)
    torch.cuda.synchronize()
    Xf = X.float().numpy()
    for r in (0, 7, 19):
        _, g, Weff, _ = oracle_pack(Ws[r], 6, 8)
        y, *_ = oracle.sparse_ternary_linear(Xf, Weff, g)
        assert_rel(Ys[r].cpu().numpy(), y, Y_TOL, f"Y of copy {r}")


@pytest.mark.parametrize("tokens,d_out", [(7000, 2560), (6980, 2500)])
def test_sparse_gemm_more_tiles_than_block_slots_ragged(tokens, d_out):
    # more tiles than the device has block slots (a second, partial round of blocks), ragged last token
    # tile, ragged rows; accumulators bit-exact on sampled tokens from both ends and the middle
    s = sbn()
    W = sbn_synth.latent_weight(d_out, 256, 2000 + d_out)
    X = sbn_synth.activations(tokens, 256, 2001)
    sample = np.unique(np.concatenate([np.arange(0, 200), np.arange(tokens - 400, tokens), np.arange(3000, 3100)]))
    check_forward(W, X, 2, 4, s.SBN_PATH_SMFMAC, token_sample=sample)


def test_streaming_decode_alternating_weight_forms_on_one_workspace():
    # 2:4 weights (sparse instruction) and dense 2-bit codes (N = M) are two instantiations of the streaming kernel;
    # alternating grouped calls on ONE workspace, with the same token and row layout and a different X every call,
    # leave each other's per-token flags behind: every call must wait for its own producers and see its own x~
    s = sbn()
    tokens, R = 8, 20
    shape = (6912, 512)
    Ws = [sbn_synth.latent_weight(shape[0], shape[1], 2100 + r) for r in range(R)]
    forms = {(2, 4): [hip_pack(W, 2, 4) for W in Ws], (8, 8): [hip_pack(W, 8, 8) for W in Ws]}
    refs = {nm: [oracle_pack(W, *nm) for W in Ws] for nm in forms}
    ws = s.new_workspace(R * max(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, shape[0], shape[1], n, m) for n, m in forms))
    for call in range(6):
        nm = (2, 4) if call % 2 == 0 else (8, 8)
        X = sbn_synth.activations(tokens, shape[1], 2150 + call)
        Xd = X.to(DEV)
        Ys = [torch.full((tokens, shape[0]), float("nan"), dtype=torch.float32, device=DEV) for _ in range(R)]
        s.sbn_sparse_ternary_linear_grouped([Xd] * R, [p for p, _ in forms[nm]], [g for _, g in forms[nm]], Ys, nm[0], nm[1], ws,
                                            path=s.SBN_PATH_GEMV)
        torch.cuda.synchronize()
        Xf = X.float().numpy()
        for r in range(R):
            y, *_ = oracle.sparse_ternary_linear(Xf, refs[nm][r][2], refs[nm][r][1])
            assert_rel(Ys[r].cpu().numpy(), y, Y_TOL, f"call {call} ({nm[0]}:{nm[1]}), copy {r}")
