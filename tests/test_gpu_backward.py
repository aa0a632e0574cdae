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


def _forward_state(W, X, N, M):
    s = sbn()
    d_out, d_in = W.shape
    T = X.shape[0]
    packed, gamma = hip_pack(W, N, M)
    Y = torch.empty(T, d_out, dtype=torch.float32, device=DEV)
    xq = torch.empty(T, d_in, dtype=torch.int8, device=DEV)
    sx = torch.empty(T, dtype=torch.float32, device=DEV)
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, d_out, d_in, N, M))
    s.sbn_sparse_ternary_linear(X.to(DEV), packed, gamma, Y, N, M, ws, xq_out=xq, sx_out=sx)
    return packed, gamma, xq, sx


@pytest.mark.parametrize("N,M", [(2, 4), (6, 8)])
@pytest.mark.parametrize("tokens,d_in,d_outs,share", [(192, 256, (256, 320, 256), True), (77, 136, (104, 520), True),
                                                      (130, 392, (520, 136, 264, 128), False)])
def test_backward_grouped_matches_single_calls_and_oracle(N, M, tokens, d_in, d_outs, share):
    # several layers in one call (Q/K/V or up/gate share the quantized input: one transpose serves them);
    # per layer the outputs equal those of the single call bit for bit, and the oracle within tolerance
    s = sbn()
    n = len(d_outs)
    X = [sbn_synth.activations(tokens, d_in, 960 + (0 if share else i)) for i in range(n)]
    W = [sbn_synth.latent_weight(d_outs[i], d_in, 970 + i) for i in range(n)]
    dY = [sbn_synth.grad_output(tokens, d_outs[i], 980 + i).to(DEV) for i in range(n)]
    st = []
    for i in range(n):
        if share and i > 0:
            packed, gamma = hip_pack(W[i], N, M)
            st.append((packed, gamma, st[0][2], st[0][3]))      # the same xq / sx tensors as layer 0
        else:
            st.append(_forward_state(W[i], X[i], N, M))
    nan = float("nan")
    dX = [torch.full((tokens, d_in), nan, dtype=torch.bfloat16, device=DEV) for _ in range(n)]
    dW = [torch.full((d_outs[i], d_in), nan, dtype=torch.bfloat16, device=DEV) for i in range(n)]
    dX[-1] = None                                               # one layer asks for dW only
    ws = s.new_workspace(sum(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, tokens, d, d_in, N, M) for d in d_outs))
    s.sbn_sparse_ternary_linear_backward_grouped(dY, [t[0] for t in st], [t[1] for t in st], [t[2] for t in st],
                                                 [t[3] for t in st], N, M, ws, [d_in] * n, dX, dW)
    torch.cuda.synchronize()
    for i in range(n):
        sX = torch.full((tokens, d_in), nan, dtype=torch.bfloat16, device=DEV) if dX[i] is not None else None
        sW = torch.full((d_outs[i], d_in), nan, dtype=torch.bfloat16, device=DEV)
        ws1 = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, tokens, d_outs[i], d_in, N, M))
        s.sbn_sparse_ternary_linear_backward(dY[i], st[i][0], st[i][1], st[i][2], st[i][3], N, M, ws1, d_in, dX=sX, dW=sW)
        torch.cuda.synchronize()
        assert torch.equal(dW[i].view(torch.int16), sW.view(torch.int16))
        if sX is not None:
            assert torch.equal(dX[i].view(torch.int16), sX.view(torch.int16))
        _, gamma, Weff, _ = oracle_pack(W[i], N, M)
        r_dw = oracle.backward_dw(dY[i].float().cpu().numpy(), st[i][2].cpu().numpy(), st[i][3].cpu().numpy())
        assert_rel_rms(dW[i].float().cpu().numpy(), r_dw, BWD_TOL, f"grouped dW {i}")
        if dX[i] is not None:
            assert_rel_rms(dX[i].float().cpu().numpy(), oracle.backward_dx(dY[i].float().cpu().numpy(), Weff, gamma), BWD_TOL,
                           f"grouped dX {i}")


def test_backward_grouped_more_products_than_one_launch_holds():
    # five layers = ten products: two matrix-multiply launches; accumulate flag applies to every layer
    s = sbn()
    tokens, d_in, n = 64, 128, 5
    X = sbn_synth.activations(tokens, d_in, 990)
    W = [sbn_synth.latent_weight(64 + 8 * i, d_in, 991 + i) for i in range(n)]
    dY = [sbn_synth.grad_output(tokens, 64 + 8 * i, 996 + i).to(DEV) for i in range(n)]
    st0 = _forward_state(W[0], X, 2, 4)
    st = [st0] + [hip_pack(W[i], 2, 4) + (st0[2], st0[3]) for i in range(1, n)]
    base = [(torch.randn(64 + 8 * i, d_in, generator=torch.Generator().manual_seed(i)) * 0.1).to(torch.bfloat16) for i in range(n)]
    dW = [b.clone().to(DEV) for b in base]
    dX = [torch.empty(tokens, d_in, dtype=torch.bfloat16, device=DEV) for _ in range(n)]
    ws = s.new_workspace(sum(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, tokens, 64 + 8 * i, d_in, 2, 4) for i in range(n)))
    s.sbn_sparse_ternary_linear_backward_grouped(dY, [t[0] for t in st], [t[1] for t in st], [t[2] for t in st],
                                                 [t[3] for t in st], 2, 4, ws, [d_in] * n, dX, dW, accumulate=True)
    torch.cuda.synchronize()
    xq, sx = st0[2].cpu().numpy(), st0[3].cpu().numpy()
    for i in range(n):
        _, gamma, Weff, _ = oracle_pack(W[i], 2, 4)
        r_dw = oracle.backward_dw(dY[i].float().cpu().numpy(), xq, sx) + base[i].float().numpy().astype(np.float64)
        assert_rel_rms(dW[i].float().cpu().numpy(), r_dw, BWD_TOL, f"dW {i}")
        assert_rel_rms(dX[i].float().cpu().numpy(), oracle.backward_dx(dY[i].float().cpu().numpy(), Weff, gamma), BWD_TOL, f"dX {i}")


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


def test_config5_training_step_as_timed():
    # configs[4] in the launch configuration the benchmark times: per step the seven matrices of a block are
    # remasked in one batched call, each of the block's four distinct inputs is quantized once, the seven forwards
    # run on the shared int8 copies, and the backward runs as four grouped calls (down; up+gate; O; Q+K+V).
    # Integers in full (packed bytes, gamma, int8 activations, scales); Y and dX on sampled token rows, dW on
    # sampled weight rows against the fp64 oracle; the grouped calls equal the single calls bit for bit.
    s = sbn()
    N, M, T = 2, 4, 8 * 2048
    H, F = sbn_synth.HIDDEN, sbn_synth.FFN
    mats = sbn_synth.BLOCK_MATRICES
    rng = np.random.default_rng(55)
    Wt = [sbn_synth.latent_weight(a, b, sbn_synth.seed_for(5, i)) for i, (_, a, b) in enumerate(mats)]
    inputs = [sbn_synth.activations(T, H, sbn_synth.seed_for(5, 20)), sbn_synth.activations(T, H, sbn_synth.seed_for(5, 21)),
              sbn_synth.activations(T, H, sbn_synth.seed_for(5, 23)), sbn_synth.activations(T, F, sbn_synth.seed_for(5, 22))]
    input_of = [0, 0, 0, 1, 2, 2, 3]
    dYh = sbn_synth.grad_output(T, H, sbn_synth.seed_for(5, 30))
    dYf = sbn_synth.grad_output(T, F, sbn_synth.seed_for(5, 31))
    Wd = [w.to(DEV) for w in Wt]
    Xd = [x.to(DEV) for x in inputs]
    dYd = {H: dYh.to(DEV), F: dYf.to(DEV)}
    pk = [torch.full((s.sbn_packed_bytes(a, b, N, M),), 0xAA, dtype=torch.uint8, device=DEV) for _, a, b in mats]
    gm = torch.zeros(len(mats), dtype=torch.float32, device=DEV)
    gl = [gm[i:i + 1] for i in range(len(mats))]
    wsp = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(mats), F, H, N, M))
    nan = float("nan")
    Yl = [torch.full((T, a), nan, dtype=torch.float32, device=DEV) for _, a, b in mats]
    xql = [torch.zeros(T, x.shape[1], dtype=torch.int8, device=DEV) for x in inputs]
    sxl = [torch.zeros(T, dtype=torch.float32, device=DEV) for _ in inputs]
    dXl = [torch.full((T, b), nan, dtype=torch.bfloat16, device=DEV) for _, a, b in mats]
    dWl = [torch.full((a, b), nan, dtype=torch.bfloat16, device=DEV) for _, a, b in mats]
    wsl = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, F, F, N, M))
    batch = s.PackBatch(Wd, N, M, pk, gl, wsp)
    groups = []
    for idx in ([6], [4, 5], [3], [0, 1, 2]):
        wsg = s.new_workspace(sum(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, T, mats[i][1], mats[i][2], N, M) for i in idx))
        groups.append(s.BackwardGroup([dYd[mats[i][1]] for i in idx], [pk[i] for i in idx], [gl[i] for i in idx],
                                      [xql[input_of[i]] for i in idx], [sxl[input_of[i]] for i in idx], N, M, wsg,
                                      [mats[i][2] for i in idx], [dXl[i] for i in idx], [dWl[i] for i in idx]))
    for _ in range(2):   # two steps back to back on the same buffers and workspaces, as the timed loop does
        batch.run()
        for j, x in enumerate(Xd):
            s.sbn_act_quant(x, xql[j], sxl[j])
        for i in range(len(mats)):
            j = input_of[i]
            s.sbn_sparse_ternary_linear(None, pk[i], gl[i], Yl[i], N, M, wsl, xq_out=xql[j], sx_out=sxl[j], path=s.SBN_PATH_SMFMAC)
        for grp in groups:
            grp.run()
    torch.cuda.synchronize()

    refs = [oracle_pack(W, N, M) for W in Wt]                     # (packed, gamma, W_eff, mask)
    for i in range(len(mats)):
        assert gm[i].item() == refs[i][1], f"gamma of {mats[i][0]}"
        assert np.array_equal(pk[i].cpu().numpy(), refs[i][0]), f"packed bytes of {mats[i][0]}"
    quant = [oracle.act_quant(x.float().numpy()) for x in inputs]
    for j in range(len(inputs)):
        assert np.array_equal(xql[j].cpu().numpy(), quant[j][0]) and np.array_equal(sxl[j].cpu().numpy(), quant[j][1])
    trow = np.unique(np.concatenate([[0, 127, 128, T - 1], rng.choice(T, 20, replace=False)]))
    tsel = torch.from_numpy(trow).to(DEV)
    wsb = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, T, F, F, N, M))
    for i, (name, a, b) in enumerate(mats):
        _, gamma, Weff, _ = refs[i]
        r_xq, r_sx = quant[input_of[i]]
        dY = dYf if a == F else dYh
        # forward on the shared int8 copy
        r_acc = oracle.acc(Weff, r_xq[trow])
        r_y = oracle.rescale(r_acc, gamma, r_sx[trow], None)
        got = Yl[i][tsel].cpu().numpy()
        assert (np.abs(got - r_y) <= 1e-3 * np.abs(r_y)).all(), f"Y of {name}"
        # dX on sampled token rows, dW on sampled weight rows
        r_dx = oracle.backward_dx(np.ascontiguousarray(dY[trow].float().numpy()), Weff, gamma)
        assert_rel_rms(dXl[i][tsel].float().cpu().numpy(), r_dx, BWD_TOL, f"dX of {name}")
        orow = np.unique(np.concatenate([[0, a - 1], rng.choice(a, 4, replace=False)]))
        r_dw = oracle.backward_dw(np.ascontiguousarray(dY[:, orow].float().numpy()), r_xq, r_sx)
        assert_rel_rms(dWl[i][torch.from_numpy(orow).to(DEV)].float().cpu().numpy(), r_dw, BWD_TOL, f"dW of {name}")
        # the same layer through the single backward call: identical bits
        sX = torch.full((T, b), nan, dtype=torch.bfloat16, device=DEV)
        sW = torch.full((a, b), nan, dtype=torch.bfloat16, device=DEV)
        s.sbn_sparse_ternary_linear_backward(dYd[a], pk[i], gl[i], xql[input_of[i]], sxl[input_of[i]], N, M, wsb, b, dX=sX, dW=sW)
        torch.cuda.synchronize()
        assert torch.equal(dXl[i].view(torch.int16), sX.view(torch.int16)), f"grouped dX of {name} differs from the single call"
        assert torch.equal(dWl[i].view(torch.int16), sW.view(torch.int16)), f"grouped dW of {name} differs from the single call"
        del sX, sW
    torch.cuda.empty_cache()
