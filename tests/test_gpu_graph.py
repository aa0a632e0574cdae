"""Calls recorded into a HIP graph and replayed: every replay must give what the eager call gives on the
inputs the buffers hold at that moment.  The library enqueues kernels only (no copies, no memsets), its
descriptor tables travel as kernel arguments and the counters of its persistent kernels are cleared by
kernels, so a replay repeats the whole call; the decode kernel that numbers its launches on the host is
replaced by its plain form while a stream captures.  Between the replays the test runs eager work of its
own and synchronizes, and every replay is checked against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import sbn_synth
from gpu_util import DEV, assert_rel, assert_rel_rms, hip_pack, oracle_pack, sbn

pytestmark = pytest.mark.gpu
Y_TOL = 1e-3
BWD_TOL = 2e-2


def _capture(fn):
    fn()                                  # first use outside capture: function attributes, device queries
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


@pytest.mark.parametrize("tokens", [1, 8, 32, 100])
def test_replayed_streaming_decode_follows_its_inputs(tokens):
    # enough rows for the persistent streaming kernel; the activations change between the replays
    # (32 tokens: the streaming kernel for decode batches; 100: the sparse GEMM kernel with its work dealt by row tile)
    s = sbn()
    shapes = [(4096, 512), (6144, 512)] * 16
    Ws = {sh: sbn_synth.latent_weight(sh[0], sh[1], 1500 + sh[0]) for sh in set(shapes)}
    packs = {sh: hip_pack(W, 2, 4) for sh, W in Ws.items()}
    refs = {sh: oracle_pack(W, 2, 4) for sh, W in Ws.items()}
    X = torch.zeros(tokens, 512, dtype=torch.bfloat16, device=DEV)
    Ys = [torch.full((tokens, a), float("nan"), dtype=torch.float32, device=DEV) for a, _ in shapes]
    ws = s.new_workspace(sum(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, tokens, a, b, 2, 4) for a, b in shapes))
    grp = s.LinearGroup([X] * len(shapes), [packs[sh][0] for sh in shapes], [packs[sh][1] for sh in shapes], Ys, 2, 4, ws,
                        s.SBN_PATH_GEMV if tokens <= 16 else s.SBN_PATH_AUTO)
    X.copy_(sbn_synth.activations(tokens, 512, 1510).to(DEV))
    graph = _capture(grp.run)
    for replay in range(4):
        Xh = sbn_synth.activations(tokens, 512, 1520 + replay)
        X.copy_(Xh.to(DEV))
        for y in Ys:
            y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i in (0, 1, len(shapes) - 1):
            sh = shapes[i]
            y, *_ = oracle.sparse_ternary_linear(Xh.float().numpy(), refs[sh][2], refs[sh][1])
            assert_rel(Ys[i].cpu().numpy(), y, Y_TOL, f"replay {replay}, problem {i}")
    # the eager call afterwards (fused quantizer again) on the same workspace
    Xh = sbn_synth.activations(tokens, 512, 1530)
    X.copy_(Xh.to(DEV))
    grp.run()
    torch.cuda.synchronize()
    y, *_ = oracle.sparse_ternary_linear(Xh.float().numpy(), refs[shapes[0]][2], refs[shapes[0]][1])
    assert_rel(Ys[0].cpu().numpy(), y, Y_TOL, "eager after replays")


def test_replayed_training_step_follows_its_inputs():
    # remask + forward + backward of one layer in one graph; weights, activations and gradients change between replays
    s = sbn()
    T, d_out, d_in, N, M = 192, 256, 384, 2, 4
    W = torch.zeros(d_out, d_in, dtype=torch.bfloat16, device=DEV)
    X = torch.zeros(T, d_in, dtype=torch.bfloat16, device=DEV)
    dY = torch.zeros(T, d_out, dtype=torch.bfloat16, device=DEV)
    packed = torch.zeros(s.sbn_packed_bytes(d_out, d_in, N, M), dtype=torch.uint8, device=DEV)
    gamma = torch.zeros(1, dtype=torch.float32, device=DEV)
    Y = torch.zeros(T, d_out, dtype=torch.float32, device=DEV)
    xq = torch.zeros(T, d_in, dtype=torch.int8, device=DEV)
    sx = torch.zeros(T, dtype=torch.float32, device=DEV)
    dX = torch.zeros(T, d_in, dtype=torch.bfloat16, device=DEV)
    dW = torch.zeros(d_out, d_in, dtype=torch.bfloat16, device=DEV)
    wsp = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, 1, d_out, d_in, N, M))
    wsl = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_LINEAR, T, d_out, d_in, N, M))
    wsb = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_BACKWARD, T, d_out, d_in, N, M))

    def step():
        s.sbn_quantize_mask_pack(W, N, M, packed, gamma, wsp)
        s.sbn_sparse_ternary_linear(X, packed, gamma, Y, N, M, wsl, xq_out=xq, sx_out=sx)
        s.sbn_sparse_ternary_linear_backward(dY, packed, gamma, xq, sx, N, M, wsb, d_in, dX=dX, dW=dW)

    W.copy_(sbn_synth.latent_weight(d_out, d_in, 1600).to(DEV))
    X.copy_(sbn_synth.activations(T, d_in, 1601).to(DEV))
    graph = _capture(step)
    for replay in range(3):
        Wh = sbn_synth.latent_weight(d_out, d_in, 1610 + replay)
        Xh = sbn_synth.activations(T, d_in, 1620 + replay)
        dYh = sbn_synth.grad_output(T, d_out, 1630 + replay)
        W.copy_(Wh.to(DEV)); X.copy_(Xh.to(DEV)); dY.copy_(dYh.to(DEV))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_packed, g, Weff, _ = oracle_pack(Wh, N, M)
        assert gamma.item() == g and np.array_equal(packed.cpu().numpy(), ref_packed)
        y, _, r_xq, r_sx = oracle.sparse_ternary_linear(Xh.float().numpy(), Weff, g)
        assert np.array_equal(xq.cpu().numpy(), r_xq) and np.array_equal(sx.cpu().numpy(), r_sx)
        assert_rel(Y.cpu().numpy(), y, Y_TOL, f"Y, replay {replay}")
        assert_rel_rms(dX.float().cpu().numpy(), oracle.backward_dx(dYh.float().numpy(), Weff, g), BWD_TOL, f"dX, replay {replay}")
        assert_rel_rms(dW.float().cpu().numpy(), oracle.backward_dw(dYh.float().numpy(), r_xq, r_sx), BWD_TOL, f"dW, replay {replay}")


def test_replayed_single_read_pack_sweep():
    # the persistent pack kernel exchanges partial sums and ready words through the workspace: a kernel of the
    # same call clears them, so a replay starts clean
    s = sbn()
    shapes = [(1024, 512), (2048, 1024), (512, 2048), (1024, 512)]
    Ws = [torch.zeros(a, b, dtype=torch.bfloat16, device=DEV) for a, b in shapes]
    pk = [torch.zeros(s.sbn_packed_bytes(a, b, 2, 4), dtype=torch.uint8, device=DEV) for a, b in shapes]
    gm = [torch.zeros(1, dtype=torch.float32, device=DEV) for _ in shapes]
    ws = s.new_workspace(s.sbn_workspace_bytes(s.SBN_OP_QUANTIZE_MASK_PACK, len(shapes), 2048, 2048, 2, 4))
    batch = s.PackBatch(Ws, 2, 4, pk, gm, ws)
    for i, (a, b) in enumerate(shapes):
        Ws[i].copy_(sbn_synth.latent_weight(a, b, 1700 + i).to(DEV))
    graph = _capture(batch.run)
    for replay in range(3):
        hosts = [sbn_synth.latent_weight(a, b, 1710 + 10 * replay + i) for i, (a, b) in enumerate(shapes)]
        for w, h in zip(Ws, hosts):
            w.copy_(h.to(DEV))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, h in enumerate(hosts):
            ref_packed, g, *_ = oracle_pack(h, 2, 4)
            assert gm[i].item() == g, f"gamma of matrix {i}, replay {replay}"
            assert np.array_equal(pk[i].cpu().numpy(), ref_packed), f"packed bytes of matrix {i}, replay {replay}"
