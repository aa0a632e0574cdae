#!/usr/bin/env python3
"""Benchmark of the MI355X-native N:M-sparse ternary linear layer (one GPU).

A timed "step" is the prefill workload of benchmark configs[2]: X 4096x2560 bf16 through
sbn_sparse_ternary_linear (activation quantizer + sparse-MFMA GEMM + rescale) against the packed
2:4 ternary matrices 2560x2560 and 6912x2560.  `value` is its dense-equivalent throughput
2*T*K*d_out / time in TOPS.  The other rows of the hot path are measured in the same run and
reported under "rows": decode GEMV streaming rate (configs[1]), the quantize_mask_pack sweep
(configs[3]), one block's training step (configs[4]) and the dense-ternary comparison path.
Prints exactly one JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
INT8_DENSE_PEAK_TOPS = 5000.0   # dense int8 MFMA; the sparse instruction runs the same executed-op rate
BF16_DENSE_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(kernel, workload):
    """HBM bytes per launch (fetch + write) from the rocprofv3 --pmc summary committed under profiles/
    (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain copy), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 5 and f[0] == "TRAFFIC" and f[1] == kernel and f[2] == workload:
                return float(f[3]) + float(f[4])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--sections", default="gemm,gemv,pack,train,dense,seq,ceil,cpu",
                    help="comma list of: gemm (always timed), gemv, pack, train, dense, ceil, cpu, copyref")
    ap.add_argument("--only", default="",
                    help="counter runs only: restrict the prefill shapes to one (e.g. 6912x2560) and/or the decode "
                         "workloads to one (e.g. down_2560x6912_T8), so that every dispatch of a persistent kernel "
                         "in the run is the same workload (their grids do not tell them apart)")
    args = ap.parse_args()
    only = set(x for x in args.only.split(",") if x)
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (across GPUs the layer would shard by rows of W, with "
            "one scalar all-reduce for the weight scale); run with --gpus 1")
        sys.exit(2)
    sections = set(args.sections.split(","))

    import torch
    import paper_2603_05168_amd as sbn
    import sbn_synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    N, M = 2, 4
    H, F = sbn_synth.HIDDEN, sbn_synth.FFN

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def ramp(fn, seconds=0.2):
        """Untimed calls of fn for a fixed wall time: the GPU leaves its idle clock state only under
        sustained load (measured here: the first ~50 ms after an idle gap run 10-15 % slower)."""
        t_end = time.perf_counter() + seconds
        while time.perf_counter() < t_end:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()

    def timed(fn, reps, warm=2):
        """Average milliseconds per call of fn over reps back-to-back calls (HIP events on the launch stream)."""
        ramp(fn)
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def pack_one(W, n=N, m=M):
        d_out, d_in = W.shape
        packed = torch.empty(sbn.sbn_packed_bytes(d_out, d_in, n, m), dtype=torch.uint8, device=dev)
        gamma = torch.empty(1, dtype=torch.float32, device=dev)
        ws = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_QUANTIZE_MASK_PACK, 1, d_out, d_in, n, m), dev)
        sbn.sbn_quantize_mask_pack(W, n, m, packed, gamma, ws)
        return packed, gamma

    out = {}
    rows = {}

    # ------------------------------------------------------------------ configs[2]: prefill GEMM (the timed step)
    T = 4096
    NSETS = 4
    shapes = [(a, b) for a, b in [(H, H), (F, H)] if not only & {"2560x2560", "6912x2560"} or f"{a}x{b}" in only]
    Wp = [pack_one(sbn_synth.latent_weight(a, b, sbn_synth.seed_for(3, a), device=dev)) for a, b in shapes]
    Xs = [sbn_synth.activations(T, H, sbn_synth.seed_for(3, 10 + i), device=dev) for i in range(NSETS)]
    Ys = [[torch.empty(T, a, dtype=torch.float32, device=dev) for a, _ in shapes] for _ in range(NSETS)]
    xq = [torch.empty(T, H, dtype=torch.int8, device=dev) for _ in range(NSETS)]
    sx = [torch.empty(T, dtype=torch.float32, device=dev) for _ in range(NSETS)]
    ws_lin = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, T, F, H, N, M), dev)
    ws_grp = sbn.new_workspace(sum(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, T, a, b, N, M) for a, b in shapes), dev)
    # one grouped call per step: the projections share X, so it is quantized once and all their
    # tiles go out in one launch (largest problem first)
    order = sorted(range(len(shapes)), key=lambda j: -shapes[j][0])
    groups = [sbn.LinearGroup([Xs[i]] * len(shapes), [Wp[j][0] for j in order], [Wp[j][1] for j in order],
                              [Ys[i][j] for j in order], N, M, ws_grp, sbn.SBN_PATH_SMFMAC) for i in range(NSETS)]
    torch.cuda.synchronize()
    counter = [0]

    def step():
        i = counter[0] % NSETS
        counter[0] += 1
        groups[i].run()

    ramp(step, 0.3)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_step = e0.elapsed_time(e1) / args.steps
    ops_step = sum(2.0 * T * b * a for a, b in shapes)
    value = ops_step / (ms_step * 1e-3) / 1e12
    log(f"[gemm] step {ms_step:.4f} ms (wall {wall_ms:.4f}) -> {value:.1f} TOPS dense-equivalent")

    # dominant kernel alone: the sparse GEMM on pre-quantized activations, per shape
    for i in range(NSETS):
        sbn.sbn_act_quant(Xs[i], xq[i], sx[i])
    gemm_rows = {}
    for j, (a, b) in enumerate(shapes):
        def gemm_only(j=j):
            i = counter[0] % NSETS
            counter[0] += 1
            sbn.sbn_sparse_ternary_linear(None, Wp[j][0], Wp[j][1], Ys[i][j], N, M, ws_lin, xq_out=xq[i], sx_out=sx[i],
                                          path=sbn.SBN_PATH_SMFMAC)
        ms = timed(gemm_only, 200, 5)
        executed = 1.0 * T * b * a               # executed int8 ops: half of the dense-equivalent 2*T*K*d_out
        bytes_alg = T * b + a * b // 4 + 4 * T * a + 4 * T
        gemm_rows[f"{a}x{b}"] = {"ms": ms, "tops_dense_equiv": 2 * executed / (ms * 1e-3) / 1e12,
                                 "executed_tops": executed / (ms * 1e-3) / 1e12,
                                 "frac_int8_mfma": executed / (ms * 1e-3) / 1e12 / INT8_DENSE_PEAK_TOPS,
                                 "algorithmic_gbps": bytes_alg / (ms * 1e-3) / 1e9,
                                 "frac_hbm": bytes_alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        log(f"[gemm] sparse kernel {a}x{b}: {ms * 1e3:.1f} us, {gemm_rows[f'{a}x{b}']['tops_dense_equiv']:.0f} TOPS, "
            f"{gemm_rows[f'{a}x{b}']['algorithmic_gbps']:.0f} GB/s")
    ms_aq = timed(lambda: sbn.sbn_act_quant(Xs[counter[0] % NSETS], xq[0], sx[0]), 200, 5)
    rows["act_quant_4096x2560"] = {"ms": ms_aq, "gbps": (3 * T * H + 4 * T) / (ms_aq * 1e-3) / 1e9}
    # Algorithm 1's Q_a(Norm(x)) in one pass: RMS normalisation with gain fused in front of the quantizer
    gain_n = (1.0 + 0.25 * torch.randn(H, generator=torch.Generator().manual_seed(3))).to(dev)
    ms_nq = timed(lambda: sbn.sbn_rmsnorm_act_quant(Xs[counter[0] % NSETS], xq[0], sx[0], gain_n, 1e-6), 200, 5)
    rows["rmsnorm_act_quant_4096x2560"] = {"ms": ms_nq, "gbps": (3 * T * H + 4 * T + 4 * H) / (ms_nq * 1e-3) / 1e9}
    log(f"[gemm] act_quant {ms_aq * 1e3:.1f} us ({rows['act_quant_4096x2560']['gbps']:.0f} GB/s); with RMS norm fused "
        f"{ms_nq * 1e3:.1f} us ({rows['rmsnorm_act_quant_4096x2560']['gbps']:.0f} GB/s)")
    rows["gemm_sparse"] = gemm_rows
    big = gemm_rows[f"{F}x{H}"] if f"{F}x{H}" in gemm_rows else next(iter(gemm_rows.values()))
    roofline = {"kernel": "gemm_smfmac_kernel", "workload": f"T={T} K={H} d_out={F}", "bound": "mfma",
                "achieved": big["executed_tops"], "peak": INT8_DENSE_PEAK_TOPS, "unit": "TOP/s",
                "frac": big["frac_int8_mfma"], "traffic": measured_traffic("gemm_smfmac_kernel", f"{F}x{H}"),
                "algorithmic_bytes": T * H + F * H // 4 + 4 * T * F + 4 * T,
                "note": "executed int8 ops T*K*d_out (the 2:4 instruction skips half of 2*T*K*d_out); "
                        "dense-equivalent TOPS / 10 POPS gives the same fraction"}

    # ------------------------------------------------------------------ dense-ternary comparison path
    if "dense" in sections:
        # the dense comparison: the same product on the dense int8 matrix cores, W_eff as int8 with explicit zeros.  Kernel
        # against kernel (weights expanded beforehand), and through SBN_PATH_DENSE_MFMA with its expansion pass per call
        dense_rows = {}
        for j, (a, b) in enumerate(shapes):
            Weff = torch.empty(a, b, dtype=torch.int8, device=dev)
            sbn.sbn_unpack(Wp[j][0], a, b, N, M, W_eff=Weff)

            def dense_kernel(j=j, Weff=Weff):
                i = counter[0] % NSETS
                counter[0] += 1
                sbn.sbn_dense_ternary_linear(xq[i], sx[i], Weff, Wp[j][1], Ys[i][j])

            def dense_call(j=j):
                i = counter[0] % NSETS
                counter[0] += 1
                sbn.sbn_sparse_ternary_linear(None, Wp[j][0], Wp[j][1], Ys[i][j], N, M, ws_lin, xq_out=xq[i],
                                              sx_out=sx[i], path=sbn.SBN_PATH_DENSE_MFMA)
            msk = timed(dense_kernel, 100, 3)
            ms = timed(dense_call, 100, 3)
            dense_rows[f"{a}x{b}"] = {"ms": msk, "ms_with_expand": ms, "tops": 2.0 * T * a * b / (msk * 1e-3) / 1e12,
                                      "frac_int8_mfma": 2.0 * T * a * b / (msk * 1e-3) / 1e12 / INT8_DENSE_PEAK_TOPS,
                                      "sparse_speedup": msk / gemm_rows[f"{a}x{b}"]["ms"]}
            log(f"[dense] {a}x{b}: kernel {msk * 1e3:.1f} us ({ms * 1e3:.1f} us with the expansion pass) -> the 2:4 sparse "
                f"kernel is {msk / gemm_rows[f'{a}x{b}']['ms']:.2f}x faster, kernel against kernel")
            del Weff
        rows["gemm_dense_ternary"] = dense_rows
        # other patterns.  The paper's main pattern 6:8 has no sparse matrix instruction of its own: it runs as dense 2-bit
        # codes through two sparse instructions per group of four - stored that way once (sbn_convert_packed, the
        # inference case) or converted per call (path selection on the 6:8 packed form); 2:8 is an instance of 2:4
        # (rewritten per call into the 2:4 operand form, then the sparse kernel)
        for (n8, m8, key) in ((6, 8, "gemm_6of8_dense_codes"), (2, 8, "gemm_2of8_sparse_mfma")):
            rows_p = {}
            for j, (a, b) in enumerate(shapes):
                pk = pack_one(sbn_synth.latent_weight(a, b, sbn_synth.seed_for(3, a), device=dev), n8, m8)

                def call_p(j=j, pk=pk, n8=n8, m8=m8):
                    i = counter[0] % NSETS
                    counter[0] += 1
                    sbn.sbn_sparse_ternary_linear(None, pk[0], pk[1], Ys[i][j], n8, m8, ws_lin, xq_out=xq[i], sx_out=sx[i],
                                                  path=sbn.SBN_PATH_AUTO)
                ms = timed(call_p, 100, 3)
                rows_p[f"{a}x{b}"] = {"ms_with_operand_rewrite": ms, "tops": 2.0 * T * a * b / (ms * 1e-3) / 1e12,
                                      "vs_2of4_sparse": ms / gemm_rows[f"{a}x{b}"]["ms"]}
                line = f"[{n8}:{m8}] {a}x{b}: {ms * 1e3:.1f} us with the per-call rewrite"
                if n8 == 6:
                    codes = torch.empty(sbn.sbn_packed_bytes(a, b, 8, 8), dtype=torch.uint8, device=dev)
                    sbn.sbn_convert_packed(pk[0], a, b, 6, 8, 8, 8, codes)

                    def call_c(j=j, pk=pk, codes=codes):
                        i = counter[0] % NSETS
                        counter[0] += 1
                        sbn.sbn_sparse_ternary_linear(None, codes, pk[1], Ys[i][j], 8, 8, ws_lin, xq_out=xq[i], sx_out=sx[i],
                                                      path=sbn.SBN_PATH_SMFMAC)
                    msc = timed(call_c, 100, 3)
                    dk = dense_rows[f"{a}x{b}"]["ms"]
                    rows_p[f"{a}x{b}"].update({"ms": msc, "tops": 2.0 * T * a * b / (msc * 1e-3) / 1e12,
                                               "frac_int8_mfma": 2.0 * T * a * b / (msc * 1e-3) / 1e12 / INT8_DENSE_PEAK_TOPS,
                                               "speedup_over_dense_kernel": dk / msc})
                    line += f"; converted once {msc * 1e3:.1f} us = {dk / msc:.2f}x the dense int8 kernel"
                    del codes
                log(line)
                del pk
            rows[key] = rows_p
    # ------------------------------------------------------------------ the paper's throughput table, by token count
    # Section 3.2 reports prefill at 512 ... 65536 tokens and decode at batch 64 ... 512 (other hardware, 6:8, whole
    # model).  The same sweep for one 6912x2560 layer on pre-quantized activations (prefill): the 2:4 sparse kernel and
    # the 6:8 layer (stored as dense 2-bit codes) against the dense int8 comparison kernel, kernel against kernel; and
    # one call through path selection including its quantizer (decode).
    if "seq" in sections:
        jF = [j for j, (a, b) in enumerate(shapes) if a == F][0]
        WeffF = torch.empty(F, H, dtype=torch.int8, device=dev)
        sbn.sbn_unpack(Wp[jF][0], F, H, N, M, W_eff=WeffF)
        pk68 = pack_one(sbn_synth.latent_weight(F, H, sbn_synth.seed_for(3, F), device=dev), 6, 8)
        codes68 = torch.empty(sbn.sbn_packed_bytes(F, H, 8, 8), dtype=torch.uint8, device=dev)
        sbn.sbn_convert_packed(pk68[0], F, H, 6, 8, 8, 8, codes68)
        by_tokens = {}
        for Ts in (512, 1024, 2048, 4096, 8192, 16384, 32768, 65536):
            Xs_ = sbn_synth.activations(Ts, H, sbn_synth.seed_for(3, 50), device=dev)
            xq_ = torch.empty(Ts, H, dtype=torch.int8, device=dev)
            sx_ = torch.empty(Ts, dtype=torch.float32, device=dev)
            Y_ = torch.empty(Ts, F, dtype=torch.float32, device=dev)
            ws_ = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, Ts, F, H, N, M), dev)
            sbn.sbn_act_quant(Xs_, xq_, sx_)
            reps = max(3, min(100, (1 << 19) // Ts))
            ms_s = timed(lambda: sbn.sbn_sparse_ternary_linear(None, Wp[jF][0], Wp[jF][1], Y_, N, M, ws_, xq_out=xq_, sx_out=sx_,
                                                               path=sbn.SBN_PATH_SMFMAC), reps, 2)
            ms_6 = timed(lambda: sbn.sbn_sparse_ternary_linear(None, codes68, pk68[1], Y_, 8, 8, ws_, xq_out=xq_, sx_out=sx_,
                                                               path=sbn.SBN_PATH_SMFMAC), reps, 2)
            ms_d = timed(lambda: sbn.sbn_dense_ternary_linear(xq_, sx_, WeffF, Wp[jF][1], Y_), reps, 2)
            by_tokens[str(Ts)] = {"sparse_ms": ms_s, "six_of_eight_ms": ms_6, "dense_ternary_ms": ms_d,
                                  "sparse_tops_dense_equiv": 2.0 * Ts * F * H / (ms_s * 1e-3) / 1e12,
                                  "tokens_per_s_sparse": Ts / (ms_s * 1e-3), "sparse_speedup": ms_d / ms_s,
                                  "six_of_eight_speedup": ms_d / ms_6}
            del Xs_, xq_, sx_, Y_, ws_
            torch.cuda.empty_cache()
        del WeffF, pk68, codes68
        rows["prefill_6912x2560_by_tokens"] = by_tokens
        log("[seq] prefill 6912x2560, 2:4 sparse TOPS (speedup of 2:4 / of 6:8 over the dense int8 kernel) by tokens: " +
            ", ".join(f"{k}: {v['sparse_tops_dense_equiv']:.0f} ({v['sparse_speedup']:.2f}x / {v['six_of_eight_speedup']:.2f}x)"
                      for k, v in by_tokens.items()))
        by_batch = {}
        for Tb in (16, 64, 128, 256, 512):
            Xb = sbn_synth.activations(Tb, H, sbn_synth.seed_for(2, 60), device=dev)
            Yb = torch.empty(Tb, F, dtype=torch.float32, device=dev)
            wsb_ = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, Tb, F, H, N, M), dev)
            ms_b = timed(lambda: sbn.sbn_sparse_ternary_linear(Xb, Wp[jF][0], Wp[jF][1], Yb, N, M, wsb_), 200, 3)
            by_batch[str(Tb)] = {"single_call_us": ms_b * 1e3, "tops_dense_equiv": 2.0 * Tb * F * H / (ms_b * 1e-3) / 1e12}
            del Xb, Yb, wsb_
        rows["decode_6912x2560_by_batch"] = by_batch
        log("[seq] decode 6912x2560, one call incl. quantizer, us by batch: " +
            ", ".join(f"{k}: {v['single_call_us']:.1f}" for k, v in by_batch.items()))
    del Ys, Xs
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ configs[1]: decode GEMV, streamed over R copies
    roofline_gemv = None
    if "gemv" in sections:
        R = 64
        gemv_rows = {}
        batch_rows = {}
        for name, (a, b) in (("up_6912x2560", (F, H)), ("down_2560x6912", (H, F))):
            packs = [pack_one(sbn_synth.latent_weight(a, b, sbn_synth.seed_for(2, 100 * r + a % 7), device=dev)) for r in range(R)]
            pbytes = sbn.sbn_packed_bytes(a, b, N, M)
            for tok in (1, 8):
                if any(o.startswith(("up_", "down_")) for o in only) and f"{name}_T{tok}" not in only:
                    continue
                X = sbn_synth.activations(tok, b, sbn_synth.seed_for(2, tok), device=dev)
                Yl = [torch.empty(tok, a, dtype=torch.float32, device=dev) for _ in range(R)]
                ws = sbn.new_workspace(R * sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, tok, a, b, N, M), dev)
                grp = sbn.LinearGroup([X] * R, [p for p, _ in packs], [g for _, g in packs], Yl, N, M, ws, sbn.SBN_PATH_GEMV)
                ms = timed(grp.run, 100, 3)
                ws1 = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, tok, a, b, N, M), dev)
                k = [0]

                def single():
                    r = k[0] % R
                    k[0] += 1
                    sbn.sbn_sparse_ternary_linear(X, packs[r][0], packs[r][1], Yl[r], N, M, ws1, path=sbn.SBN_PATH_GEMV)
                ms1 = timed(single, 256, 8)
                gbps = R * pbytes / (ms * 1e-3) / 1e9
                # every byte the decode of one matrix must move: packed weights, bf16 activations in, fp32 outputs
                allb = pbytes + 2 * tok * b + 4 * tok * a
                gemv_rows[f"{name}_T{tok}"] = {"stream_ms_per_matrix": ms / R, "stream_gbps": gbps,
                                               "frac_hbm": gbps / HBM_PEAK_GBPS, "single_call_us": ms1 * 1e3,
                                               "packed_bytes": pbytes, "copies": R,
                                               "frac_hbm_with_activation_and_output_bytes": gbps * allb / pbytes / HBM_PEAK_GBPS}
                log(f"[gemv] {name} T={tok}: stream {gbps:.0f} GB/s ({gbps / HBM_PEAK_GBPS:.1%} of HBM peak), "
                    f"single call {ms1 * 1e3:.1f} us")
                del Yl, ws, grp
            # decode at the batch sizes of the paper's throughput table (Section 3.2): the same R copies in one grouped
            # call on automatic path selection (17 .. 64 tokens: the streaming kernel for decode batches; more: the
            # sparse GEMM kernel with its work dealt by row tile), and one call alone
            if not any(o.startswith(("up_", "down_")) for o in only):
                for tok in (32, 64, 128, 256, 512):
                    X = sbn_synth.activations(tok, b, sbn_synth.seed_for(2, tok), device=dev)
                    Yl = [torch.empty(tok, a, dtype=torch.float32, device=dev) for _ in range(R)]
                    ws = sbn.new_workspace(R * sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, tok, a, b, N, M), dev)
                    grp = sbn.LinearGroup([X] * R, [p for p, _ in packs], [g for _, g in packs], Yl, N, M, ws, sbn.SBN_PATH_AUTO)
                    ms = timed(grp.run, 50, 3)
                    ws1 = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, tok, a, b, N, M), dev)
                    k = [0]

                    def single_b():
                        r = k[0] % R
                        k[0] += 1
                        sbn.sbn_sparse_ternary_linear(X, packs[r][0], packs[r][1], Yl[r], N, M, ws1, path=sbn.SBN_PATH_AUTO)
                    ms1 = timed(single_b, 128, 8)
                    gbps = R * pbytes / (ms * 1e-3) / 1e9
                    # what a layer of the batch must move: packed weights, bf16 activations in, fp32 outputs (the outputs
                    # are 40 % of the weights' bytes at 64 tokens and 3.2 times them at 512)
                    allb = pbytes + 2 * tok * b + 4 * tok * a
                    batch_rows[f"{name}_B{tok}"] = {"stream_us_per_matrix": ms / R * 1e3, "stream_gbps_packed_bytes": gbps,
                                                    "frac_hbm": gbps / HBM_PEAK_GBPS,
                                                    "frac_hbm_with_activation_and_output_bytes": gbps * allb / pbytes / HBM_PEAK_GBPS,
                                                    "tops_dense_equiv": 2.0 * tok * a * b * R / (ms * 1e-3) / 1e12,
                                                    "single_call_us": ms1 * 1e3, "copies": R}
                    log(f"[batch] {name} batch {tok}: stream {ms / R * 1e3:.2f} us per matrix ({gbps / HBM_PEAK_GBPS:.1%} of HBM peak "
                        f"on packed bytes, {gbps * allb / pbytes / HBM_PEAK_GBPS:.1%} with activations and outputs, "
                        f"{2.0 * tok * a * b * R / (ms * 1e-3) / 1e12:.0f} TOPS dense-equivalent), single call {ms1 * 1e3:.1f} us")
                    del Yl, ws, grp, ws1
            del packs
            torch.cuda.empty_cache()
        rows["gemv"] = gemv_rows
        rows["decode_batches"] = batch_rows
        # decode of other patterns at 6912x2560, T = 8, through automatic path selection: 1:4 is read as stored (the
        # kernel builds the sparse operands in registers), the other instances of 2:4 are rewritten into the 2:4
        # operand form per call, everything else into dense 2-bit codes (6:8 is the paper's main pattern); N = M is
        # stored as dense codes; 1:4 and N = M also stream in a grouped call
        other = {}
        X8 = sbn_synth.activations(8, H, sbn_synth.seed_for(2, 8), device=dev)
        Y8 = [torch.empty(8, F, dtype=torch.float32, device=dev) for _ in range(8)]
        for (n8, m8) in ((6, 8), (2, 8), (1, 4), (8, 8)):
            pk = [pack_one(sbn_synth.latent_weight(F, H, sbn_synth.seed_for(2, 300 + r), device=dev), n8, m8) for r in range(8)]
            ws1 = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, 8, F, H, n8, m8), dev)
            k = [0]

            def single_p(pk=pk, n8=n8, m8=m8, ws1=ws1):
                r = k[0] % 8
                k[0] += 1
                sbn.sbn_sparse_ternary_linear(X8, pk[r][0], pk[r][1], Y8[r], n8, m8, ws1, path=sbn.SBN_PATH_AUTO)
            us = timed(single_p, 256, 8) * 1e3
            other[f"{n8}of{m8}"] = {"single_call_us": us, "rewritten_per_call": (n8, m8) in ((6, 8), (2, 8)),
                                    "packed_bytes": sbn.sbn_packed_bytes(F, H, n8, m8)}
            log(f"[gemv] {n8}:{m8} 6912x2560 T=8 single call {us:.1f} us")
            del pk, ws1
        packs = [pack_one(sbn_synth.latent_weight(F, H, sbn_synth.seed_for(2, 400 + r), device=dev), 8, 8) for r in range(R)]
        pbytes = sbn.sbn_packed_bytes(F, H, 8, 8)
        Yl = [torch.empty(8, F, dtype=torch.float32, device=dev) for _ in range(R)]
        ws = sbn.new_workspace(R * sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, 8, F, H, 8, 8), dev)
        grp = sbn.LinearGroup([X8] * R, [p for p, _ in packs], [g for _, g in packs], Yl, 8, 8, ws, sbn.SBN_PATH_GEMV)
        ms = timed(grp.run, 100, 3)
        gbps = R * pbytes / (ms * 1e-3) / 1e9
        other["8of8"].update({"stream_gbps": gbps, "frac_hbm": gbps / HBM_PEAK_GBPS, "copies": R})
        log(f"[gemv] 8:8 (dense 2-bit codes) 6912x2560 T=8: stream {gbps:.0f} GB/s ({gbps / HBM_PEAK_GBPS:.1%} of HBM peak)")
        del packs, grp
        # 1:4 as stored (one bit per weight), counted on its own packed bytes
        packs = [pack_one(sbn_synth.latent_weight(F, H, sbn_synth.seed_for(2, 450 + r), device=dev), 1, 4) for r in range(R)]
        pb14 = sbn.sbn_packed_bytes(F, H, 1, 4)
        grp = sbn.LinearGroup([X8] * R, [p for p, _ in packs], [g for _, g in packs], Yl, 1, 4, ws, sbn.SBN_PATH_GEMV)
        ms = timed(grp.run, 100, 3)
        gbps = R * pb14 / (ms * 1e-3) / 1e9
        other["1of4"].update({"stream_gbps": gbps, "frac_hbm": gbps / HBM_PEAK_GBPS, "copies": R, "stream_ms_per_matrix": ms / R,
                              "stream_time_vs_2of4": ms / R / gemv_rows["up_6912x2560_T8"]["stream_ms_per_matrix"]
                              if "up_6912x2560_T8" in gemv_rows else None})
        log(f"[gemv] 1:4 as stored 6912x2560 T=8: stream {gbps:.0f} GB/s of its packed bytes ({gbps / HBM_PEAK_GBPS:.1%} of HBM peak), "
            f"{ms / R * 1e3:.2f} us per matrix")
        del packs, grp
        # 6:8 converted once into dense codes (sbn_convert_packed), then streamed like any pre-packed weight
        convs = []
        for r in range(R):
            p68, g68 = pack_one(sbn_synth.latent_weight(F, H, sbn_synth.seed_for(2, 500 + r), device=dev), 6, 8)
            c = torch.empty(pbytes, dtype=torch.uint8, device=dev)
            sbn.sbn_convert_packed(p68, F, H, 6, 8, 8, 8, c)
            convs.append((c, g68))
        torch.cuda.synchronize()
        grp = sbn.LinearGroup([X8] * R, [c for c, _ in convs], [g for _, g in convs], Yl, 8, 8, ws, sbn.SBN_PATH_GEMV)
        ms = timed(grp.run, 100, 3)
        gbps = R * pbytes / (ms * 1e-3) / 1e9
        k = [0]

        def single_c():
            r = k[0] % R
            k[0] += 1
            sbn.sbn_sparse_ternary_linear(X8, convs[r][0], convs[r][1], Yl[r], 8, 8, ws, path=sbn.SBN_PATH_GEMV)
        us = timed(single_c, 256, 8) * 1e3
        other["6of8"].update({"converted_once_stream_gbps": gbps, "converted_once_frac_hbm": gbps / HBM_PEAK_GBPS,
                              "converted_once_single_call_us": us, "converted_bytes": pbytes})
        log(f"[gemv] 6:8 converted once to dense codes: stream {gbps:.0f} GB/s ({gbps / HBM_PEAK_GBPS:.1%} of HBM peak), "
            f"single call {us:.1f} us")
        del convs, Yl, ws, grp, Y8
        torch.cuda.empty_cache()
        rows["gemv_other_patterns"] = other
        # the figure that is reported is the slowest of the four workloads, on packed weight bytes alone
        worst_name = min(gemv_rows, key=lambda k: gemv_rows[k]["frac_hbm"])
        worst = gemv_rows[worst_name]
        shape, tok = worst_name.split("_")[1], worst_name.split("_T")[1]
        roofline_gemv = {"kernel": "gemv_stream_kernel",
                         "workload": f"64 x ({shape} packed 2:4), T={tok}, grouped (slowest of {sorted(gemv_rows)})",
                         "bound": "hbm", "achieved": worst["stream_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": worst["frac_hbm"], "traffic": measured_traffic("gemv_stream_kernel", "64x" + shape),
                         "algorithmic_bytes": R * worst["packed_bytes"],
                         # the same kernel per matrix shape and token count, on packed weight bytes only, and with the
                         # bf16 activations read and the fp32 outputs written counted too (5 % more bytes at eight tokens)
                         "frac_by_workload": {k: v["frac_hbm"] for k, v in gemv_rows.items()},
                         "frac_by_workload_with_activation_and_output_bytes":
                             {k: v["frac_hbm_with_activation_and_output_bytes"] for k, v in gemv_rows.items()}}

    # ------------------------------------------------------------------ configs[3]: quantize_mask_pack sweep, 210 matrices
    if "pack" in sections:
        Wl = []
        for layer in range(sbn_synth.LAYERS):
            for mi, (_, a, b) in enumerate(sbn_synth.BLOCK_MATRICES):
                Wl.append(sbn_synth.latent_weight(a, b, sbn_synth.seed_for(4, 10 * layer + mi), device=dev))
        nweights = sum(w.numel() for w in Wl)
        gam = torch.empty(len(Wl), dtype=torch.float32, device=dev)
        glist = [gam[i:i + 1] for i in range(len(Wl))]
        wsp = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_QUANTIZE_MASK_PACK, len(Wl), F, H, N, M), dev)
        pack_rows = {}
        for n, m in ((2, 4), (1, 4), (2, 8)):
            pl = [torch.empty(sbn.sbn_packed_bytes(w.shape[0], w.shape[1], n, m), dtype=torch.uint8, device=dev) for w in Wl]
            batch = sbn.PackBatch(Wl, n, m, pl, glist, wsp)
            ms = timed(batch.run, 5, 1)
            bytes_alg = 2 * nweights + sum(p.numel() for p in pl) + 4 * len(Wl)
            pack_rows[f"{n}:{m}"] = {"sweep_ms": ms, "algorithmic_gb": bytes_alg / 1e9,
                                     "gbps": bytes_alg / (ms * 1e-3) / 1e9,
                                     "frac_hbm": bytes_alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
            log(f"[pack] {n}:{m} sweep of {len(Wl)} matrices: {ms:.3f} ms, {pack_rows[f'{n}:{m}']['gbps']:.0f} GB/s "
                f"on single-read bytes")
            # the same sweep in place over the previous packed forms, counting every matrix's mask flips on the way
            # (it also reads the old index fields: N * log2(M) / (8 M) bytes per weight more)
            fl = torch.zeros(len(Wl), dtype=torch.int64, device=dev)
            batch_f = sbn.PackBatch(Wl, n, m, pl, glist, wsp, fl)
            ms_f = timed(batch_f.run, 5, 1)
            idx_bytes = sum(p.numel() for p in pl) * {4: 2, 8: 3}[m] // ({4: 2, 8: 3}[m] + 2)
            pack_rows[f"{n}:{m}"].update({"with_flip_counts_ms": ms_f, "with_flip_counts_gbps": (bytes_alg + idx_bytes) / (ms_f * 1e-3) / 1e9,
                                          "flip_count_extra_ms": ms_f - ms})
            log(f"[pack] {n}:{m} sweep in place with flip counts: {ms_f:.3f} ms (+{(ms_f / ms - 1) * 100:.1f} %)")
            del pl, batch, batch_f
        rows["quantize_mask_pack"] = pack_rows
        # mask flips between two packed forms of the largest matrix (ablation study, mask flip rate equation)
        pa = pack_one(Wl[4])
        pb = pack_one((Wl[4].float() + 0.25 * Wl[5].float()).to(torch.bfloat16))
        flips = torch.zeros(1, dtype=torch.int64, device=dev)
        wsf = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_MASK_FLIPS, 1, F, H, N, M), dev)
        ms = timed(lambda: sbn.sbn_mask_flips(pa[0], pb[0], F, H, N, M, flips, wsf), 100, 3)
        rows["mask_flips_6912x2560"] = {"us": ms * 1e3, "flip_rate": flips.item() / (F * H),
                                        "gbps_index_bytes": 2 * (F * H // 8) / (ms * 1e-3) / 1e9}
        log(f"[flips] 6912x2560 2:4, separate pass over two packed forms: {ms * 1e3:.1f} us, flip rate {flips.item() / (F * H):.4f}")
        del Wl
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ configs[4]: one block's training step
    if "train" in sections:
        Tt = 8 * 2048
        mats = sbn_synth.BLOCK_MATRICES
        Wt = [sbn_synth.latent_weight(a, b, sbn_synth.seed_for(5, i), device=dev) for i, (_, a, b) in enumerate(mats)]
        # the block's four distinct layer inputs: attention input (Q, K, V), attention output (O), FFN input (up, gate),
        # FFN hidden (down); each is quantized once per step and the layers that share it reuse the int8 copy
        inputs = [sbn_synth.activations(Tt, H, sbn_synth.seed_for(5, 20), device=dev),
                  sbn_synth.activations(Tt, H, sbn_synth.seed_for(5, 21), device=dev),
                  sbn_synth.activations(Tt, H, sbn_synth.seed_for(5, 23), device=dev),
                  sbn_synth.activations(Tt, F, sbn_synth.seed_for(5, 22), device=dev)]
        input_of = [0, 0, 0, 1, 2, 2, 3]                     # per matrix of BLOCK_MATRICES
        dYh = sbn_synth.grad_output(Tt, H, sbn_synth.seed_for(5, 30), device=dev)
        dYf = sbn_synth.grad_output(Tt, F, sbn_synth.seed_for(5, 31), device=dev)
        pk = [torch.empty(sbn.sbn_packed_bytes(a, b, N, M), dtype=torch.uint8, device=dev) for _, a, b in mats]
        gm = torch.empty(len(mats), dtype=torch.float32, device=dev)
        gl = [gm[i:i + 1] for i in range(len(mats))]
        wsp = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_QUANTIZE_MASK_PACK, len(mats), F, H, N, M), dev)
        batch = sbn.PackBatch(Wt, N, M, pk, gl, wsp)
        Yl = [torch.empty(Tt, a, dtype=torch.float32, device=dev) for _, a, b in mats]
        xql = [torch.empty(Tt, x.shape[1], dtype=torch.int8, device=dev) for x in inputs]
        sxl = [torch.empty(Tt, dtype=torch.float32, device=dev) for _ in inputs]
        dXl = [torch.empty(Tt, b, dtype=torch.bfloat16, device=dev) for _, a, b in mats]
        dWl = [torch.empty(a, b, dtype=torch.bfloat16, device=dev) for _, a, b in mats]
        wsl = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, Tt, F, F, N, M), dev)
        wsb = sbn.new_workspace(sbn.sbn_workspace_bytes(sbn.SBN_OP_BACKWARD, Tt, F, F, N, M), dev)

        def remask():
            batch.run()

        def forward():
            for j, x in enumerate(inputs):
                sbn.sbn_act_quant(x, xql[j], sxl[j])
            for i in range(len(mats)):
                j = input_of[i]
                sbn.sbn_sparse_ternary_linear(None, pk[i], gl[i], Yl[i], N, M, wsl, xq_out=xql[j], sx_out=sxl[j],
                                              path=sbn.SBN_PATH_SMFMAC)

        def backward_layer_by_layer():
            for i, (_, a, b) in enumerate(mats):
                j = input_of[i]
                sbn.sbn_sparse_ternary_linear_backward(dYf if a == F else dYh, pk[i], gl[i], xql[j], sxl[j], N, M, wsb, b,
                                                       dX=dXl[i], dW=dWl[i])

        # backward in the order of backpropagation, the layers whose output gradients arrive together in one call:
        # down; up and gate; O; Q, K and V (layers of a call that share their input share its transpose)
        groups = []
        for idx in ([6], [4, 5], [3], [0, 1, 2]):
            wsg = sbn.new_workspace(sum(sbn.sbn_workspace_bytes(sbn.SBN_OP_BACKWARD, Tt, mats[i][1], mats[i][2], N, M)
                                        for i in idx), dev)
            groups.append(sbn.BackwardGroup([dYf if mats[i][1] == F else dYh for i in idx], [pk[i] for i in idx],
                                            [gl[i] for i in idx], [xql[input_of[i]] for i in idx],
                                            [sxl[input_of[i]] for i in idx], N, M, wsg, [mats[i][2] for i in idx],
                                            [dXl[i] for i in idx], [dWl[i] for i in idx]))

        def backward_grouped():
            for grp in groups:
                grp.run()

        def train_step():
            remask()
            forward()
            backward_grouped()

        ms_all = timed(train_step, 3, 1)
        ms_pack = timed(remask, 5, 1)
        ms_fwd = timed(forward, 3, 1)
        ms_bwd = timed(backward_grouped, 3, 1)
        ms_bwd_single = timed(backward_layer_by_layer, 3, 1)
        wsum = sum(a * b for _, a, b in mats)
        rows["train_step_block"] = {
            "tokens": Tt, "ms": ms_all, "remask_pack_ms": ms_pack, "forward_ms": ms_fwd, "backward_ms": ms_bwd,
            "backward_layer_by_layer_ms": ms_bwd_single,
            "forward_tops_dense_equiv": 2.0 * Tt * wsum / (ms_fwd * 1e-3) / 1e12,
            "backward_tflops": 4.0 * Tt * wsum / (ms_bwd * 1e-3) / 1e12,
            "backward_frac_bf16_mfma": 4.0 * Tt * wsum / (ms_bwd * 1e-3) / 1e12 / BF16_DENSE_PEAK_TFLOPS,
            "step_tops_total": 6.0 * Tt * wsum / (ms_all * 1e-3) / 1e12}
        log(f"[train] block step {ms_all:.2f} ms (pack {ms_pack:.3f}, fwd {ms_fwd:.2f}, bwd {ms_bwd:.2f} in four grouped calls, "
            f"{ms_bwd_single:.2f} layer by layer); "
            f"bwd {rows['train_step_block']['backward_tflops']:.0f} TFLOP/s")
        del Wt, inputs, dYh, dYf, Yl, xql, sxl, dXl, dWl, wsl, wsb, groups
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ plain copy of known size (scale of the HBM counters)
    if "copyref" in sections:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        b = torch.empty_like(a)
        ms = timed(lambda: b.copy_(a), 5, 1)
        rows["copyref_1GiB"] = {"ms": ms, "gbps": 2 * (1 << 30) / (ms * 1e-3) / 1e9}
        del a, b

    # ------------------------------------------------------------------ ceilings this board sustains, next to the datasheet peaks
    ceilings = None
    if "ceil" in sections:
        from paper_2603_05168_amd import probe as sbn_probe   # libsbn_probe.so: measurement support, not the layer's library
        buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)   # 1 GiB: four times the Infinity Cache
        ceilings = {}
        for key, kind, iters, unit in (("smfmac_i8_dense_equiv", sbn_probe.SBN_CEIL_SMFMAC_I8, 100, 1e12),
                                       ("mfma_i8", sbn_probe.SBN_CEIL_MFMA_I8, 100, 1e12),
                                       ("mfma_bf16", sbn_probe.SBN_CEIL_MFMA_BF16, 100, 1e12),
                                       ("hbm_read", sbn_probe.SBN_CEIL_HBM_READ, 1, 1e9),
                                       ("hbm_write", sbn_probe.SBN_CEIL_HBM_WRITE, 1, 1e9),
                                       ("lds_read", sbn_probe.SBN_CEIL_LDS_READ, 2000, 1e9)):
            work = [0.0]

            def probe(kind=kind, iters=iters):
                work[0] = sbn_probe.sbn_ceiling_probe(kind, buf, iters)
            ms = timed(probe, 200 if unit == 1e12 else 20, 2)
            ceilings[key] = work[0] / (ms * 1e-3) / unit
        ceilings["units"] = "TOP/s or TFLOP/s with random operands (matrix kinds), GB/s over 1 GiB (stream kinds), GB/s of conflict-free 16-byte LDS reads summed over all multiprocessors"
        log("[ceil] sustained on this board: sparse int8 MFMA %.0f TOPS dense-equivalent, int8 MFMA %.0f TOPS, bf16 MFMA %.0f "
            "TFLOP/s, HBM read %.0f GB/s, write %.0f GB/s, LDS read %.0f GB/s" % (
                ceilings["smfmac_i8_dense_equiv"], ceilings["mfma_i8"], ceilings["mfma_bf16"], ceilings["hbm_read"],
                ceilings["hbm_write"], ceilings["lds_read"]))
        del buf
        torch.cuda.empty_cache()
        roofline["measured_ceiling"] = ceilings["smfmac_i8_dense_equiv"] / 2.0   # executed ops, like `achieved`
        roofline["frac_of_measured_ceiling"] = roofline["achieved"] / roofline["measured_ceiling"]
        if roofline_gemv is not None:
            roofline_gemv["measured_ceiling"] = ceilings["hbm_read"]
            roofline_gemv["frac_of_measured_ceiling"] = roofline_gemv["achieved"] / ceilings["hbm_read"]

    # ------------------------------------------------------------------ CPU oracle on a bounded sample of the same workload
    cpu_baseline = None
    if "cpu" in sections:
        import numpy as np
        import oracle
        # the oracle runs the whole timed step once: both matrices, all 4096 tokens (a few seconds on the box)
        Xc = sbn_synth.activations(T, H, sbn_synth.seed_for(3, 10)).float().numpy()
        weights = []
        t1 = time.perf_counter()
        for a, b in shapes:
            Wc = sbn_synth.latent_weight(a, b, sbn_synth.seed_for(3, a)).float().numpy()
            weights.append(oracle.quantize_mask(Wc, N, M))
        pack_s = time.perf_counter() - t1
        t1 = time.perf_counter()
        for Weff, mask, g in weights:
            oracle.sparse_ternary_linear(Xc, Weff, g)
        dt = time.perf_counter() - t1
        cpu_baseline = {"value": ops_step / dt / 1e12, "unit": "TOPS", "cores": oracle.threads(), "kind": "oracle",
                        "sample": f"the whole timed step once: forward of all {T} tokens against both matrices "
                                  f"(activation quantizer, dense brute-force accumulate, rescale) in {dt:.1f} s; "
                                  f"the untimed weight side (mask, quantize) of both matrices took {pack_s:.2f} s"}
        log(f"[cpu] oracle: {cpu_baseline['value']:.4f} TOPS on {cpu_baseline['cores']} threads ({cpu_baseline['sample']})")

    out = {
        "metric": "N:M ternary GEMM TOPS + decode GEMV GB/s (% of MI355X roofline)",
        "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "configs[2] prefill: X 4096x2560 bf16 -> act-quant + 2:4 sparse-MFMA GEMM + rescale "
                               "against packed ternary 2560x2560 and 6912x2560, fp32 Y; ops counted dense-equivalent "
                               "2*T*K*d_out", "tokens": T, "pattern": "2:4", "rotating_buffer_sets": NSETS},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "gemv_gbps": None if roofline_gemv is None else roofline_gemv["achieved"],
        "roofline_gemv": roofline_gemv,
        "ceilings": ceilings,
        "rows": rows,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
