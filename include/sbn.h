/*
 * sbn.h - C ABI of libsbn: the N:M-sparse ternary linear layer of Sparse-BitNet
 * (arxiv 2603.05168) for AMD MI355X (gfx950).
 *
 * Conventions for every entry point
 *   - Pointers marked "device" are HIP device pointers owned by the caller; "host" are host
 *     pointers.  The library never allocates, frees or synchronises: a call validates its
 *     arguments on the host, then only enqueues kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and returns.
 *   - Matrices are row-major.  W is [d_out, d_in] with d_in contiguous; groups of M consecutive
 *     weights of a row form the N:M groups (Section 2.1, N:M definition; Section 2.2, mask).
 *   - Supported patterns: M in {2, 4, 8}, 1 <= N <= M, d_in % M == 0.
 *   - Return value: SBN_OK or a negative sbn_status.  All argument errors are detected before
 *     anything is launched.  After SBN_EHIP, sbn_last_error() returns the HIP error text.
 *   - Inputs must be finite; the result for NaN/Inf inputs is unspecified.
 *   - Stream capture: every call may be recorded into a HIP graph and replayed (no memory copies or
 *     memsets are enqueued, descriptor tables travel as kernel arguments, counters are cleared by
 *     kernels).  Call each entry point once outside capture first: the first use of a kernel sets
 *     function attributes and queries the device.  While a stream captures, grouped decode calls
 *     launch the activation quantizer in front of the streaming kernel instead of fusing it (the
 *     fused form numbers its launches on the host).  Pointers and sizes are frozen in the graph.
 *   - No environment variable changes what a call does.
 *
 * Packed weight layout (the paper asks only that the N:M metadata have a defined layout; this one
 * is the library's).  b = log2(M) index bits per kept weight (none when N == M).  Each row is cut
 * into chunks of 128 consecutive weights, the last chunk zero-padded (a padded group keeps its
 * first N positions with value 0).  Inside a chunk the kept weights form S = 128*N/M slots, group
 * after group, ascending position within a group; a slot = (position in its group, 2-bit two's
 * complement ternary code: 0 -> 00, +1 -> 01, -1 -> 11; 10 never occurs).  A chunk is stored as
 *     index field,  S*b/8 bytes: slot s at bits [s*b, s*b+b) of a little-endian bit string;
 *     code field,   S/4 bytes = S/16 little-endian 32-bit words: slot s in word s/16, and with
 *                   v = s%16 at bits [8*(v%4) + 2*(v/4), +2) of that word.
 * Chunks of a row, then rows, follow one another without gaps.  For 2:4 a chunk is 32 bytes
 * (2 bits per weight): four index words (one nibble per group: pos0 | pos1 << 2) and four code
 * words; each (index word, code word) pair describes 32 consecutive weights and feeds one lane of
 * a CDNA4 sparse MFMA directly.
 */
#ifndef SBN_H
#define SBN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SBN_OK = 0,
    SBN_EINVAL = -1,       /* null pointer, non-positive size, N/M out of range, d_in % M != 0 */
    SBN_EUNSUPPORTED = -2, /* valid request this build has no kernel for (e.g. sparse MFMA path, pattern not 2:4) */
    SBN_ESIZE = -3,        /* workspace too small */
    SBN_EALIGN = -4,       /* pointer or leading dimension not aligned as documented */
    SBN_EHIP = -5          /* a HIP call failed; see sbn_last_error() */
} sbn_status;

typedef enum { SBN_F32 = 0, SBN_BF16 = 1 } sbn_dtype;

typedef enum {
    SBN_PATH_AUTO = 0,       /* d_in % 128 == 0: GEMV for tokens <= 16, sparse MFMA GEMM for more.  Any other case: dense
                                MFMA if d_in % 64 == 0, generic else */
    SBN_PATH_GEMV = 1,       /* decode kernel: streams the packed weights once; tokens <= 16, d_in % 128 == 0.  2:4 runs
                                on the sparse instruction and N = M (dense 2-bit codes) on the dense one as stored; 1:4
                                is read as stored too (one bit per weight: the kernel builds the sparse instruction's
                                operands in registers); other patterns are rewritten per call into one of the two forms
                                (a pass over the packed weights: sbn_convert_packed does it once instead) */
    SBN_PATH_SMFMAC = 2,     /* prefill/training GEMM on sparse int8 MFMA (v_smfmac); d_in % 128 == 0.  2:4 runs as
                                stored, its instances (1:2, 1:4, 1:8, 2:8) after a rewrite into the 2:4 operand form.
                                Every other pattern (6:8, N:8, ...) runs as dense 2-bit codes - N = M as stored, the
                                rest converted per call (sbn_convert_packed to N = M does it once instead) - with two
                                sparse instructions per group of four weights (positions 0, 1 and positions 2, 3): the
                                matrix-core time of a dense int8 product at a quarter of its weight bytes.
                                Decode batches (Section 3.2 measures decoding at batch 64 .. 512) take this path too:
                                up to 64 tokens with neither bias nor acc_out a kernel that streams the weights once
                                into registers (same instructions on 16 x 16 tiles), up to 512 tokens the GEMM kernel
                                with its work dealt by row tile */
    SBN_PATH_DENSE_MFMA = 3, /* W_eff expanded to int8 with explicit zeros, dense int8 MFMA: the comparison path;
                                d_in % 64 == 0 */
    SBN_PATH_GENERIC = 4     /* any supported pattern, plain integer kernel (reference speed only) */
} sbn_path;

typedef enum {
    SBN_OP_QUANTIZE_MASK_PACK = 0,
    SBN_OP_LINEAR = 1,
    SBN_OP_BACKWARD = 2,
    SBN_OP_MASK_FLIPS = 3
} sbn_op;

/* Bytes of the packed form of a [d_out, d_in] matrix at N:M.  Host only, no GPU needed. */
sbn_status sbn_packed_bytes(int64_t d_out, int64_t d_in, int N, int M, size_t *bytes);

/* Workspace (device scratch, 256-byte aligned, contents undefined on entry and exit) the given
 * operation needs at these sizes.  For SBN_OP_QUANTIZE_MASK_PACK `tokens` is the number of matrices
 * packed in one batched call (1 for the single call).  Host only. */
sbn_status sbn_workspace_bytes(sbn_op op, int64_t tokens, int64_t d_out, int64_t d_in, int N, int M,
                               size_t *bytes);

/*
 * Weight side of the layer, every training step (Section 2.2 mask generation and quant-and-mask;
 * Section 2.3 per-step mask recomputation; Appendix B listing, weight function):
 *   gamma = max(mean |W| over the whole matrix, 1e-5)     (sum in fp64, rounded to fp32 once)
 *   mask  = top-N of every M consecutive |w| of the LATENT weights, ties to the lower index
 *   W_eff = clip(round_half_even(w / gamma), -1, +1) at the kept positions, 0 elsewhere
 * and packs W_eff with its positions into `packed` (layout above).
 *   W_latent  device, [d_out, ld_w] elements of type wdt, ld_w >= d_in; read only
 *   packed    device, sbn_packed_bytes() bytes, 16-byte aligned; written
 *   gamma     device, one float; written
 *   workspace device, >= sbn_workspace_bytes(SBN_OP_QUANTIZE_MASK_PACK, 1, ...) bytes
 */
sbn_status sbn_quantize_mask_pack(const void *W_latent, sbn_dtype wdt, int64_t d_out, int64_t d_in,
                                  int64_t ld_w, int N, int M, void *packed, float *gamma,
                                  void *workspace, size_t ws_bytes, void *stream);

/*
 * The same for `count` matrices in one enqueue (the per-step remask of all linear weights of a
 * model: Section 2.3).  The arrays are HOST arrays of length count; W_latent[i], packed[i],
 * gamma[i] are device pointers as above.  All matrices share wdt, N and M; ld_w[i] == d_in[i].
 * workspace >= sbn_workspace_bytes(SBN_OP_QUANTIZE_MASK_PACK, count, max d_out, max d_in, N, M).
 */
sbn_status sbn_quantize_mask_pack_batched(int count, const void *const *W_latent, sbn_dtype wdt,
                                          const int64_t *d_out, const int64_t *d_in, int N, int M,
                                          void *const *packed, float *const *gamma,
                                          void *workspace, size_t ws_bytes, void *stream);

/*
 * Algorithm 1, x~ <- Q_a(Norm(x)): RMS normalisation (the paper names no particular Norm; this is the
 * one BitNet-style models put in front of every quantised linear layer) fused with the activation
 * quantizer of Section 2.1, X read once:
 *   r = fp32(1 / sqrt(mean_k x[t,k]^2 + eps))   mean in double
 *   n[t,k] = bf16( fp32(x[t,k] * r) * gain[k] )  two fp32 multiplies, one rounding to bf16 (gain NULL: 1)
 *   s_x[t], x~[t,:] = the activation quantizer of sbn_act_quant applied to n[t,:]
 * The result feeds sbn_sparse_ternary_linear in its pre-quantized mode (X = NULL, xq_out / sx_out given).
 *   X bf16 [tokens, d_in] device, 16-byte aligned; gain fp32 [d_in] device, 16-byte aligned, or NULL
 *   xq int8 [tokens, d_in], sx fp32 [tokens]: device, overwritten; xn_out bf16 [tokens, d_in] or NULL
 * Errors: SBN_EINVAL, SBN_EALIGN, SBN_EUNSUPPORTED (d_in % 8 != 0 or d_in > 16384), SBN_EHIP.  One kernel.
 */
sbn_status sbn_rmsnorm_act_quant(const void *X, int64_t tokens, int64_t d_in, const float *gain, float eps, int8_t *xq,
                                 float *sx, void *xn_out, void *stream);

/*
 * Activation quantizer alone (Section 2.1, absmax int8 activations; Appendix B listing, forward()):
 *   s_x[t] = 127 / max(max_k |X[t,k]|, 1e-5),  xq[t,k] = clip(round_half_even(X[t,k] * s_x[t]), -128, 127)
 *   X  device, bf16 [tokens, d_in], 16-byte aligned, d_in % 8 == 0;  xq device int8 [tokens, d_in], 16-byte
 *   aligned; sx device fp32 [tokens].  The forward call below runs this itself; it is exported for callers
 *   that quantize once and feed several layers (Q/K/V, up/gate).
 */
sbn_status sbn_act_quant(const void *X, int64_t tokens, int64_t d_in, int8_t *xq, float *sx, void *stream);

/*
 * Forward of the layer (Section 2.1 activation quantizer; Section 2.2 forward-pass equation;
 * Appendix B listing, forward()):
 *   s_x[t]   = 127 / max(max_k |X[t,k]|, 1e-5)                       (fp32)
 *   xq[t,k]  = clip(round_half_even(X[t,k] * s_x[t]), -128, 127)     (int8)
 *   acc[t,o] = sum_k W_eff[o,k] * xq[t,k]                            (int32, exact)
 *   Y[t,o]   = acc[t,o] * gamma / s_x[t] (+ bias[o])                 (fp32)
 *   X        device, bf16 [tokens, d_in], 16-byte aligned, d_in % 8 == 0 (d_in % 128 == 0 for the MFMA paths);
 *            or NULL: then xq_out and sx_out are INPUTS holding activations already quantized by
 *            sbn_act_quant, and the quantizer is skipped
 *   packed   device, from sbn_quantize_mask_pack with the same d_out, d_in, N, M
 *   gamma    device, one float (stays on the device between the two calls: no host sync)
 *   bias     device, fp32 [d_out], or NULL
 *   Y        device, fp32 [tokens, d_out]; written
 *   xq_out   device, int8 [tokens, d_in], or NULL; written (kept for the backward call)
 *   sx_out   device, fp32 [tokens], or NULL; written
 *   acc_out  device, int32 [tokens, d_out], or NULL; written (the exact accumulators, for checks)
 *   workspace >= sbn_workspace_bytes(SBN_OP_LINEAR, tokens, d_out, d_in, N, M)
 */
sbn_status sbn_sparse_ternary_linear(const void *X, int64_t tokens, int64_t d_in, int64_t d_out,
                                     int N, int M, const void *packed, const float *gamma,
                                     const float *bias, float *Y, int8_t *xq_out, float *sx_out,
                                     int32_t *acc_out, sbn_path path, void *workspace,
                                     size_t ws_bytes, void *stream);

/*
 * The forward call for callers that cannot allocate or carry a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): sbn_sparse_ternary_linear without the workspace arguments.
 * Its scratch (the int8 activations and per-token scales of the call) lives in a buffer of
 * SBN_STATIC_SCRATCH_MIB MiB inside the library's device image; every GPU the library runs on holds its own copy
 * until the process ends.  The call allocates and frees nothing and enqueues the same kernels as the call above,
 * so Y, xq_out, sx_out and acc_out are the same bit for bit.
 *   arguments   as sbn_sparse_ternary_linear
 *   limits      align256(tokens * d_in) + align256(4 * tokens) <= SBN_STATIC_SCRATCH_MIB MiB, else SBN_ESIZE
 *               (sbn_last_error() then says how much was needed); only paths that read the weights as stored:
 *               2:4 and N = M on SBN_PATH_GEMV / SBN_PATH_SMFMAC, 1:4 on SBN_PATH_GEMV, any pattern on SBN_PATH_GENERIC
 *               (SBN_PATH_AUTO when it resolves to one of these); every other case SBN_EUNSUPPORTED
 *   sharing     all calls on a GPU use that GPU's one buffer, which keeps the last call's contents (nothing in it has
 *               to start at zero: flags left behind carry the number of the launch that raised them).  Calls that
 *               overlap on one GPU (two streams, two threads) race on it: serialise them, or use the call above.
 */
enum { SBN_STATIC_SCRATCH_MIB = 16 };
sbn_status sbn_sparse_ternary_linear_static(const void *X, int64_t tokens, int64_t d_in, int64_t d_out,
                                            int N, int M, const void *packed, const float *gamma,
                                            const float *bias, float *Y, int8_t *xq_out, float *sx_out,
                                            int32_t *acc_out, sbn_path path, void *stream);

/*
 * `count` independent forward problems in one enqueue (decode: every projection that is ready at
 * the same time; also used to stream many matrices through the GEMV kernel).  HOST arrays of
 * device pointers / sizes; all problems share N, M and path; bias is not applied.
 * workspace >= sum over problems of sbn_workspace_bytes(SBN_OP_LINEAR, ...).
 */
sbn_status sbn_sparse_ternary_linear_grouped(int count, const void *const *X, const int64_t *tokens,
                                             const int64_t *d_in, const int64_t *d_out, int N, int M,
                                             const void *const *packed, const float *const *gamma,
                                             float *const *Y, sbn_path path, void *workspace,
                                             size_t ws_bytes, void *stream);

/*
 * Backward products of the layer under the dual straight-through estimator (Section 2.3;
 * Appendix B listing, backward()): the output is linear(xq / s_x, gamma * W_eff), so
 *   dX[t,k] = gamma * sum_o dY[t,o] * W_eff[o,k]            (bf16 out, fp32 accumulation)
 *   dW[o,k] = sum_t dY[t,o] * xq[t,k] / s_x[t]              (bf16 out, fp32 accumulation)
 * dW is the gradient of the LATENT weight: dense, not multiplied by the mask, no clipping window.
 *   dY       device, bf16 [tokens, d_out], 16-byte aligned
 *   xq, sx   device, as written by the forward call (needed only when dW != NULL)
 *   dX, dW   device, bf16 [tokens, d_in] / [d_out, d_in], or NULL to skip that product
 *   flags    SBN_BWD_ACCUMULATE: dW += (read-modify-write in bf16), else dW is overwritten;
 *            SBN_BWD_MASK_DW: the ablation study's "gradient masking" variant, dW = M (.) dense dW (only the
 *            weights of the current mask receive the term; needs `packed`); the paper's method leaves it off
 *   workspace >= sbn_workspace_bytes(SBN_OP_BACKWARD, tokens, d_out, d_in, N, M)
 */
enum { SBN_BWD_ACCUMULATE = 1, SBN_BWD_MASK_DW = 2 };
sbn_status sbn_sparse_ternary_linear_backward(const void *dY, int64_t tokens, int64_t d_in,
                                              int64_t d_out, int N, int M, const void *packed,
                                              const float *gamma, const int8_t *xq, const float *sx,
                                              void *dX, void *dW, int flags, void *workspace,
                                              size_t ws_bytes, void *stream);

/*
 * The backward products of `count` (<= SBN_BACKWARD_GROUP_MAX) layers whose output gradients are ready at the
 * same time (Section 2.3: Q/K/V, or up and gate, of one block), in one enqueue: every dW and dX tile of the
 * call goes into one matrix-multiply launch, longest contraction first, and layers that share their quantized
 * input (same xq pointer, tokens and d_in) share its transposed copy.  Per layer the results are those of
 * sbn_sparse_ternary_linear_backward, bit for bit.  HOST arrays of device pointers / sizes, one entry per
 * layer, meanings as above (dX[i] or dW[i] may be NULL; packed, gamma, xq, sx entries may be NULL where the
 * single call allows it); all layers share N, M and flags.
 * workspace >= sum over layers of sbn_workspace_bytes(SBN_OP_BACKWARD, ...).
 */
enum { SBN_BACKWARD_GROUP_MAX = 8 };
sbn_status sbn_sparse_ternary_linear_backward_grouped(int count, const void *const *dY, const int64_t *tokens,
                                                      const int64_t *d_in, const int64_t *d_out, int N, int M,
                                                      const void *const *packed, const float *const *gamma,
                                                      const int8_t *const *xq, const float *const *sx,
                                                      void *const *dX, void *const *dW, int flags,
                                                      void *workspace, size_t ws_bytes, void *stream);

/*
 * The per-step remask with the mask flip count as a by-product (Section 2.3: the mask is recomputed every step;
 * ablation study, mask flip rate equation): sbn_quantize_mask_pack_batched IN PLACE over the previous step's packed
 * forms.  On entry packed[i] holds the packed form an earlier call wrote for a matrix of the same shape at the same
 * N:M; on return it holds the new one (bytes and gamma exactly as sbn_quantize_mask_pack_batched writes them) and
 *   flips_out[i] = || m(W_t) - m(W_{t-1}) ||_1  of matrix i   (as sbn_mask_flips counts it; the caller divides).
 * The kernel that packs a block of weights compares its new index words with the old ones it is about to replace: no
 * second pass over the packed forms.
 *   flips_out  device, `count` uint64, overwritten (integer sums in a fixed order)
 *   supported  bf16 weights, rows contiguous (ld_w = d_in), d_in % 128 == 0, 16-byte aligned, N:M = 2:4, 1:4 or 2:8;
 *              anything else SBN_EUNSUPPORTED (pack, then sbn_mask_flips on two buffers).  If packed[i] does not
 *              hold a valid packed form on entry the new form is still written correctly and flips_out[i] is
 *              meaningless.
 * Everything else as sbn_quantize_mask_pack_batched.
 */
sbn_status sbn_quantize_mask_pack_flips_batched(int count, const void *const *W_latent, sbn_dtype wdt,
                                                const int64_t *d_out, const int64_t *d_in, int N, int M,
                                                void *const *packed, float *const *gamma, uint64_t *flips_out,
                                                void *workspace, size_t ws_bytes, void *stream);

/* Test hook, not timed: expands `packed` to dense W_eff (int8 [d_out, d_in]) and the 0/1 mask
 * (uint8 [d_out, d_in]); either output may be NULL. */
sbn_status sbn_unpack(const void *packed, int64_t d_out, int64_t d_in, int N, int M,
                      int8_t *W_eff, uint8_t *mask, void *stream);

/*
 * Mask dynamics (ablation study, mask flip rate equation): the number of positions at which the N:M
 * masks of two packed forms of the same [d_out, d_in] matrix at the same N:M differ,
 *   flips = || m(W_t) - m(W_{t-1}) ||_1,   flip rate r_t = flips / (d_out * d_in)  (the caller divides).
 * Only the index fields of the packed forms are read (N == M: always 0).
 *   packed_a, packed_b  device, as written by sbn_quantize_mask_pack, 16-byte aligned
 *   flips_out           device, one uint64, overwritten
 *   workspace >= sbn_workspace_bytes(SBN_OP_MASK_FLIPS, 0, d_out, d_in, N, M); enqueues two kernels, deterministic
 */
sbn_status sbn_mask_flips(const void *packed_a, const void *packed_b, int64_t d_out, int64_t d_in, int N,
                          int M, uint64_t *flips_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * Rewrites a packed N:M matrix into the packed form of another pattern that can hold the same
 * W_eff, so that decode calls stream the weights as stored instead of rewriting them per call
 * ("weights pre-packed once"; Section 3.2 measures decode on the 6:8 model):
 *   to_N:to_M = 2:4  for patterns that keep at most two weights of every aligned four (1:2, 1:4, 1:8, 2:8):
 *                    the operand form of the sparse matrix instruction, with zero-code padding slots;
 *   to_N == to_M     for any pattern: dense 2-bit codes with explicit zeros at the dropped positions
 *                    (2 bits per weight; 6:8's own packed form is 3.75).
 * The result is used with N = to_N, M = to_M in sbn_sparse_ternary_linear[_grouped] and gives the same
 * accumulators and Y as the original; it no longer tells kept zeros from dropped weights, so it serves
 * the forward only (sbn_mask_flips and the backward want the original).
 *   packed  device, as written by sbn_quantize_mask_pack at N:M, 16-byte aligned; d_in % 128 == 0
 *   out     device, sbn_packed_bytes(d_out, d_in, to_N, to_M) bytes, 16-byte aligned, overwritten
 * Errors: SBN_EINVAL (null, bad sizes), SBN_EUNSUPPORTED (target cannot hold the pattern, target equal
 * to the source, ragged d_in), SBN_EALIGN, SBN_EHIP.  Enqueues one kernel.
 */
sbn_status sbn_convert_packed(const void *packed, int64_t d_out, int64_t d_in, int N, int M, int to_N, int to_M,
                              void *out, void *stream);

/*
 * The dense comparison kernel on its own (Section 3.2 compares the sparse layer with a dense one of the same
 * precision): the same product on the dense int8 matrix cores with W_eff given as int8 with explicit zeros, so that
 * a benchmark can time it without the expansion pass that SBN_PATH_DENSE_MFMA runs in front of it.
 *   xq, sx      device, int8 [tokens, d_in] row-major and fp32 [tokens] as written by sbn_act_quant, 16-byte aligned
 *   W_eff       device, int8 [d_out, d_in] row-major, values in {-1, 0, +1} as written by sbn_unpack, 16-byte aligned
 *   gamma       device, one fp32;  bias: device fp32 [d_out] or NULL
 *   Y           device, fp32 [tokens, d_out], overwritten: Y = acc * gamma / s_x[t] (+ bias), the same arithmetic as
 *               sbn_sparse_ternary_linear; acc_out: device int32 [tokens, d_out] or NULL
 * d_in % 64 == 0, else SBN_EUNSUPPORTED.  Errors as above.  Enqueues one kernel; nothing is owned or freed.
 */
sbn_status sbn_dense_ternary_linear(const int8_t *xq, const float *sx, int64_t tokens, int64_t d_in, int64_t d_out,
                                    const int8_t *W_eff, const float *gamma, const float *bias, float *Y,
                                    int32_t *acc_out, void *stream);

/*
 * Test hook: bounds of the library's two bounded inter-block waits, in polls.  The streaming decode kernel lets
 * its first blocks quantize the activations while the others wait for their flags, and the single-read pack
 * kernel lets one block finalize a matrix's scale while the others wait for its ready word; a block out of polls
 * does the awaited work itself, so results never depend on these numbers (the tests set them to 0 and below to
 * force that branch).  A negative value means "never wait"; INT_MIN restores the default (about a millisecond of
 * polling, far above any wait of a launch whose blocks are co-resident).  Process-wide; not for use while calls
 * are being enqueued from other threads.
 */
void sbn_test_set_spin_limits(int gemv_polls, int pack_polls);

/* Text of the last HIP error seen by this thread ("" if none). */
const char *sbn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SBN_H */
