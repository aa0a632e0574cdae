/*
 * CPU oracle for the N:M-sparse ternary linear layer of Sparse-BitNet (arxiv 2603.05168).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the layer computes.
 * It is called by the tests, by the smoke check and by the benchmark's cpu_baseline leg; the
 * product library never links, loads or calls it, and it shares no code, header or table with
 * the GPU sources.  Every function follows one passage of the paper, cited above it; where the
 * paper is silent the reading taken is stated.  Plain loops, fp64 wherever a float result is
 * later compared with a tolerance, exact fp32 where the paper's arithmetic decides an integer.
 *
 * Pins (tests that fix each function to something other than itself) live in tests/test_oracle_*.py:
 * closed forms for Gaussian weights, brute-force sorting, scale/sign invariances, the N = M
 * reduction to the plain BitLinear layer, the layer written as an fp64 graph whose gradients an
 * autograd engine derives, and pack/unpack round trips.  The packed byte layout is this build's own
 * (the paper asks only that the N:M metadata have a defined layout), so sbn_oracle_pack and
 * sbn_oracle_unpack are pinned by hand-assembled bytes for one row at 2:4, 1:4, 2:8, 6:8 and 8:8
 * (every index width: 2 bits, 3 bits, none), by a second decoder written separately, by each other
 * and by structural invariants; no value printed in the paper covers it: for the byte layout
 * itself, parity unpinned by the paper.
 *
 * Build:  gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC -o libsbn_oracle.so sbn_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ---------------------------------------------------------------------------------------------
 * Section 2.1, ternary quantizer: gamma = ||W||_1 / (d_out * d_in).
 * Appendix B listing: the scale is the mean of |w| over the WHOLE, unmasked matrix, clamped from
 * below at 1e-5 (no additive epsilon).  Reading: one gamma per matrix; the sum runs in double over
 * the fp32 inputs (each term exact), in row-major order, and is rounded to fp32 once.
 * ------------------------------------------------------------------------------------------- */
float sbn_oracle_absmean(const float *W, int64_t d_out, int64_t d_in)
{
    double sum = 0.0;
    for (int64_t i = 0; i < d_out * d_in; ++i)
        sum += fabs((double)W[i]);
    float gamma = (float)(sum / (double)(d_out * d_in));
    return gamma < 1e-5f ? 1e-5f : gamma;
}

/* ---------------------------------------------------------------------------------------------
 * Section 2.2, magnitude-based mask generation (the Top-N indicator per group of M):
 * for every contiguous group of M weights along the input dimension keep the N largest |w| of the
 * LATENT weights.  Exactly N ones per group.
 * Reading (the paper gives no tie rule): among equal magnitudes the lower index wins, so element j
 * is kept iff  #{j' : |w_j'| > |w_j|} + #{j' < j : |w_j'| == |w_j|}  <  N.   -0.0 ties with +0.0.
 * ------------------------------------------------------------------------------------------- */
void sbn_oracle_nm_mask(const float *W, int64_t d_out, int64_t d_in, int N, int M, uint8_t *mask)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < d_out; ++i) {
        for (int64_t g = 0; g < d_in / M; ++g) {
            const float *w = W + i * d_in + g * M;
            uint8_t *m = mask + i * d_in + g * M;
            for (int j = 0; j < M; ++j) {
                float aj = fabsf(w[j]);
                int rank = 0;
                for (int jj = 0; jj < M; ++jj) {
                    float a = fabsf(w[jj]);
                    if (a > aj || (a == aj && jj < j))
                        ++rank;
                }
                m[j] = (uint8_t)(rank < N);
            }
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Section 2.1, W_q = RoundClip(W / gamma, -1, +1); Appendix B listing: divide by the scale, round, clamp to [-1, 1].
 * Reading: an IEEE fp32 division, round-half-to-even (the listing's tensor round), then the clip.
 * ------------------------------------------------------------------------------------------- */
void sbn_oracle_ternary(const float *W, int64_t n, float gamma, int8_t *Wq)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        volatile float r = W[i] / gamma; /* volatile: keep the fp32 rounding of the quotient */
        float q = rintf(r);
        if (q > 1.0f) q = 1.0f;
        if (q < -1.0f) q = -1.0f;
        Wq[i] = (int8_t)q;
    }
}

/* Section 2.2, W_eff = W_q (.) M_{N:M}  (quantize first, then apply the mask). */
void sbn_oracle_apply_mask(const int8_t *Wq, const uint8_t *mask, int64_t n, int8_t *Weff)
{
    for (int64_t i = 0; i < n; ++i)
        Weff[i] = mask[i] ? Wq[i] : (int8_t)0;
}

/* ---------------------------------------------------------------------------------------------
 * Section 2.1, activation quantizer; Appendix B listing, forward(): per token (last dimension)
 *   s_x = 127 / max(amax|x|, 1e-5),   x~ = clamp(round(x * s_x), -128, 127).
 * Reading: all of it in fp32 on exactly up-converted inputs: one fp32 division for s_x, one fp32
 * multiply, round-half-to-even.
 * ------------------------------------------------------------------------------------------- */
void sbn_oracle_act_quant(const float *X, int64_t T, int64_t K, int8_t *xq, float *sx)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(X[t * K + k]);
            if (a > amax) amax = a;
        }
        if (amax < 1e-5f) amax = 1e-5f;
        volatile float s = 127.0f / amax;
        sx[t] = s;
        for (int64_t k = 0; k < K; ++k) {
            volatile float p = X[t * K + k] * s;
            float q = rintf(p);
            if (q > 127.0f) q = 127.0f;
            if (q < -128.0f) q = -128.0f;
            xq[t * K + k] = (int8_t)q;
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Algorithm 1, the line that forms the layer input: x~ <- Q_a(Norm(x)).  The paper does not say
 * which normalisation; reading: the RMS normalisation BitNet-style models place in front of every
 * quantised linear layer, per token over the last dimension, with a learnable gain and no bias:
 *   n[k] = x[k] / sqrt(mean_k(x^2) + eps) * g[k].
 * Arithmetic fixed here so that the int8 codes that follow are well defined: the mean of squares in
 * double over exactly up-converted inputs, in order; r = 1/sqrt(mean + eps) in double, rounded to
 * fp32 once; x * r and then * g as two fp32 multiplies; the result rounded to bf16 (the model's
 * activation type, round-to-nearest-even), returned as float.  gain == NULL means g = 1 (no multiply).
 * ------------------------------------------------------------------------------------------- */
static float round_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;   /* finite inputs only */
    memcpy(&f, &u, 4);
    return f;
}

void sbn_oracle_rmsnorm(const float *X, const float *gain, float eps, int64_t T, int64_t K, float *Xn)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double ssq = 0.0;
        for (int64_t k = 0; k < K; ++k) ssq += (double)X[t * K + k] * (double)X[t * K + k];
        const float r = (float)(1.0 / sqrt(ssq / (double)K + (double)eps));
        for (int64_t k = 0; k < K; ++k) {
            volatile float y = X[t * K + k] * r;
            if (gain) y = y * gain[k];
            Xn[t * K + k] = round_to_bf16(y);
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Section 2.2, forward pass, the integer part of  y ~ s * (W_eff x~):
 *   acc[t, o] = sum_k W_eff[o, k] * x~[t, k]   in int32 (dense brute force over every k).
 * ------------------------------------------------------------------------------------------- */
void sbn_oracle_acc(const int8_t *Weff, const int8_t *xq, int64_t T, int64_t K, int64_t d_out,
                    int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t o = 0; o < d_out; ++o) {
            int32_t a = 0;
            for (int64_t k = 0; k < K; ++k)
                a += (int32_t)Weff[o * K + k] * (int32_t)xq[t * K + k];
            acc[t * d_out + o] = a;
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Section 2.2, forward-pass equation, the scalar s carries both quantization scales: the weight scale gamma multiplies back and the
 * activation scale s_x divides back (the listing rescales w_q by scale and x_q by 1/s_x), plus the
 * layer's optional bias.  Computed in double:  y = acc * gamma / s_x[t] (+ bias[o]).
 * ------------------------------------------------------------------------------------------- */
void sbn_oracle_rescale(const int32_t *acc, float gamma, const float *sx, const float *bias,
                        int64_t T, int64_t d_out, double *y)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t o = 0; o < d_out; ++o) {
            double v = (double)acc[t * d_out + o] * (double)gamma / (double)sx[t];
            if (bias) v += (double)bias[o];
            y[t * d_out + o] = v;
        }
}

/* ---------------------------------------------------------------------------------------------
 * Section 2.3 (dual straight-through estimator) + the listing's linear projection: the layer's
 * output is linear(x_q, w_q) with w_q = gamma * W_eff and x_q = x~ / s_x, so
 *   dX[t, k] = gamma * sum_o dY[t, o] * W_eff[o, k]        (identity STE through the activation
 *                                                            quantizer, standard BitNet training)
 *   dW[o, k] = sum_t dY[t, o] * (x~[t, k] / s_x[t])         (handed to the latent weight unchanged:
 *                                                            no mask, no clipping window)
 * Both in double from exactly converted inputs.
 * ------------------------------------------------------------------------------------------- */
void sbn_oracle_backward_dx(const float *dY, const int8_t *Weff, float gamma, int64_t T, int64_t K,
                            int64_t d_out, double *dX)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double *dx = dX + t * K;
        for (int64_t k = 0; k < K; ++k) dx[k] = 0.0;
        for (int64_t o = 0; o < d_out; ++o) {
            double dy = (double)dY[t * d_out + o];
            const int8_t *w = Weff + o * K;
            for (int64_t k = 0; k < K; ++k)
                dx[k] += dy * (double)w[k];
        }
        for (int64_t k = 0; k < K; ++k) dx[k] *= (double)gamma;
    }
}

void sbn_oracle_backward_dw(const float *dY, const int8_t *xq, const float *sx, int64_t T, int64_t K,
                            int64_t d_out, double *dW)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < d_out; ++o) {
        double *dw = dW + o * K;
        for (int64_t k = 0; k < K; ++k) dw[k] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double dy = (double)dY[t * d_out + o];
            double inv = 1.0 / (double)sx[t];
            const int8_t *x = xq + t * K;
            for (int64_t k = 0; k < K; ++k)
                dw[k] += dy * ((double)x[k] * inv);
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Packed layout (this build's own; Section 2.2 asks only that the N:M metadata have a defined layout).
 *
 * M in {2, 4, 8}, 1 <= N <= M, d_in % M == 0.  Let b = log2(M) (b = 0 when N == M: no indices).
 * A row of W is cut into chunks of 128 consecutive weights, the last one zero-padded (a padded
 * group is an all-zero group: the tie rule keeps its first N positions, all codes 0).
 * Inside a chunk the kept weights form S = 128*N/M slots, group after group, ascending position
 * within a group.  A slot is (index: position within the group, b bits; code: 2-bit two's
 * complement of the ternary value, 0 -> 00, +1 -> 01, -1 -> 11; 10 never occurs).
 * A chunk is stored as
 *   index field, S*b/8 bytes: slot s at bits [s*b, s*b + b) of the field read as a little-endian
 *                             bit string (bit p is bit p%8 of byte p/8);
 *   code field,  S/4 bytes:   S/16 little-endian 32-bit words; slot s lies in word s/16 and, with
 *                             v = s%16, at bits [8*(v%4) + 2*(v/4), +2) of that word.
 * Rows follow one another: packed[row * nchunks * chunk_bytes + chunk * chunk_bytes + ...].
 * ------------------------------------------------------------------------------------------- */
static int log2_of(int M) { return M == 2 ? 1 : M == 4 ? 2 : M == 8 ? 3 : -1; }

int64_t sbn_oracle_chunk_bytes(int N, int M)
{
    int b = log2_of(M);
    if (b < 0 || N < 1 || N > M) return -1;
    if (N == M) b = 0;
    int64_t S = 128 * N / M;
    return S * b / 8 + S / 4;
}

int64_t sbn_oracle_packed_bytes(int64_t d_out, int64_t d_in, int N, int M)
{
    int64_t cb = sbn_oracle_chunk_bytes(N, M);
    if (cb < 0 || d_in % M != 0) return -1;
    return d_out * ((d_in + 127) / 128) * cb;
}

static void put_bits(uint8_t *field, int64_t pos, int nbits, unsigned value)
{
    for (int i = 0; i < nbits; ++i)
        if ((value >> i) & 1u)
            field[(pos + i) / 8] |= (uint8_t)(1u << ((pos + i) % 8));
}

static unsigned get_bits(const uint8_t *field, int64_t pos, int nbits)
{
    unsigned v = 0;
    for (int i = 0; i < nbits; ++i)
        v |= (unsigned)((field[(pos + i) / 8] >> ((pos + i) % 8)) & 1u) << i;
    return v;
}

static int64_t code_bit_position(int64_t s)
{
    int64_t word = s / 16, v = s % 16;
    return word * 32 + 8 * (v % 4) + 2 * (v / 4);
}

/* mask and Weff are dense [d_out, d_in]; returns 0, or -1 on an unsupported pattern or a mask row
 * whose group does not hold exactly N ones. */
int sbn_oracle_pack(const int8_t *Weff, const uint8_t *mask, int64_t d_out, int64_t d_in, int N,
                    int M, uint8_t *packed)
{
    int64_t cb = sbn_oracle_chunk_bytes(N, M);
    if (cb < 0 || d_in % M != 0) return -1;
    int b = (N == M) ? 0 : log2_of(M);
    int64_t S = 128 * N / M, nchunks = (d_in + 127) / 128, idx_bytes = S * b / 8;
    memset(packed, 0, (size_t)(d_out * nchunks * cb));
    for (int64_t i = 0; i < d_out; ++i)
        for (int64_t c = 0; c < nchunks; ++c) {
            uint8_t *idx_field = packed + (i * nchunks + c) * cb;
            uint8_t *code_field = idx_field + idx_bytes;
            int64_t s = 0;
            for (int64_t g = 0; g < 128 / M; ++g) {
                int64_t col0 = c * 128 + g * M;
                int kept = 0;
                for (int j = 0; j < M; ++j) {
                    int in_range = col0 + j < d_in;
                    int keep = in_range ? mask[i * d_in + col0 + j] : (j < N);
                    if (!keep) continue;
                    int q = in_range ? Weff[i * d_in + col0 + j] : 0;
                    put_bits(idx_field, s * b, b, (unsigned)j);
                    put_bits(code_field, code_bit_position(s), 2, (unsigned)q & 3u);
                    ++s;
                    ++kept;
                }
                if (kept != N) return -1;
            }
        }
    return 0;
}

/* Inverse of the layout above, written on its own: fills dense W_eff and the 0/1 mask. */
int sbn_oracle_unpack(const uint8_t *packed, int64_t d_out, int64_t d_in, int N, int M,
                      int8_t *Weff, uint8_t *mask)
{
    int64_t cb = sbn_oracle_chunk_bytes(N, M);
    if (cb < 0 || d_in % M != 0) return -1;
    int b = (N == M) ? 0 : log2_of(M);
    int64_t S = 128 * N / M, nchunks = (d_in + 127) / 128, idx_bytes = S * b / 8;
    memset(Weff, 0, (size_t)(d_out * d_in));
    memset(mask, 0, (size_t)(d_out * d_in));
    for (int64_t i = 0; i < d_out; ++i)
        for (int64_t c = 0; c < nchunks; ++c) {
            const uint8_t *idx_field = packed + (i * nchunks + c) * cb;
            const uint8_t *code_field = idx_field + idx_bytes;
            for (int64_t s = 0; s < S; ++s) {
                int64_t g = s / N;
                int j = (N == M) ? (int)(s % N) : (int)get_bits(idx_field, s * b, b);
                unsigned code = get_bits(code_field, code_bit_position(s), 2);
                int64_t col = c * 128 + g * M + j;
                if (col >= d_in) continue;
                if (code == 2u) return -2; /* the reserved code */
                mask[i * d_in + col] = 1;
                Weff[i * d_in + col] = (int8_t)(code == 1u ? 1 : code == 3u ? -1 : 0);
            }
        }
    return 0;
}

/* Ablation study, mask flip rate equation: r_t = || m(w_t) - m(w_{t-1}) ||_1 / D. */
double sbn_oracle_flip_rate(const uint8_t *mask_a, const uint8_t *mask_b, int64_t n)
{
    int64_t diff = 0;
    for (int64_t i = 0; i < n; ++i)
        diff += (mask_a[i] != mask_b[i]);
    return (double)diff / (double)n;
}
