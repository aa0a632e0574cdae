// Forward of the N:M-sparse ternary linear layer: activation quantizer, decode GEMV, generic path.
// Section 2.1 (per-token absmax int8 activations), Section 2.2 (forward-pass equation),
// Appendix B listing (forward()).
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <type_traits>
#include <vector>

#include "sbn_internal.hpp"
#include "sbn_mfma.hpp"

namespace sbn {

namespace {

// ---- pieces of the activation quantizer shared by its kernels -------------------------------------
// largest 15-bit magnitude pattern among eight bf16 values and a running maximum (bf16 magnitudes order like integers);
// the two halves of a word are compared as a pair of 16-bit integers
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t absmax_bits_bf16x8(const uint4 &d, uint32_t m)
{
    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
    ushort2_t best = {0, 0};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t mag = w[k] & 0x7fff7fffu;
        best = __builtin_elementwise_max(best, __builtin_bit_cast(ushort2_t, mag));
    }
    const uint32_t both = __builtin_bit_cast(uint32_t, best), lo = both & 0xffffu, hi = both >> 16;
    m = lo > m ? lo : m;
    m = hi > m ? hi : m;
    return m;
}

// s_x from the largest magnitude pattern: 127 / max(amax, 1e-5), one IEEE division
__device__ __forceinline__ float scale_from_absmax_bits(uint32_t m)
{
    float amax = __uint_as_float(m << 16);
    amax = amax < 1e-5f ? 1e-5f : amax;
    return __fdiv_rn(127.0f, amax);
}

// eight bf16 values of a row -> eight int8: clip(rint(x * s)) with one fp32 multiply and half-to-even rounding, s the
// scale of that same row.  The rounding is an addition of 1.5 * 2^23: the sum has an ulp of 1, so the (round-to-nearest-
// even) addition rounds the product exactly as rint does, and the low byte of the sum's bit pattern is the integer in
// two's complement.  No clip is needed: |x| <= amax <= max(amax, 1e-5) and s = fl(127 / max(amax, 1e-5)), so
// |fl(x * s)| <= 127 (1 + 2^-24)^2 < 127.5 and the rounded value already lies in [-127, 127].
__device__ __forceinline__ uint2 quantize_bf16x8(const uint4 &d, float s)
{
    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
    uint32_t z[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        z[2 * k] = __float_as_uint(__fadd_rn(__fmul_rn(__uint_as_float(w[k] << 16), s), 12582912.0f));
        z[2 * k + 1] = __float_as_uint(__fadd_rn(__fmul_rn(__uint_as_float(w[k] & 0xffff0000u), s), 12582912.0f));
    }
    uint32_t packed[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t lo = __builtin_amdgcn_perm(z[4 * h + 1], z[4 * h], 0x0c0c0400u);      // bytes 0, 1
        const uint32_t hi = __builtin_amdgcn_perm(z[4 * h + 3], z[4 * h + 2], 0x04000c0cu);  // bytes 2, 3
        packed[h] = lo | hi;
    }
    return make_uint2(packed[0], packed[1]);
}

// ---- activation quantizer -----------------------------------------------------------------------
// TPT threads share one token (256 = a block of four wavefronts per token for prefill, 1024 = a larger
// block per token for decode, where only a handful of tokens exist).  A thread keeps its 16-byte vectors of the row
// in registers, so X is read once; the maximum magnitude is taken on the bf16 bit patterns (exact).
// s_x = 127 / max(amax, 1e-5) is one IEEE fp32 division, x * s_x one fp32 multiply, rounding is
// half-to-even.  Rows longer than VMAX * TPT vectors take the two-pass kernel below.
template <int TPT, int VMAX>
__global__ void __launch_bounds__(TPT < 256 ? 256 : TPT) act_quant_kernel(const uint4 *__restrict__ X, int64_t tokens, int nvec,
                                                                         int8_t *__restrict__ xq, float *__restrict__ sx)
{
    constexpr int BLOCK = TPT < 256 ? 256 : TPT;
    constexpr int TOK_PER_BLOCK = BLOCK / TPT;
    __shared__ uint32_t wave_max[BLOCK / 64];
    const int sub = threadIdx.x % TPT;
    const int64_t t = (int64_t)blockIdx.x * TOK_PER_BLOCK + threadIdx.x / TPT;
    const bool live = t < tokens;
    const uint4 *row = X + (live ? t : 0) * nvec;
    uint4 v[VMAX];
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < VMAX; ++i) {
        const int idx = sub + i * TPT;
        v[i] = (live && idx < nvec) ? row[idx] : make_uint4(0, 0, 0, 0);
        m = absmax_bits_bf16x8(v[i], m);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
        m = o > m ? o : m;
    }
    if constexpr (TPT > 64) {
        if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < TPT / 64; ++w) {
            const uint32_t o = wave_max[w];
            m = o > m ? o : m;
        }
    }
    const float s = scale_from_absmax_bits(m);
    if (!live) return;
    if (sub == 0) sx[t] = s;
    uint2 *out = reinterpret_cast<uint2 *>(xq + t * (int64_t)nvec * 8);
#pragma unroll
    for (int i = 0; i < VMAX; ++i) {
        const int idx = sub + i * TPT;
        if (idx >= nvec) break;
        out[idx] = quantize_bf16x8(v[i], s);
    }
}

// any row length: one wavefront per token, the row is read twice (the second read is cache resident)
__global__ void __launch_bounds__(256) act_quant_two_pass_kernel(const uint4 *__restrict__ X, int64_t tokens, int nvec,
                                                                int8_t *__restrict__ xq, float *__restrict__ sx)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= tokens) return;
    const uint4 *row = X + t * nvec;
    uint32_t m = 0;
    for (int v = lane; v < nvec; v += 64) {
        m = absmax_bits_bf16x8(row[v], m);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
        m = o > m ? o : m;
    }
    const float s = scale_from_absmax_bits(m);
    if (lane == 0) sx[t] = s;
    uint2 *out = reinterpret_cast<uint2 *>(xq + t * (int64_t)nvec * 8);
    for (int v = lane; v < nvec; v += 64) out[v] = quantize_bf16x8(row[v], s);
}

// ---- RMS normalisation fused in front of the quantizer (Algorithm 1: x~ <- Q_a(Norm(x))) ---------
// Same ownership of a token row as act_quant_kernel, the row held in registers throughout, X read
// once.  The mean of squares is summed in double (every square of a bf16 value is exact), r =
// 1/sqrt(mean + eps) is rounded to fp32 once, n = bf16(fp32(x * r) * g) replaces the row in the
// registers, and the quantizer runs on it as it would on a stored bf16 tensor.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;   // round to nearest even; finite inputs
}

template <int TPT, int VMAX>
__global__ void __launch_bounds__(TPT < 256 ? 256 : TPT) rmsnorm_act_quant_kernel(const uint4 *__restrict__ X, const float *__restrict__ gain,
                                                                                 float eps, int64_t tokens, int nvec, int8_t *__restrict__ xq,
                                                                                 float *__restrict__ sx, uint4 *__restrict__ xn)
{
    constexpr int BLOCK = TPT < 256 ? 256 : TPT;
    constexpr int TOK_PER_BLOCK = BLOCK / TPT;
    __shared__ double wave_ssq[BLOCK / 64];
    __shared__ uint32_t wave_max[BLOCK / 64];
    const int sub = threadIdx.x % TPT;
    const int64_t t = (int64_t)blockIdx.x * TOK_PER_BLOCK + threadIdx.x / TPT;
    const bool live = t < tokens;
    const uint4 *row = X + (live ? t : 0) * nvec;
    uint4 v[VMAX];
    double ssq = 0.0;
#pragma unroll
    for (int i = 0; i < VMAX; ++i) {
        const int idx = sub + i * TPT;
        v[i] = (live && idx < nvec) ? row[idx] : make_uint4(0, 0, 0, 0);
        const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const double lo = (double)__uint_as_float(w[k] << 16), hi = (double)__uint_as_float(w[k] & 0xffff0000u);
            ssq += lo * lo;
            ssq += hi * hi;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ssq += __shfl_xor(ssq, off, 64);
    if constexpr (TPT > 64) {
        if ((threadIdx.x & 63) == 0) wave_ssq[threadIdx.x >> 6] = ssq;
        __syncthreads();
        ssq = 0.0;
#pragma unroll
        for (int w = 0; w < TPT / 64; ++w) ssq += wave_ssq[w];
    }
    const float r = (float)(1.0 / sqrt(ssq / (double)(nvec * 8) + (double)eps));
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < VMAX; ++i) {
        const int idx = sub + i * TPT;
        if (idx >= nvec) break;
        float g[8];
        if (gain) {
            const float4 g0 = *reinterpret_cast<const float4 *>(gain + (int64_t)idx * 8);
            const float4 g1 = *reinterpret_cast<const float4 *>(gain + (int64_t)idx * 8 + 4);
            g[0] = g0.x; g[1] = g0.y; g[2] = g0.z; g[3] = g0.w; g[4] = g1.x; g[5] = g1.y; g[6] = g1.z; g[7] = g1.w;
        }
        uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float lo = __fmul_rn(__uint_as_float(w[k] << 16), r), hi = __fmul_rn(__uint_as_float(w[k] & 0xffff0000u), r);
            if (gain) {
                lo = __fmul_rn(lo, g[2 * k]);
                hi = __fmul_rn(hi, g[2 * k + 1]);
            }
            w[k] = f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
        }
        v[i] = make_uint4(w[0], w[1], w[2], w[3]);
        m = absmax_bits_bf16x8(v[i], m);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
        m = o > m ? o : m;
    }
    if constexpr (TPT > 64) {
        if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < TPT / 64; ++w) {
            const uint32_t o = wave_max[w];
            m = o > m ? o : m;
        }
    }
    const float s = scale_from_absmax_bits(m);
    if (!live) return;
    if (sub == 0) sx[t] = s;
    uint2 *out = reinterpret_cast<uint2 *>(xq + t * (int64_t)nvec * 8);
#pragma unroll
    for (int i = 0; i < VMAX; ++i) {
        const int idx = sub + i * TPT;
        if (idx >= nvec) break;
        out[idx] = quantize_bf16x8(v[i], s);
        if (xn) xn[t * nvec + idx] = v[i];
    }
}

// ---- decode GEMV on the sparse MFMA (tokens <= 16, 2:4) -----------------------------------------
// A block owns 16 rows of W.  Its wavefronts split the input dimension in super-steps of 512
// weights: for such a super-step a lane (row r = lane % 16, quarter c = lane / 16) loads the whole
// 32-byte chunk c of its row (one 16-byte index load, one 16-byte code load; a wavefront reads
// 128 contiguous bytes per row), then issues four v_smfmac_i32_16x16x128_i8, the j-th using index
// word j and code word j.  The tokens are the B operand (16 columns; columns >= tokens are zero).
// Partial accumulators of the wavefronts are summed through LDS, rescaled and stored.
struct GemvItem {
    const int8_t *xq;
    const float *sx;
    const uint8_t *packed;
    const float *gamma;
    const float *bias;
    float *Y;
    int32_t *acc_out;
    const uint4 *X;   // bf16 activations when the block quantizes them itself (then xq and sx are unused), else null
    int d_in, d_out, tokens, pad;
};
constexpr int GEMV_MAX_ITEMS = 40;
constexpr int GEMV_ROW_VEC = 14;   // 16-byte vectors of a token row per lane when a wavefront of the single-call kernel quantizes it
struct GemvTable {
    GemvItem it[GEMV_MAX_ITEMS];   // problem = blockIdx.y; row tile = blockIdx.x (surplus blocks exit at once)
};
static_assert(sizeof(GemvTable) <= 4096, "the table travels as a kernel argument");

// DENSE = true is the same kernel for weights stored as dense 2-bit codes (the packed form of
// N = M, and what other patterns are rewritten to for decode): a chunk is eight code words, every
// word is the A operand of one v_mfma_i32_16x16x64_i8 (lane quarter c holds k = 16c .. 16c+15 of
// the instruction on both operands), so a super-step is eight dense instructions instead of four sparse.
// FORM = GEMV_1OF4 reads the 1:4 packed form as stored (16-byte chunks, one load per lane and super-step) and builds
// the sparse instruction's operands in registers (expand_1of4): half the weight bytes for three times the vector work.
template <int FORM>
__global__ void __launch_bounds__(1024) gemv_smfmac_kernel(GemvTable tab)
{
    constexpr bool DENSE = FORM == GEMV_DENSE, ONE4 = FORM == GEMV_1OF4;
    constexpr int CB = ONE4 ? 16 : 32;   // bytes of a chunk
    extern __shared__ __attribute__((aligned(16))) int8_t xs[];   // self-quantized activations [tokens][d_in + 16]
    __shared__ v4i red[16][64];
    __shared__ uint32_t amax_s[16][16];   // [token][wavefront]
    __shared__ float sx_s[16];
    const GemvItem &it = tab.it[blockIdx.y];
    const int row0 = (int)blockIdx.x * 16;
    if (row0 >= it.d_out) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int r = lane & 15, c4 = lane >> 4;
    const uint32_t ones = vgpr_ones();
    const int K = it.d_in, nchunks = K / CHUNK, nsuper = (nchunks + 3) / 4;
    int row = row0 + r;
    row = row < it.d_out ? row : it.d_out - 1;   // rows past the end are computed and dropped
    const uint8_t *wrow = it.packed + (int64_t)row * nchunks * CB;
    const bool tok_ok = r < it.tokens;           // as B operand the lane holds token r
    const bool self_quant = it.X != nullptr;
    const int pitch = K + 16;
    const int8_t *xrow = self_quant ? xs + (tok_ok ? r : 0) * pitch : it.xq + (int64_t)(tok_ok ? r : 0) * K;

    // the wavefront's first weight words go out before anything else: they fly while the block quantizes
    uint4 idx4 = make_uint4(0, 0, 0, 0), code4 = make_uint4(0, 0, 0, 0);
    auto fetch = [&](int s) {
        const int chunk = 4 * s + c4;
        idx4 = make_uint4(0, 0, 0, 0);
        code4 = make_uint4(0, 0, 0, 0);
        if (s < nsuper && chunk < nchunks) {
            idx4 = *reinterpret_cast<const uint4 *>(wrow + (int64_t)chunk * CB);
            if constexpr (!ONE4) code4 = *reinterpret_cast<const uint4 *>(wrow + (int64_t)chunk * CB + 16);
        }
    };
    fetch(wave);
    if (self_quant) {
        // every block quantizes the few token rows itself (the quantizer's arithmetic), saving the quantizer's
        // launch in front of a latency-bound call
        const int nvec = K / 8, nthreads = (int)blockDim.x;
        if (nvec <= 64 * GEMV_ROW_VEC) {
            // a wavefront per token row, the row in registers (two short rows at a time): the rows of a block cost one
            // or two trips to memory in all, the maximum needs no barrier, the int8 row goes straight into LDS
            auto finish = [&](int t, uint32_t m, auto &xv, auto nv) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
                    m = o > m ? o : m;
                }
                const float sc = scale_from_absmax_bits(m);
                if (lane == 0) sx_s[t] = sc;
#pragma unroll
                for (int i = 0; i < nv(); ++i) {
                    const int idx = lane + 64 * i;
                    if (idx < nvec) *reinterpret_cast<uint2 *>(xs + t * pitch + idx * 8) = quantize_bf16x8(xv[i], sc);
                }
            };
            auto request = [&](int t, auto &xv, auto nv) {
                uint32_t m = 0;
#pragma unroll
                for (int i = 0; i < nv(); ++i) {
                    const int idx = lane + 64 * i;
                    xv[i] = it.X[(int64_t)t * nvec + (idx < nvec ? idx : nvec - 1)];   // past the end the last vector again
                }
#pragma unroll
                for (int i = 0; i < nv(); ++i) m = absmax_bits_bf16x8(xv[i], m);
                return m;
            };
            if (nvec <= 64 * (GEMV_ROW_VEC / 2)) {
                std::integral_constant<int, GEMV_ROW_VEC / 2> nv;
                for (int t = wave; t < it.tokens; t += 2 * nwaves) {
                    uint4 xa[GEMV_ROW_VEC / 2], xb[GEMV_ROW_VEC / 2];
                    const int t2 = t + nwaves < it.tokens ? t + nwaves : t;   // the last row alone: quantized twice, alike
                    const uint32_t ma = request(t, xa, nv), mb = request(t2, xb, nv);
                    finish(t, ma, xa, nv);
                    finish(t2, mb, xb, nv);
                }
            } else {
                std::integral_constant<int, GEMV_ROW_VEC> nv;
                for (int t = wave; t < it.tokens; t += nwaves) {
                    uint4 xa[GEMV_ROW_VEC];
                    const uint32_t ma = request(t, xa, nv);
                    finish(t, ma, xa, nv);
                }
            }
        } else {
            // long rows: pass 1 per-token maxima, pass 2 int8 rows into LDS
            for (int t = 0; t < it.tokens; ++t) {
                uint32_t m = 0;
                for (int idx = threadIdx.x; idx < nvec; idx += nthreads) m = absmax_bits_bf16x8(it.X[(int64_t)t * nvec + idx], m);
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
                    m = o > m ? o : m;
                }
                if (lane == 0) amax_s[t][wave] = m;
            }
            __syncthreads();
            for (int t = 0; t < it.tokens; ++t) {
                uint32_t m = 0;
                for (int w = 0; w < nwaves; ++w) m = amax_s[t][w] > m ? amax_s[t][w] : m;
                const float sc = scale_from_absmax_bits(m);
                if (threadIdx.x == 0) sx_s[t] = sc;
                for (int idx = threadIdx.x; idx < nvec; idx += nthreads)
                    *reinterpret_cast<uint2 *>(xs + t * pitch + idx * 8) = quantize_bf16x8(it.X[(int64_t)t * nvec + idx], sc);
            }
        }
        __syncthreads();
    }

    v4i acc = {0, 0, 0, 0};
    for (int s = wave; s < nsuper; s += nwaves) {
        const uint32_t idxw[4] = {idx4.x, idx4.y, idx4.z, idx4.w};
        const uint32_t codew[4] = {code4.x, code4.y, code4.z, code4.w};
        fetch(s + nwaves);   // the next super-step of this wavefront (zeros past the end)
        // B operand: elements 0..15 pair with the A lanes of quarters 0/1, elements 16..31 with
        // quarters 2/3 (measured operand layout of the instruction)
        if constexpr (DENSE) {
            const uint32_t w8[8] = {idxw[0], idxw[1], idxw[2], idxw[3], codew[0], codew[1], codew[2], codew[3]};
            const int kd = s * 512 + 128 * c4;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint4 bv = make_uint4(0, 0, 0, 0);
                if (tok_ok && kd + 16 * j < K) bv = *reinterpret_cast<const uint4 *>(xrow + kd + 16 * j);
                const v4i b = {(int)bv.x, (int)bv.y, (int)bv.z, (int)bv.w};
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(expand_codes(w8[j], ones), b, acc, 0, 0, 0);
            }
            continue;
        }
        const int kb = s * 512 + 128 * (c4 >> 1) + 16 * (c4 & 1);
        uint32_t iw1[2][2];
        v4i a1[2][2];
        if constexpr (ONE4) {   // the chunk is two index words and two code words
            expand_1of4(idxw[0], idxw[2], ones, iw1[0], a1[0]);
            expand_1of4(idxw[1], idxw[3], ones, iw1[1], a1[1]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k_lo = kb + 32 * j, k_hi = k_lo + 256;
            uint4 blo = make_uint4(0, 0, 0, 0), bhi = make_uint4(0, 0, 0, 0);
            if (tok_ok && k_lo < K) blo = *reinterpret_cast<const uint4 *>(xrow + k_lo);
            if (tok_ok && k_hi < K) bhi = *reinterpret_cast<const uint4 *>(xrow + k_hi);
            const v8i b = {(int)blo.x, (int)blo.y, (int)blo.z, (int)blo.w, (int)bhi.x, (int)bhi.y, (int)bhi.z, (int)bhi.w};
            if constexpr (ONE4)
                acc = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a1[j >> 1][j & 1], b, acc, (int)iw1[j >> 1][j & 1], 0, 0);
            else
                acc = __builtin_amdgcn_smfmac_i32_16x16x128_i8(expand_codes(codew[j], ones), b, acc, (int)idxw[j], 0, 0);
        }
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        for (int w = 1; w < nwaves; ++w) acc += red[w][lane];
        // D layout: lane holds token (lane % 16), rows 4 * (lane / 16) + i
        const int tok = lane & 15, rbase = row0 + 4 * (lane >> 4);
        if (tok < it.tokens) {
            const float scale = __fdiv_rn(*it.gamma, self_quant ? sx_s[tok] : it.sx[tok]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int o = rbase + i;
                if (o < it.d_out) {
                    float y = (float)acc[i] * scale;
                    if (it.bias) y += it.bias[o];
                    it.Y[(int64_t)tok * it.d_out + o] = y;
                    if (it.acc_out) it.acc_out[(int64_t)tok * it.d_out + o] = acc[i];
                }
            }
        }
    }
}

// ---- streaming decode GEMV for grouped calls ---------------------------------------------------
// Persistent blocks, one per multiprocessor: the rows of all problems are cut into units of 16*RT
// rows x the whole input dimension (a contiguous range of packed bytes); every block takes a
// contiguous run of units and hands them to its NW wavefronts one at a time.  The int8 activations
// of the current problem (tokens x d_in) are staged in LDS once per block and problem; the packed weights
// go straight from HBM to registers through a queue of DEPTH super-steps (512 weights each) per
// wavefront, so that several 16-byte loads per lane are always in flight.  No cross-wave reduction.
// The blocks' shares are equal and fixed.  Measured with timestamps (64 x (2560 x 6912), eight tokens, 52 us): the
// blocks finish between 43 and 52 us - multiprocessors in alternate positions of an XCD run about 10 % apart, and so
// do the older and the younger wavefronts of a SIMD - and the wavefronts idle 7 us on average before the kernel ends.
// Holding back a sixth of the units as a device-wide pool for wavefronts out of work did not recover that (52.7 us):
// a unit of 16 rows is 10 us of one wavefront's time at K = 6912, as coarse as the imbalance itself, and a counter
// that 2048 wavefronts ask per unit is far too hot (5800 returning atomics on one word: 55 us), so the pool had to be
// drawn per block, eight units at a time.  Finer balancing would need units split along K across wavefronts.
struct GemvStreamItem {
    const int8_t *xq;
    const float *sx;
    const uint8_t *packed;
    const float *gamma;
    float *Y;
    int d_in, d_out, tokens;
    int input;   // index into GemvStreamTable::in when the kernel quantizes the activations itself, else -1
};
// A distinct activation matrix of the call that the kernel quantizes itself: the first blocks of the
// grid take one token row each (same arithmetic as the quantizer kernels), write the int8 row and its
// scale to the workspace and raise a per-token flag; every block waits for the flags of an input, with
// its first weight loads already in flight, before it stages that input - the quantizer then costs no
// launch of its own.  Rows and scales are ordinary stores and loads; the flag is stored with release
// and, once seen, followed by an acquire fence, both at device scope, so the hand-over rests on the
// language's memory model alone (one L2 write-back per producer block, one invalidation per consumer).
// The wait is bounded: a block out of polls quantizes the rows itself into LDS (same result).
struct GemvStreamInput {
    const uint4 *X;              // bf16 [tokens, d_in]
    unsigned long long *xq;      // workspace, int8 [tokens, d_in] as 8-byte words
    unsigned *sx;                // workspace, fp32 bits [tokens]
    unsigned long long *flags;   // workspace, one per token
    int tokens, d_in;
};
constexpr int GEMV_STREAM_MAX = 64;
constexpr int GEMV_STREAM_INPUTS = 4;
constexpr int GEMV_QUANT_VEC = 4;    // 16-byte vectors of a row per thread when a block quantizes it
constexpr int STAGE_BATCH = 8;       // activation loads a thread has in flight while it stages a block's input in LDS
constexpr int GEMV_OWN_VEC = 14;     // 16-byte vectors of a token row per lane when a wavefront quantizes a row for its own block
struct GemvStreamTable {
    GemvStreamItem it[GEMV_STREAM_MAX];
    int unit0[GEMV_STREAM_MAX + 1];   // first unit of each problem
    int count;
    GemvStreamInput in[GEMV_STREAM_INPUTS];
    int tok0[GEMV_STREAM_INPUTS + 1]; // first producer block of each input
    int nin;
    unsigned epoch;                   // distinguishes this launch's flags from whatever the workspace held
    int spin_limit;
    int share, share_rem;             // units per block: the first share_rem blocks take share + 1, the others share
    int pad;
};
static_assert(sizeof(GemvStreamTable) <= 4096 && sizeof(GemvStreamTable) % 8 == 0, "the table travels as a kernel argument");

// A value every lane holds alike, moved to a scalar register: what is read from the LDS copy of a launch table decides
// loop bounds and branches, which must stay scalar.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ unsigned uni(unsigned x) { return (unsigned)__builtin_amdgcn_readfirstlane((int)x); }
template <typename T> __device__ __forceinline__ T *uni(T *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    // rebuilt as a pointer into global memory, so that what is read through it stays a global (not a flat) access
    typedef T __attribute__((address_space(1))) *global_ptr;
    return (T *)(global_ptr)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ unsigned long long gemv_flag_value(unsigned epoch, int t)
{
    return ((unsigned long long)epoch << 32) | (0x5bd1e995u ^ (unsigned)t);
}

template <int RT, int DEPTH, int NW, int FORM>
__global__ void __launch_bounds__(64 * NW) gemv_stream_kernel(GemvStreamTable tab_arg)
{
    constexpr bool DENSE = FORM == GEMV_DENSE, ONE4 = FORM == GEMV_1OF4;
    constexpr int CB = ONE4 ? 16 : 32;   // bytes of a chunk: the 1:4 form is one 16-byte load per lane and super-step
    extern __shared__ __attribute__((aligned(16))) int8_t xlds[];   // [tokens][d_in + 16]
    // The launch table is fetched once, by the whole block in one round trip, into LDS.  Read through the kernel
    // argument it costs a chain of dependent scalar loads before the first weight load can go out (which problem, its
    // shape, its pointers: a dozen, each a trip to memory: measured 5.6 us from the block's start to its first load).
    __shared__ __attribute__((aligned(16))) GemvStreamTable tab;
    {
        (void)tab_arg;
        const uint2 *src = (const uint2 *)__builtin_amdgcn_kernarg_segment_ptr();   // the table is the only argument
        uint2 *dst = reinterpret_cast<uint2 *>(&tab);
        for (int i = threadIdx.x; i < (int)(sizeof(GemvStreamTable) / 8); i += 64 * NW) dst[i] = src[i];
        __syncthreads();
    }
    __shared__ int unit_ctr;                                        // next unit of the current problem nobody has taken
    __shared__ float sx_lds[16];                                    // s_x of the staged tokens of a self-quantized input
    __shared__ uint32_t wave_amax[NW];
    __shared__ int stage_ok;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // quantize token row t of an input with the whole block: to the workspace (publish) or to the LDS copy
    auto quantize_row = [&](const GemvStreamInput &in, int t, int8_t *lds_row, bool publish) {
        const int nvec = in.d_in / 8;
        const uint4 *row = in.X + (int64_t)t * nvec;
        uint4 v[GEMV_QUANT_VEC];
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < GEMV_QUANT_VEC; ++i) {
            const int idx = threadIdx.x + i * 64 * NW;
            v[i] = idx < nvec ? row[idx] : make_uint4(0, 0, 0, 0);
            m = absmax_bits_bf16x8(v[i], m);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
            m = o > m ? o : m;
        }
        __syncthreads();   // wave_amax is free again
        if (lane == 0) wave_amax[wave] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w) m = wave_amax[w] > m ? wave_amax[w] : m;
        const float s = scale_from_absmax_bits(m);
        if (threadIdx.x == 0) {
            if (publish) in.sx[t] = __float_as_uint(s);
            else sx_lds[t] = s;
        }
#pragma unroll
        for (int i = 0; i < GEMV_QUANT_VEC; ++i) {
            const int idx = threadIdx.x + i * 64 * NW;
            if (idx >= nvec) continue;
            const uint2 q = quantize_bf16x8(v[i], s);
            if (publish)
                reinterpret_cast<uint2 *>(in.xq)[(int64_t)t * nvec + idx] = q;
            else
                reinterpret_cast<uint2 *>(lds_row)[idx] = q;
        }
    };
    auto load_input = [&](int j) {
        const GemvStreamInput &src = tab.in[j];
        GemvStreamInput d;
        d.X = uni(src.X); d.xq = uni(src.xq); d.sx = uni(src.sx); d.flags = uni(src.flags);
        d.tokens = uni(src.tokens); d.d_in = uni(src.d_in);
        return d;
    };
    auto load_item = [&](int i) {
        const GemvStreamItem &src = tab.it[i];
        GemvStreamItem d;
        d.xq = uni(src.xq); d.sx = uni(src.sx); d.packed = uni(src.packed); d.gamma = uni(src.gamma); d.Y = uni(src.Y);
        d.d_in = uni(src.d_in); d.d_out = uni(src.d_out); d.tokens = uni(src.tokens); d.input = uni(src.input);
        return d;
    };
    auto unit0 = [&](int i) { return uni(tab.unit0[i]); };
    // What stands between a block's start and its first requests is a chain of dependent reads of this table, so the
    // chain is kept short: the block's share from two numbers the host divided out, its first problem from one read
    // of all problem boundaries and a vote.
    const unsigned epoch = uni(tab.epoch);
    const int spin_limit = uni(tab.spin_limit);
    const int share = uni(tab.share), share_rem = uni(tab.share_rem);
    const int bound = tab.unit0[1 + lane];   // boundaries past the last problem hold the total
    if ((int)blockIdx.x < uni(tab.tok0[GEMV_STREAM_INPUTS])) {   // producer role: one token row of one input
        int j = 0;
        while ((int)blockIdx.x >= uni(tab.tok0[j + 1])) ++j;
        const GemvStreamInput in = load_input(j);
        const int t = (int)blockIdx.x - uni(tab.tok0[j]);
        quantize_row(in, t, nullptr, true);
        // The row and its scale are ordinary stores. The barrier orders every thread's part before thread 0,
        // whose release store of the flag makes all of it visible to the whole device before the flag is.
        __syncthreads();
        if (threadIdx.x == 0)
            __hip_atomic_store(&in.flags[t], gemv_flag_value(epoch, t), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int b0 = share * (int)blockIdx.x + ((int)blockIdx.x < share_rem ? (int)blockIdx.x : share_rem);
    const int b1 = b0 + share + ((int)blockIdx.x < share_rem ? 1 : 0);
    const int r = lane & 15, c4 = lane >> 4;
    const uint32_t ones = vgpr_ones();
    // the block's first problem: as many problems end at or before its first unit
    int item = __builtin_popcountll(__ballot(bound <= b0));
    int u = b0;
    const int8_t *staged_xq = nullptr;   // what the LDS copy currently holds (block-uniform)
    int staged_tokens = 0, staged_k = 0;
    bool first_problem = true;
    while (u < b1) {
        while (u >= unit0(item + 1)) ++item;
        const GemvStreamItem it = load_item(item);
        const int item_u0 = unit0(item), item_u1 = unit0(item + 1);
        const int seg_end = b1 < item_u1 ? b1 : item_u1;
        const int ua = u - item_u0, ub = seg_end - item_u0;   // units of this problem for the block
        u = seg_end;
        const int K = it.d_in, nchunks = K / CHUNK, nsuper = (nchunks + 3) / 4, pitch = K + 16;
        const bool tok_ok = r < it.tokens;
        const int xoff = (tok_ok ? r : 0) * pitch + (DENSE ? 128 * c4 : 128 * (c4 >> 1) + 16 * (c4 & 1));
        const bool ragged = (nchunks & 3) != 0;   // the last super-step of a unit then covers fewer than four chunks

        // Wavefronts of a block advance at very different speeds (measured: the first one to finish
        // an equal share is done in half the time of the last), so the units of the block are handed
        // out one at a time from a counter in LDS: wavefront w starts with unit ua + w and takes the
        // next free one whenever its load stream reaches the end of a unit.  The loads run DEPTH
        // super-steps ahead of the arithmetic; with nsuper > DEPTH they are at most one unit ahead,
        // so one register (nu) carries the unit number from the load side to the arithmetic.  Shorter
        // rows fall back to equal contiguous shares.
        const bool dyn = nsuper > DEPTH;
        const int wa = dyn ? ua + wave : ua + (int)((int64_t)(ub - ua) * wave / NW);
        const int wb = dyn ? ub : ua + (int)((int64_t)(ub - ua) * (wave + 1) / NW);   // first unit number that is not this wavefront's
        __syncthreads();   // nobody still uses the previous problem's counter or activations
        if (threadIdx.x == 0) unit_ctr = ua + NW;
        int iu = wa, is = 0, cu = wa, cs = 0, nu = wb;
        int grabbed = wb;   // prefetched from the counter one unit ahead of its use
        uint4 qi[DEPTH][RT], qc[DEPTH][RT];
        // Every load is unconditional, so the loop below is straight-line code and the wait the
        // compiler places before a slot is consumed leaves the DEPTH - 1 younger super-steps in
        // flight (a load inside a branch makes it wait for everything).  Past the end of the
        // wavefront's work the last unit is fetched again (cache hits, no HBM traffic) and ignored.
        // The lane's packed rows of the unit being loaded: the 64-bit address arithmetic runs once per unit, a load
        // adds the chunk's offset (the vector unit is the scarce resource of the 1:4 form).
        const uint8_t *prow[RT];
        auto locate = [&](int unit) {
#pragma unroll
            for (int a = 0; a < RT; ++a) {
                int row = unit * 16 * RT + 16 * a + r;
                row = row < it.d_out ? row : it.d_out - 1;
                prow[a] = it.packed + (int64_t)row * nchunks * CB;
            }
        };
        locate(wa < wb ? wa : ub - 1);
        auto issue = [&](uint4(&ib)[RT], uint4(&cb)[RT]) {
            int ch = 4 * is + c4;
            ch = ch < nchunks ? ch : nchunks - 1;
#pragma unroll
            for (int a = 0; a < RT; ++a) {
                const uint8_t *p = prow[a] + (uint32_t)ch * CB;
                ib[a] = *reinterpret_cast<const uint4 *>(p);        // plain loads: nontemporal ones measured 30 % slower
                if constexpr (ONE4) cb[a] = make_uint4(0, 0, 0, 0);
                else cb[a] = *reinterpret_cast<const uint4 *>(p + 16);
            }
            if (++is == nsuper) {
                is = 0;
                if (dyn) {
                    iu = nu = __builtin_amdgcn_readfirstlane(grabbed);
                    if (lane == 0) grabbed = atomicAdd(&unit_ctr, 1);
                } else {
                    ++iu;
                }
                locate(iu < wb ? iu : ub - 1);
            }
        };
        // Activations are staged only when they differ from what the block already holds (projections
        // that share an input, Q/K/V or up/gate, come one after the other).
        const bool restage = it.xq != staged_xq || it.tokens != staged_tokens || K != staged_k;
        const bool self_quant = it.input >= 0;
        // The input of a block's FIRST problem is quantized by the block itself, a wavefront per token row with the
        // whole row in registers: one trip to memory for the bf16 rows (requested before the weight queue fills),
        // a wavefront-level maximum, the int8 row written straight into LDS.  Waiting for the producer blocks
        // instead put the staged activations 8-10 us behind the block's start (row read, release, poll, acquire,
        // staging read: five trips in a row) with only the DEPTH queued super-steps of weights to cover them.
        // Inputs that a block meets later were published by the producer blocks long before.
        const bool own = restage && self_quant && first_problem && K <= 8 * 64 * GEMV_OWN_VEC;
        first_problem = false;
        uint4 xv[GEMV_OWN_VEC];
        const uint4 *own_X = nullptr;
        auto own_request = [&](int t) {
            const uint4 *row = own_X + (int64_t)t * (K / 8);
#pragma unroll
            for (int i = 0; i < GEMV_OWN_VEC; ++i) {
                if (64 * i >= K / 8) break;   // the same for every lane
                const int idx = lane + 64 * i;
                xv[i] = row[idx < K / 8 ? idx : K / 8 - 1];   // past the end the last vector again: the maximum is the same
            }
        };
        auto own_quantize = [&](int t) {
            uint32_t m = 0;
#pragma unroll
            for (int i = 0; i < GEMV_OWN_VEC; ++i) {
                if (64 * i >= K / 8) break;
                m = absmax_bits_bf16x8(xv[i], m);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const uint32_t o = (uint32_t)__shfl_xor((int)m, off, 64);
                m = o > m ? o : m;
            }
            const float s = scale_from_absmax_bits(m);
            if (lane == 0) sx_lds[t] = s;
            uint2 *lds_row = reinterpret_cast<uint2 *>(xlds + t * pitch);
#pragma unroll
            for (int i = 0; i < GEMV_OWN_VEC; ++i) {
                if (64 * i >= K / 8) break;
                const int idx = lane + 64 * i;
                if (idx < K / 8) lds_row[idx] = quantize_bf16x8(xv[i], s);
            }
        };
        if (own) {
            own_X = uni(tab.in[it.input].X);
            if (wave < it.tokens) own_request(wave);
        }
        // copy tokens x K quantized activations into the LDS rows; the loads go out in batches so that
        // their latencies overlap instead of adding up
        auto stage = [&](const int8_t *src, int tokens) {
            const int n16 = tokens * (K / 16);
            for (int v0 = threadIdx.x; v0 < n16; v0 += 64 * NW * STAGE_BATCH) {
                uint4 q[STAGE_BATCH];
#pragma unroll
                for (int b = 0; b < STAGE_BATCH; ++b) {
                    const int v = v0 + 64 * NW * b;
                    q[b] = *reinterpret_cast<const uint4 *>(src + (int64_t)(v < n16 ? v : n16 - 1) * 16);
                }
#pragma unroll
                for (int b = 0; b < STAGE_BATCH; ++b) {
                    // past the end the last vector is written again (same bytes, same place): no branch, so the batch
                    // stays in registers
                    const int v = v0 + 64 * NW * b < n16 ? v0 + 64 * NW * b : n16 - 1;
                    *reinterpret_cast<uint4 *>(&xlds[(v / (K / 16)) * pitch + (v % (K / 16)) * 16]) = q[b];
                }
            }
        };
        if (restage && !self_quant) stage(it.xq, it.tokens);
        __syncthreads();   // counter and activations in place
        if (dyn && lane == 0) grabbed = atomicAdd(&unit_ctr, 1);
        if (wa < wb) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) issue(qi[d], qc[d]);
        }
        if (own) {
            for (int t = wave; t < it.tokens; t += NW) {
                if (t != wave) own_request(t);
                own_quantize(t);
            }
            __syncthreads();
        } else if (restage && self_quant) {
            // the first weight loads are in flight; now wait (bounded) for the blocks that quantize this input
            const GemvStreamInput in = load_input(it.input);
            if (threadIdx.x == 0) stage_ok = 1;
            __syncthreads();
            if ((int)threadIdx.x < in.tokens) {
                const unsigned long long want = gemv_flag_value(epoch, threadIdx.x);
                int spins = 0, ok = spin_limit >= 0;
                while (ok && __hip_atomic_load(&in.flags[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != want) {
                    if (++spins > spin_limit) ok = 0;
                    else __builtin_amdgcn_s_sleep(4);
                }
                if (!ok) stage_ok = 0;   // several lanes may write the same value
                // acquire: what the producers stored before their flags is what the loads below see; the
                // barrier hands that on to the block's other threads
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            __syncthreads();
            if (!stage_ok) {   // out of patience: quantize the rows here, straight into LDS (same arithmetic, same result)
                for (int t = 0; t < in.tokens; ++t) quantize_row(in, t, xlds + t * pitch, false);
            } else {
                if ((int)threadIdx.x < in.tokens) sx_lds[threadIdx.x] = __uint_as_float(in.sx[threadIdx.x]);
                stage(reinterpret_cast<const int8_t *>(in.xq), in.tokens);
            }
            __syncthreads();
        }
        if (restage) {
            staged_xq = it.xq;
            staged_tokens = it.tokens;
            staged_k = K;
        }
        const float scale = tok_ok ? __fdiv_rn(*it.gamma, self_quant ? sx_lds[r] : it.sx[r]) : 0.0f;

        v4i acc[RT];
#pragma unroll
        for (int a = 0; a < RT; ++a) acc[a] = v4i{0, 0, 0, 0};
        // Lanes of absent tokens read token 0's activations (their accumulator columns are never
        // stored); activations past the input dimension are read from the slack behind the staged
        // rows and meet zero codes.
        while (cu < wb) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                uint4 ic[RT], cc[RT];
#pragma unroll
                for (int a = 0; a < RT; ++a) { ic[a] = qi[d][a]; cc[a] = qc[d][a]; }
                issue(qi[d], qc[d]);
                if ((ragged && cs == nsuper - 1 && 4 * cs + c4 >= nchunks) || cu >= wb) {
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        cc[a] = make_uint4(0, 0, 0, 0);
                        if constexpr (DENSE) ic[a] = make_uint4(0, 0, 0, 0);   // all eight words are codes
                        if constexpr (ONE4) ic[a].z = ic[a].w = 0;             // the chunk's two code words
                    }
                }
                if constexpr (DENSE) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const v4i b = *reinterpret_cast<const v4i *>(&xlds[xoff + cs * 512 + 16 * j]);
#pragma unroll
                        for (int a = 0; a < RT; ++a) {
                            const uint4 &half = j < 4 ? ic[a] : cc[a];
                            const uint32_t cw = (j & 3) == 0 ? half.x : (j & 3) == 1 ? half.y : (j & 3) == 2 ? half.z : half.w;
                            acc[a] = __builtin_amdgcn_mfma_i32_16x16x64_i8(expand_codes(cw, ones), b, acc[a], 0, 0, 0);
                        }
                    }
                }
                // sparse forms: the super-step's activations are asked for first, so that the LDS latency passes under
                // the vector work that builds the A operands
                v8i bq[DENSE ? 1 : 4];
#pragma unroll
                for (int j = 0; j < (DENSE ? 0 : 4); ++j) {
                    const uint4 blo = *reinterpret_cast<const uint4 *>(&xlds[xoff + cs * 512 + 32 * j]);
                    const uint4 bhi = *reinterpret_cast<const uint4 *>(&xlds[xoff + cs * 512 + 32 * j + 256]);
                    bq[j] = v8i{(int)blo.x, (int)blo.y, (int)blo.z, (int)blo.w, (int)bhi.x, (int)bhi.y, (int)bhi.z, (int)bhi.w};
                }
                uint32_t iw1[RT][2][2];
                v4i a1[RT][2][2];
                if constexpr (ONE4) {
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        expand_1of4(ic[a].x, ic[a].z, ones, iw1[a][0], a1[a][0]);
                        expand_1of4(ic[a].y, ic[a].w, ones, iw1[a][1], a1[a][1]);
                    }
                }
#pragma unroll
                for (int j = 0; j < (DENSE ? 0 : 4); ++j) {
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        if constexpr (ONE4) {
                            acc[a] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a1[a][j >> 1][j & 1], bq[j], acc[a], (int)iw1[a][j >> 1][j & 1], 0, 0);
                            continue;
                        }
                        const uint32_t cw = j == 0 ? cc[a].x : j == 1 ? cc[a].y : j == 2 ? cc[a].z : cc[a].w;
                        const uint32_t iw = j == 0 ? ic[a].x : j == 1 ? ic[a].y : j == 2 ? ic[a].z : ic[a].w;
                        acc[a] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(expand_codes(cw, ones), bq[j], acc[a], (int)iw, 0, 0);
                    }
                }
                if (++cs == nsuper) {
                    // unit cu complete: lane holds token r, rows 4 * c4 + i of each row tile
                    if (tok_ok && cu < wb) {
#pragma unroll
                        for (int a = 0; a < RT; ++a) {
                            const int o = cu * 16 * RT + 16 * a + 4 * c4;
                            if (o + 3 < it.d_out && (it.d_out & 3) == 0) {
                                const v4f y = {(float)acc[a][0] * scale, (float)acc[a][1] * scale, (float)acc[a][2] * scale,
                                               (float)acc[a][3] * scale};
                                // streaming store: Y is not read again here and should not displace the weight stream in L2
                                __builtin_nontemporal_store(y, reinterpret_cast<v4f *>(it.Y + (int64_t)r * it.d_out + o));
                            } else {
                                for (int i = 0; i < 4; ++i)
                                    if (o + i < it.d_out) it.Y[(int64_t)r * it.d_out + o + i] = (float)acc[a][i] * scale;
                            }
                        }
                    }
#pragma unroll
                    for (int a = 0; a < RT; ++a) acc[a] = v4i{0, 0, 0, 0};
                    cs = 0;
                    cu = dyn ? nu : cu + 1;
                }
            }
        }
    }
}

// ---- generic path: any supported pattern, plain integer arithmetic ---------------------------------
// One thread per output row, eight tokens per block row; decodes every slot of the packed row.
__global__ void __launch_bounds__(128) linear_generic_kernel(const int8_t *__restrict__ xq, const float *__restrict__ sx,
                                                            const uint8_t *__restrict__ packed, const float *gamma,
                                                            const float *bias, float *Y, int32_t *acc_out,
                                                            int64_t tokens, int d_in, int d_out, Pattern pat)
{
    const int o = blockIdx.x * 128 + threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.y * 8;
    if (o >= d_out) return;
    const int nchunks = (d_in + CHUNK - 1) / CHUNK;
    int acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int c = 0; c < nchunks; ++c) {
        const uint8_t *idx_field = packed + ((int64_t)o * nchunks + c) * pat.chunk_bytes;
        const uint8_t *code_field = idx_field + pat.idx_bytes;
        for (int s = 0; s < pat.slots; ++s) {
            const int v = s & 15;
            const int cp = 32 * (s >> 4) + 8 * (v & 3) + 2 * (v >> 2);
            const uint32_t code = (code_field[cp >> 3] >> (cp & 7)) & 3u;
            if (code == 0) continue;
            int j = s % pat.N;
            if (pat.b) {
                const int p = s * pat.b;
                const uint32_t two = (uint32_t)idx_field[p >> 3] | ((uint32_t)idx_field[(p >> 3) + ((p >> 3) + 1 < pat.idx_bytes ? 1 : 0)] << 8);
                j = (two >> (p & 7)) & ((1u << pat.b) - 1u);
            }
            const int col = c * CHUNK + (s / pat.N) * pat.M + j;
            if (col >= d_in) continue;
            const int w = code == 1u ? 1 : -1;
#pragma unroll
            for (int tt = 0; tt < 8; ++tt)
                if (t0 + tt < tokens) acc[tt] += w * (int)xq[(t0 + tt) * d_in + col];
        }
    }
    const float g = *gamma;
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) {
        if (t0 + tt >= tokens) break;
        float y = (float)acc[tt] * __fdiv_rn(g, sx[t0 + tt]);
        if (bias) y += bias[o];
        Y[(t0 + tt) * d_out + o] = y;
        if (acc_out) acc_out[(t0 + tt) * d_out + o] = acc[tt];
    }
}

}  // namespace

size_t linear_workspace_bytes(int64_t tokens, int64_t d_out, int64_t d_in)
{
    // int8 activations + per-token scales + dense int8 weights of the comparison path
    return align_up((size_t)tokens * d_in, 256) + align_up((size_t)tokens * sizeof(float), 256) +
           align_up((size_t)d_out * d_in, 256);
}

sbn_status launch_act_quant(const void *X, int64_t tokens, int64_t d_in, int8_t *xq, float *sx, hipStream_t stream)
{
    const uint4 *x = static_cast<const uint4 *>(X);
    const int nvec = (int)(d_in / 8);
    if (tokens <= 64 && nvec <= 2 * 1024) {
        hipLaunchKernelGGL((act_quant_kernel<1024, 2>), dim3((unsigned)tokens), dim3(1024), 0, stream, x, tokens, nvec, xq, sx);
    } else if (nvec <= 2 * 256) {
        // a block of four wavefronts per token (measured against one or two wavefronts per token with longer loops: same
        // kernel time, but the step that follows starts 1-2 % earlier)
        hipLaunchKernelGGL((act_quant_kernel<256, 2>), dim3((unsigned)tokens), dim3(256), 0, stream, x, tokens, nvec, xq, sx);
    } else if (nvec <= 4 * 256) {
        hipLaunchKernelGGL((act_quant_kernel<256, 4>), dim3((unsigned)tokens), dim3(256), 0, stream, x, tokens, nvec, xq, sx);
    } else {
        hipLaunchKernelGGL(act_quant_two_pass_kernel, dim3((unsigned)ceil_div(tokens, 4)), dim3(256), 0, stream, x, tokens, nvec, xq, sx);
    }
    return check_launch("act_quant_kernel");
}

sbn_status launch_rmsnorm_act_quant(const void *X, const float *gain, float eps, int64_t tokens, int64_t d_in, int8_t *xq,
                                    float *sx, void *xn, hipStream_t stream)
{
    const uint4 *x = static_cast<const uint4 *>(X);
    uint4 *n = static_cast<uint4 *>(xn);
    const int nvec = (int)(d_in / 8);
    if (nvec <= 2 * 256 && tokens > 64) {
        hipLaunchKernelGGL((rmsnorm_act_quant_kernel<256, 2>), dim3((unsigned)tokens), dim3(256), 0, stream, x, gain, eps, tokens, nvec,
                           xq, sx, n);
    } else if (nvec <= 4 * 256 && tokens > 64) {
        hipLaunchKernelGGL((rmsnorm_act_quant_kernel<256, 4>), dim3((unsigned)tokens), dim3(256), 0, stream, x, gain, eps, tokens, nvec,
                           xq, sx, n);
    } else if (nvec <= 2 * 1024) {
        hipLaunchKernelGGL((rmsnorm_act_quant_kernel<1024, 2>), dim3((unsigned)tokens), dim3(1024), 0, stream, x, gain, eps, tokens,
                           nvec, xq, sx, n);
    } else {
        return SBN_EUNSUPPORTED;   // rows longer than 16384 do not fit the registers of a block
    }
    return check_launch("rmsnorm_act_quant_kernel");
}

static void fill_gemv_item(GemvItem &g, const LinearItem &li)
{
    g.xq = li.xq; g.sx = li.sx; g.packed = static_cast<const uint8_t *>(li.packed);
    g.gamma = li.gamma; g.bias = li.bias; g.Y = li.Y; g.acc_out = li.acc_out;
    g.d_in = (int)li.d_in; g.d_out = (int)li.d_out; g.tokens = (int)li.tokens; g.pad = 0;
    g.X = nullptr;
}

// multiprocessors of the current device (cached per thread)
int device_cus()
{
    static thread_local int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

template <int FORM>
static sbn_status launch_gemv_as(int count, const LinearItem *items, hipStream_t stream);

sbn_status launch_gemv(int count, const LinearItem *items, GemvForm form, hipStream_t stream)
{
    switch (form) {
    case GEMV_2OF4: return launch_gemv_as<GEMV_2OF4>(count, items, stream);
    case GEMV_DENSE: return launch_gemv_as<GEMV_DENSE>(count, items, stream);
    case GEMV_1OF4: return launch_gemv_as<GEMV_1OF4>(count, items, stream);
    }
    return SBN_EINVAL;
}

// Launch number of the streaming kernel with the fused quantizer: it tags the per-token flags a launch raises in
// the caller's workspace (never cleared), so that flags left by any earlier launch - of either instantiation of
// the kernel, on any workspace - can never be taken for this launch's.  One counter for the whole library.
static std::atomic<unsigned> g_gemv_stream_epoch{1};

// true while `stream` records into a graph (or when that cannot be told)
static bool stream_is_capturing(hipStream_t stream)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &status) != hipSuccess) {
        (void)hipGetLastError();
        return true;
    }
    return status != hipStreamCaptureStatusNone;
}

template <int FORM>
static sbn_status launch_gemv_as(int count, const LinearItem *items, hipStream_t stream)
{
    constexpr int RT = 1;
    static thread_local std::vector<const int8_t *> written;   // xq buffers a quantizer kernel of this call has filled
    written.clear();
    // quantizer launches for the problems first .. first + n - 1 that still need one (shared inputs once)
    auto quantize_run = [&](int first, int n) -> sbn_status {
        for (int i = 0; i < n; ++i) {
            const LinearItem &li = items[first + i];
            if (li.quantized || std::find(written.begin(), written.end(), li.xq) != written.end()) continue;
            sbn_status st = launch_act_quant(li.X, li.tokens, li.d_in, li.xq, li.sx, stream);
            if (st != SBN_OK) return st;
            written.push_back(li.xq);
        }
        return SBN_OK;
    };
    int first = 0;
    while (first < count) {
        // --- persistent streaming kernel when a run of problems holds enough rows to keep every block busy
        int n = count - first < GEMV_STREAM_MAX ? count - first : GEMV_STREAM_MAX;
        int64_t units = 0, lds_need = 16;
        bool plain = true;
        for (int i = 0; i < n; ++i) {
            const LinearItem &li = items[first + i];
            units += ceil_div(li.d_out, 16 * RT);
            const int64_t b = li.tokens * (li.d_in + 16) + 512;   // slack: reads past a ragged input dimension stay inside
            lds_need = b > lds_need ? b : lds_need;
            if (li.bias || li.acc_out) plain = false;
        }
        // one block of NW wavefronts per multiprocessor, sharing one staged copy of the activations
        const int nblocks = device_cus();
        constexpr int GEMV_STREAM_LDS = 160 * 1024 - 4608;   // the kernel's copy of the launch table, its counter and scales are static LDS
        if (plain && lds_need <= GEMV_STREAM_LDS && units >= 16 * (int64_t)nblocks) {
            // One row tile per unit, DEPTH 5 and 8 wavefronts per block measured best among one or two row tiles,
            // depths 2..8 and 6..16 wavefronts (more wavefronts finish their shares further apart, fewer leave too
            // few loads in flight; units of 16 rows balance the wavefronts better than units of 32: +2.5 to +4 %)
            // (the 1:4 form has half the bytes per super-step: twice the depth keeps the same bytes in flight)
            constexpr int DEPTH = FORM == GEMV_1OF4 ? 10 : 5, NW = 8;
            GemvStreamTable tab;
            tab.count = n;
            tab.nin = 0;
            for (int j = 0; j <= GEMV_STREAM_INPUTS; ++j) tab.tok0[j] = 0;
            // the kernel quantizes up to GEMV_STREAM_INPUTS distinct inputs itself; more than that (or rows too
            // long for one block's registers) go through the quantizer kernel first
            // Not under stream capture: the flags carry a per-launch number that the host hands out, and a replayed
            // graph would present the previous replay's flags again.  A captured launch takes the quantizer kernels.
            // One case needs neither flags nor producer blocks and is taken under capture as well: every problem of
            // the launch reads the same unquantized input and its rows fit a wavefront's registers; each block then
            // quantizes that input once, for itself, in front of its first problem and never stages anything else.
            bool fuse = true, one_input = true;
            int nin = 0;
            const int8_t *in_xq[GEMV_STREAM_INPUTS];
            for (int i = 0; i < n && fuse; ++i) {
                const LinearItem &li = items[first + i];
                if (li.quantized || std::find(written.begin(), written.end(), li.xq) != written.end()) { one_input = false; continue; }
                if (li.d_in > 8 * GEMV_QUANT_VEC * 64 * NW || li.tokens > 16) { fuse = false; break; }
                if (li.d_in > 8 * 64 * GEMV_OWN_VEC) one_input = false;
                bool seen = false;
                for (int j = 0; j < nin; ++j) seen = seen || in_xq[j] == li.xq;
                if (seen) continue;
                if (nin == GEMV_STREAM_INPUTS) { fuse = false; break; }
                in_xq[nin++] = li.xq;
            }
            one_input = one_input && fuse && nin == 1;
            if (fuse && !one_input && stream_is_capturing(stream)) fuse = false;
            if (!fuse) {
                sbn_status st = quantize_run(first, n);
                if (st != SBN_OK) return st;
                nin = 0;
            }
            int u = 0;
            for (int i = 0; i < n; ++i) {
                const LinearItem &li = items[first + i];
                GemvStreamItem &g = tab.it[i];
                g.xq = li.xq; g.sx = li.sx; g.packed = static_cast<const uint8_t *>(li.packed); g.gamma = li.gamma; g.Y = li.Y;
                g.d_in = (int)li.d_in; g.d_out = (int)li.d_out; g.tokens = (int)li.tokens; g.input = -1;
                for (int j = 0; j < nin; ++j)
                    if (in_xq[j] == li.xq) {
                        g.input = j;
                        if (j == tab.nin) {   // first problem with this input: describe it
                            GemvStreamInput &in = tab.in[j];
                            in.X = static_cast<const uint4 *>(li.X);
                            in.xq = reinterpret_cast<unsigned long long *>(li.xq);
                            in.sx = reinterpret_cast<unsigned *>(li.sx);
                            // the scales of at most 16 tokens fill 64 bytes of their 256-byte region; the flags take its second half
                            in.flags = reinterpret_cast<unsigned long long *>(reinterpret_cast<uint8_t *>(li.sx) + 128);
                            in.tokens = (int)li.tokens; in.d_in = (int)li.d_in;
                            tab.tok0[j + 1] = tab.tok0[j] + in.tokens;
                            ++tab.nin;
                        }
                    }
                tab.unit0[i] = u;
                u += (int)ceil_div(li.d_out, 16 * RT);
            }
            for (int i = n; i <= GEMV_STREAM_MAX; ++i) tab.unit0[i] = u;
            tab.share = u / nblocks;
            tab.share_rem = u % nblocks;
            tab.pad = 0;
            for (int j = tab.nin; j < GEMV_STREAM_INPUTS; ++j) tab.tok0[j + 1] = tab.tok0[tab.nin];
            if (one_input)   // no producer blocks: nobody would read what they publish
                for (int j = 0; j <= GEMV_STREAM_INPUTS; ++j) tab.tok0[j] = 0;
            tab.epoch = g_gemv_stream_epoch.fetch_add(1, std::memory_order_relaxed);
            tab.spin_limit = gemv_spin_limit();
            static thread_local bool raised = false;
            if (!raised) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemv_stream_kernel<RT, DEPTH, NW, FORM>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, GEMV_STREAM_LDS);
                if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute"); return SBN_EHIP; }
                raised = true;
            }
            hipLaunchKernelGGL((gemv_stream_kernel<RT, DEPTH, NW, FORM>), dim3(nblocks), dim3(64 * NW), (size_t)lds_need, stream, tab);
            sbn_status st = check_launch("gemv_stream_kernel");
            if (st != SBN_OK) return st;
            first += n;
            continue;
        }
        // --- otherwise: one block per 16 rows, wavefronts split the input dimension (lowest latency)
        n = count - first < GEMV_MAX_ITEMS ? count - first : GEMV_MAX_ITEMS;
        // the blocks quantize the activations themselves (measured at 6912 x 2560 and 2560 x 6912: 9.3-9.7 us for
        // 1-16 tokens against 12 us with the quantizer launched in front; a wavefront per token row with the row in
        // registers - walking the tokens one after the other cost a trip to memory per token and pass: 13-16 us at 8)
        constexpr int64_t GEMV_SELF_QUANT_LDS = 112 * 1024;
        constexpr int64_t GEMV_SELF_QUANT_TOKENS = 16;
        int64_t dyn_lds = 0;
        bool self_quant = true;
        for (int i = 0; i < n; ++i) {
            const LinearItem &li = items[first + i];
            if (li.quantized) continue;
            const int64_t b = li.tokens * (li.d_in + 16);
            if (b > GEMV_SELF_QUANT_LDS || li.tokens > GEMV_SELF_QUANT_TOKENS ||
                std::find(written.begin(), written.end(), li.xq) != written.end())
                self_quant = false;
            dyn_lds = b > dyn_lds ? b : dyn_lds;
        }
        if (!self_quant) {
            sbn_status st = quantize_run(first, n);
            if (st != SBN_OK) return st;
            dyn_lds = 0;
        }
        GemvTable tab;
        int blocks = 0, max_super = 1;
        for (int i = 0; i < n; ++i) {
            const LinearItem &li = items[first + i];
            fill_gemv_item(tab.it[i], li);
            if (self_quant && !li.quantized) tab.it[i].X = static_cast<const uint4 *>(li.X);
            const int nb = (int)ceil_div(li.d_out, 16);
            blocks = nb > blocks ? nb : blocks;
            const int nsuper = (int)ceil_div(li.d_in / CHUNK, 4);
            max_super = nsuper > max_super ? nsuper : max_super;
        }
        // one wavefront per super-step up to 16, so that every wavefront has loads in flight at once
        const int nwaves = max_super < 16 ? max_super : 16;
        if (dyn_lds > 0) {
            static thread_local bool raised_single = false;
            if (!raised_single) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemv_smfmac_kernel<FORM>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMV_SELF_QUANT_LDS);
                if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute"); return SBN_EHIP; }
                raised_single = true;
            }
        }
        hipLaunchKernelGGL(gemv_smfmac_kernel<FORM>, dim3(blocks, n), dim3(64 * nwaves), (size_t)dyn_lds, stream, tab);
        sbn_status st = check_launch("gemv_smfmac_kernel");
        if (st != SBN_OK) return st;
        first += n;
    }
    return SBN_OK;
}

sbn_status launch_linear_generic(const LinearItem &it, const Pattern &pat, hipStream_t stream)
{
    dim3 grid((unsigned)ceil_div(it.d_out, 128), (unsigned)ceil_div(it.tokens, 8));
    hipLaunchKernelGGL(linear_generic_kernel, grid, dim3(128), 0, stream, it.xq, it.sx,
                       static_cast<const uint8_t *>(it.packed), it.gamma, it.bias, it.Y, it.acc_out, it.tokens,
                       (int)it.d_in, (int)it.d_out, pat);
    return check_launch("linear_generic_kernel");
}

}  // namespace sbn
