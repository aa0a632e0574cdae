// Backward products of the sparse ternary linear layer under the dual straight-through estimator
// (Section 2.3; Appendix B listing, backward()):
//   dX[t,k] = gamma * sum_o dY[t,o] * W_eff[o,k]          contraction over d_out
//   dW[o,k] = sum_t (dY[t,o] / s_x[t]) * xq[t,k]          contraction over tokens; dense, unmasked
// Both run on the dense bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): the 2:4
// structure lies along d_in, which is not the contracted dimension of either product, so the sparse
// instruction does not apply.  One "NT" GEMM kernel serves both; small layout kernels put the
// operands contraction-major first (ternary values and int8 activations are exact in bf16).
#include <algorithm>
#include <vector>

#include "sbn_internal.hpp"
#include "sbn_mfma.hpp"

namespace sbn {

namespace {

__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;   // round to nearest even; inputs are finite
}

// ---- layout kernels -------------------------------------------------------------------------------
constexpr int TP = 64 + 8;   // padded LDS row (bf16 elements) of the 64-wide transposition tiles

// writes a [rows][64] bf16 LDS tile (row pitch TP) to dst[(r0 + row) * ld + c0 + 0..63], 16 bytes per thread
__device__ __forceinline__ void write_tile_rows(const uint16_t *tile, int rows, uint16_t *dst, int64_t ld, int64_t r0,
                                                int64_t c0, int64_t rmax, int64_t cmax)
{
    for (int v = threadIdx.x; v < rows * 8; v += 256) {
        const int row = v >> 3, col = (v & 7) * 8;
        if (r0 + row >= rmax) continue;
        const uint16_t *s = tile + row * TP + col;
        uint16_t *d = dst + (r0 + row) * ld + c0 + col;
        if (c0 + col + 8 <= cmax) {
            *reinterpret_cast<uint4 *>(d) = *reinterpret_cast<const uint4 *>(s);
        } else {
            for (int e = 0; e < 8; ++e)
                if (c0 + col + e < cmax) d[e] = s[e];
        }
    }
}

// packed 2:4 weights -> W_eff^T as bf16 [d_in, ld] (ld >= d_out): block = 64 rows of W x one chunk
__global__ void __launch_bounds__(256) unpack_transpose_kernel(const uint8_t *__restrict__ packed, int d_out, int d_in,
                                                              uint16_t *__restrict__ wt, int64_t ld)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[128 * TP];
    const int nchunks = d_in / CHUNK;
    const int chunk = blockIdx.x, o0 = blockIdx.y * 64;
    const int ro = threadIdx.x & 63, word = threadIdx.x >> 6;
    const int o = o0 + ro;
    for (int k = 0; k < 32; ++k) tile[(32 * word + k) * TP + ro] = 0;
    if (o < d_out) {
        const uint32_t *cw = reinterpret_cast<const uint32_t *>(packed + ((int64_t)o * nchunks + chunk) * 32);
        const uint32_t idx = cw[word], codes = cw[4 + word];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int v = 2 * t + h;
                const uint32_t code = (codes >> (8 * (v & 3) + 2 * (v >> 2))) & 3u;
                const uint32_t pos = (idx >> (4 * t + 2 * h)) & 3u;
                if (code) tile[(32 * word + 4 * t + pos) * TP + ro] = code == 1u ? 0x3f80u : 0xbf80u;
            }
        }
    }
    __syncthreads();
    write_tile_rows(tile, 128, wt, ld, (int64_t)chunk * CHUNK, o0, d_in, ld);
}

// Transposition of a 64 x 64 bf16 tile through LDS: rows go in as they are read (vector loads along
// the source's contiguous dimension), come out as eight values of one column per thread
// (ds_read_u16 with a pitch of 33 words: the 64 lanes of a read hit 32 different banks, two lanes
// per word), and leave as 16-byte stores, eight lanes per 128-byte line of the destination.
constexpr int TQ = 66;   // LDS row pitch of these tiles in bf16 elements (33 words)

// tile[a][b] (a = source row, b = source column) -> dst[(c0 + b) * ld + r0 + a]
__device__ __forceinline__ void write_tile_transposed(const uint16_t *tile, uint16_t *dst, int64_t ld, int64_t c0, int64_t r0,
                                                      int64_t cmax, int64_t rmax)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int v = threadIdx.x + 256 * h;
        const int b = v >> 3, av = (v & 7) * 8;
        if (c0 + b >= cmax) continue;
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)tile[(av + 2 * i) * TQ + b] | ((uint32_t)tile[(av + 2 * i + 1) * TQ + b] << 16);
        uint16_t *d = dst + (c0 + b) * ld + r0 + av;
        if (r0 + av + 8 <= rmax && (ld & 7) == 0) {
            *reinterpret_cast<uint4 *>(d) = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            for (int e = 0; e < 8; ++e)
                if (r0 + av + e < rmax) d[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
    }
}

// int8 [rows, cols] -> bf16 transposed: dst [cols, ld] with dst[c, r] = src[r, c], zeros for r in [rows, ld)
__global__ void __launch_bounds__(256) transpose_i8_kernel(const int8_t *__restrict__ src, int64_t rows, int64_t cols,
                                                          uint16_t *__restrict__ dst, int64_t ld)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TQ];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int r = threadIdx.x >> 2, cv = (threadIdx.x & 3) * 16;   // one 16-byte vector of a source row per thread
    __attribute__((aligned(16))) int8_t q[16];
    const bool row_ok = r0 + r < rows;
    if (row_ok && c0 + cv + 16 <= cols && (cols & 15) == 0) {
        *reinterpret_cast<uint4 *>(q) = *reinterpret_cast<const uint4 *>(src + (r0 + r) * cols + c0 + cv);
    } else {
        for (int e = 0; e < 16; ++e) q[e] = (row_ok && c0 + cv + e < cols) ? src[(r0 + r) * cols + c0 + cv + e] : (int8_t)0;
    }
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
        const uint32_t lo = __float_as_uint((float)q[e]) >> 16, hi = __float_as_uint((float)q[e + 1]) & 0xffff0000u;
        *reinterpret_cast<uint32_t *>(&tile[r * TQ + cv + e]) = lo | hi;   // |q| <= 128: exact in bf16
    }
    __syncthreads();
    write_tile_transposed(tile, dst, ld, c0, r0, cols, ld);
}

// dY [tokens, d_out] bf16 -> (dY[t,:] / s_x[t])^T as bf16 [d_out, ld], zeros for t in [tokens, ld)
__global__ void __launch_bounds__(256) transpose_scale_dy_kernel(const uint16_t *__restrict__ dY, const float *__restrict__ sx,
                                                                int64_t tokens, int64_t d_out, uint16_t *__restrict__ dst,
                                                                int64_t ld)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TQ];
    const int64_t t0 = (int64_t)blockIdx.y * 64, o0 = (int64_t)blockIdx.x * 64;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int v = threadIdx.x + 256 * h;
        const int t = v >> 3, ov = (v & 7) * 8;
        __attribute__((aligned(16))) uint16_t q[8];
        const bool row_ok = t0 + t < tokens;
        if (row_ok && o0 + ov + 8 <= d_out && (d_out & 7) == 0) {
            *reinterpret_cast<uint4 *>(q) = *reinterpret_cast<const uint4 *>(dY + (t0 + t) * d_out + o0 + ov);
        } else {
            for (int e = 0; e < 8; ++e) q[e] = (row_ok && o0 + ov + e < d_out) ? dY[(t0 + t) * d_out + o0 + ov + e] : (uint16_t)0;
        }
        const float s = row_ok ? sx[t0 + t] : 1.0f;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const uint32_t lo = f32_to_bf16(__fdiv_rn(__uint_as_float((uint32_t)q[e] << 16), s));
            const uint32_t hi = f32_to_bf16(__fdiv_rn(__uint_as_float((uint32_t)q[e + 1] << 16), s));
            *reinterpret_cast<uint32_t *>(&tile[t * TQ + ov + e]) = lo | (hi << 16);
        }
    }
    __syncthreads();
    write_tile_transposed(tile, dst, ld, o0, t0, d_out, ld);
}

// ---- bf16 "NT" GEMM ---------------------------------------------------------------------------------
// C[m, n] (+)= alpha * sum_k Q[m, k] * P[n, k];  P is [N, ldp], Q is [M, ldq], both bf16 with k
// contiguous; C is bf16 [M, ldc].  P supplies the rows of the MFMA result so that a lane ends up
// with four consecutive n of one C row (one 8-byte store).
// Block: 256 threads = 2 x 2 wavefronts, block tile 256 (n) x 128 (m), wave tile 128 (n) x 64 (m),
// 64 k per iteration through a single LDS buffer with register prefetch of the next tile.
constexpr int GB_N = 256, GB_M = 128, GB_K = 64;
constexpr int GROW = GB_K * 2 + 16;   // LDS row pitch in bytes (128 data + 16 pad)

struct GemmBf16Args {
    const uint16_t *P;
    const uint16_t *Q;
    uint16_t *C;
    const float *alpha;   // device scalar or null (= 1)
    int64_t ldp, ldq, ldc;
    int N, M, K;
    int accumulate;
    int tiles_n, tiles_m;
    const uint32_t *mask;   // null, or one bit per element of C (rows of mask_wpr words): zero bits block the new term
    int mask_wpr;
};

// Tile order.  Blocks go to the eight XCDs round-robin and every XCD has its own L2, so XCD x takes
// a contiguous eighth of an order in which consecutive tiles form compact rectangles: super-tiles of
// 8 x 8 tiles (3072 operand rows for 64 tiles instead of up to all of them), bands of eight tile rows,
// super-tiles left to right in a band, the row index fastest inside a super-tile.  With plain row-major
// order the L2s missed on two thirds of their requests.  bid = block index inside the product's
// range; returns false for the blocks that pad the range to a multiple of eight.
__device__ __forceinline__ bool bf16_tile_of_block(const GemmBf16Args &g, int bid, int &tn, int &tm)
{
    const int nb = g.tiles_n * g.tiles_m;
    const int per = (nb + 7) >> 3;
    const int id = (bid & 7) * per + (bid >> 3);
    if ((bid >> 3) >= per || id >= nb) return false;
    const int band_tiles = 8 * g.tiles_n;
    const int nbands = (g.tiles_m + 7) >> 3;
    int band = id / band_tiles;
    band = band < nbands - 1 ? band : nbands - 1;
    const int h = band == nbands - 1 ? g.tiles_m - 8 * band : 8;      // tile rows of this band
    const int rem = id - band * band_tiles;
    const int ncols = (g.tiles_n + 7) >> 3;
    int col = rem / (8 * h);
    col = col < ncols - 1 ? col : ncols - 1;
    const int rem2 = rem - col * 8 * h;
    tn = 8 * col + rem2 / h;
    tm = 8 * band + rem2 % h;
    return true;
}

// Result of a wavefront: 4 x 2 tiles of 32 x 32 at rows (of C) mw + 32 b + .., columns nw + 32 a + ..;
// tile (a, b): lane holds m = column r, n = rows 8q + 4c + i: four consecutive n of one C row per store.
template <int TBM>
__device__ __forceinline__ void bf16_wave_epilogue(const GemmBf16Args &g, const v16f (&acc)[4][TBM], int nw, int mw, int lane)
{
    const int r = lane & 31, c = lane >> 5;
    const float alpha = g.alpha ? *g.alpha : 1.0f;
#pragma unroll
    for (int b = 0; b < TBM; ++b) {
        const int m = mw + 32 * b + r;
        if (m >= g.M) continue;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = nw + 32 * a + 8 * q + 4 * c;
                uint16_t *dst = g.C + (int64_t)m * g.ldc + n;
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = acc[a][b][4 * q + i] * alpha;
                if (g.mask && n < g.N) {   // n is a multiple of 4: its four mask bits sit in one word
                    const uint32_t mb = g.mask[(int64_t)m * g.mask_wpr + (n >> 5)] >> (n & 31);
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (mb >> i) & 1u ? v[i] : 0.0f;
                }
                if (n + 4 <= g.N && (g.ldc & 3) == 0) {
                    if (g.accumulate) {
                        const uint2 old = *reinterpret_cast<const uint2 *>(dst);
                        v[0] += __uint_as_float(old.x << 16);
                        v[1] += __uint_as_float(old.x & 0xffff0000u);
                        v[2] += __uint_as_float(old.y << 16);
                        v[3] += __uint_as_float(old.y & 0xffff0000u);
                    }
                    uint2 out;
                    out.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
                    out.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
                    *reinterpret_cast<uint2 *>(dst) = out;
                } else {
                    for (int i = 0; i < 4; ++i) {
                        if (n + i < g.N) {
                            float x = v[i];
                            if (g.accumulate) x += __uint_as_float((uint32_t)dst[i] << 16);
                            dst[i] = (uint16_t)f32_to_bf16(x);
                        }
                    }
                }
            }
        }
    }
}

// Up to two products share one launch (dW and dX of a layer): the block index space is the
// concatenation of their tiles, the product with the longer contraction first, so that the short
// tiles of the second fill the multiprocessors the first leaves idle in its last round (dW of a
// 2560 x 2560 layer is 200 tiles for 512 block slots).  Each range starts at a multiple of 8 (the
// blocks in between exit at once), which keeps block index mod 8 = XCD for the tile order below.
// one launch covers the tiles of up to GB_GROUP_MAX products: product p owns the blocks [block0[p], block0[p + 1])
constexpr int GB_GROUP_MAX = 8;
struct GemmBf16Group {
    GemmBf16Args g[GB_GROUP_MAX];
    int block0[GB_GROUP_MAX + 1];
    int count;
};

__device__ __forceinline__ int bf16_product_of_block(const GemmBf16Group &grp)
{
    int prob = 0;
    while (prob + 1 < grp.count && (int)blockIdx.x >= grp.block0[prob + 1]) ++prob;
    return prob;
}

__global__ void __launch_bounds__(256, 2) gemm_bf16_nt_kernel(GemmBf16Group grp)
{
    __shared__ __attribute__((aligned(16))) uint8_t ldsP[GB_N * GROW];
    __shared__ __attribute__((aligned(16))) uint8_t ldsQ[GB_M * GROW];
    const int prob = bf16_product_of_block(grp);
    const GemmBf16Args &g = grp.g[prob];
    int tn, tm;
    if (!bf16_tile_of_block(g, (int)blockIdx.x - grp.block0[prob], tn, tm)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;
    const int r = lane & 31, c = lane >> 5;
    const int n0 = tn * GB_N, m0 = tm * GB_M;

    // copy roles: 8 threads per row (16 bytes each), 32 rows per pass.  Addresses are a uniform tile base
    // (scalar registers, advanced by 128 bytes per k step) plus a 32-bit byte offset per thread and pass,
    // rows past the end clamped to the last one: the loads of the loop need no vector arithmetic.
    const int cp_row = tid >> 3, cp_col = (tid & 7) * 8;   // column in elements
    const char *pbase = reinterpret_cast<const char *>(g.P + (int64_t)n0 * g.ldp);
    const char *qbase = reinterpret_cast<const char *>(g.Q + (int64_t)m0 * g.ldq);
    uint32_t poff[8], qoff[4];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int n = n0 + cp_row + 32 * p;
        n = (n < g.N ? n : g.N - 1) - n0;
        poff[p] = (uint32_t)(((int64_t)n * g.ldp + cp_col) * 2);
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int m = m0 + cp_row + 32 * p;
        m = (m < g.M ? m : g.M - 1) - m0;
        qoff[p] = (uint32_t)(((int64_t)m * g.ldq + cp_col) * 2);
    }

    v16f acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // k steps that lie entirely inside K load unconditionally (straight-line loop body); a ragged last
    // step (K % 8 == 0: a 16-byte vector is entirely inside or outside) masks its loads
    const int nk_full = g.K / GB_K;
    const int nk = (g.K + GB_K - 1) / GB_K;
    uint4 preg[8], qreg[4];
    auto load_full = [&](int kt) {
        const char *pb = pbase + (int64_t)kt * (GB_K * 2), *qb = qbase + (int64_t)kt * (GB_K * 2);
#pragma unroll
        for (int p = 0; p < 8; ++p) preg[p] = *reinterpret_cast<const uint4 *>(pb + poff[p]);
#pragma unroll
        for (int p = 0; p < 4; ++p) qreg[p] = *reinterpret_cast<const uint4 *>(qb + qoff[p]);
    };
    auto load_ragged = [&](int kt) {
        const char *pb = pbase + (int64_t)kt * (GB_K * 2), *qb = qbase + (int64_t)kt * (GB_K * 2);
        const bool ok = kt * GB_K + cp_col + 8 <= g.K;
#pragma unroll
        for (int p = 0; p < 8; ++p) preg[p] = ok ? *reinterpret_cast<const uint4 *>(pb + poff[p]) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int p = 0; p < 4; ++p) qreg[p] = ok ? *reinterpret_cast<const uint4 *>(qb + qoff[p]) : make_uint4(0, 0, 0, 0);
    };
    auto store_tile_lds = [&]() {
#pragma unroll
        for (int p = 0; p < 8; ++p) *reinterpret_cast<uint4 *>(&ldsP[(cp_row + 32 * p) * GROW + cp_col * 2]) = preg[p];
#pragma unroll
        for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4 *>(&ldsQ[(cp_row + 32 * p) * GROW + cp_col * 2]) = qreg[p];
    };
    auto multiply_tile = [&]() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // lane (r, c) supplies k = 16u + 8c + 0..7 of the tile for both operands
            v8bf pf[4], qf[2];
#pragma unroll
            for (int a = 0; a < 4; ++a)
                pf[a] = *reinterpret_cast<const v8bf *>(&ldsP[(wn * 128 + 32 * a + r) * GROW + 32 * u + 16 * c]);
#pragma unroll
            for (int b = 0; b < 2; ++b)
                qf[b] = *reinterpret_cast<const v8bf *>(&ldsQ[(wm * 64 + 32 * b + r) * GROW + 32 * u + 16 * c]);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[a], qf[b], acc[a][b], 0, 0, 0);
        }
    };

    if (nk_full > 0) load_full(0); else load_ragged(0);
    store_tile_lds();
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < nk_full; ++kt) {   // the next step is a full one
        load_full(kt + 1);
        multiply_tile();
        __syncthreads();
        store_tile_lds();
        __syncthreads();
    }
    if (kt + 1 < nk) {                 // one ragged step follows
        load_ragged(kt + 1);
        multiply_tile();
        __syncthreads();
        store_tile_lds();
        __syncthreads();
    }
    multiply_tile();                   // last step: nothing left to fetch

    bf16_wave_epilogue<2>(g, acc, n0 + wn * 128, m0 + wm * 64, lane);
}

// ---- the same product with the operands streamed into LDS by the DMA path --------------------------
// Timing-only ablations of the kernel above (2 x 2 wavefronts, register prefetch, one LDS buffer): LDS
// reads + matrix instructions alone run at 86 % of what the board sustains; the global-load ->
// register -> LDS-store path costs the rest (the scheduler sinks the loads to the end of a k step to
// save registers, and forcing them early costs the LDS read-ahead instead).  Here no operand touches a
// register on its way in: block tile 256 (n) x 256 (m), 512 threads = 2 x 4 wavefronts of 128 x 64 (one
// block per multiprocessor, two wavefronts per SIMD), two LDS stages of 64 k (128-byte rows, 64 KB per
// stage), each wavefront issues eight LDS-DMA loads for the next stage before it multiplies the
// current one; one barrier per k step.  The 16-byte column of a row is XOR-swizzled with (row >> 1) & 7 (on
// the global side of the DMA, which deposits lane l at base + 16 l), so the 32 rows x 2 columns of an
// operand read spread over all banks.  Needs K % 64 == 0 (no partial rows in a stage).
// The matrix pipe still waits for the operands about a third of the time.  Measured on the backward of one 6912 x 2560
// layer at 16384 tokens (1.05 ms in this kernel): without the DMA requests (LDS reads, matrix instructions and
// barriers only) 0.75 ms, 80 % of what the board sustains; with every block fetching the same 512 operand rows (all
// requests hit L2) 0.95 ms; the L2 miss rate of the real launch is 19.5 %, what 32 multiprocessors sharing a 4 x 8
// rectangle of tiles must miss ((4 + 8) / 64).  So it is the deposit path into LDS, not L2 or HBM, that costs most: at
// 64 bytes per clock the 64 KB of a stage take half of the stage's matrix time, and the fragment reads (192 KB at 256
// bytes per clock) take most of the other half.  Tried and measured slower: a ring of four stages of 32 k with eight
// wavefronts (5.96 against 5.43 ms for the backward of the block); one wavefront per SIMD with 128 x 128 wave tiles,
// four stages of 32 k and counted waits (a third fewer LDS reads, no conflicts: 1.13 ms against 1.05); warming L2 two
// steps ahead with one extra line-touching DMA load per wavefront and step (5.99 ms: it doubles the L2 requests).
constexpr int GD_N = 256, GD_M = 256, GD_K = 64;
constexpr int GD_STAGE = (GD_N + GD_M) * GD_K * 2;   // 64 KB
constexpr int GD_LDS = 2 * GD_STAGE;

__global__ void __launch_bounds__(512) gemm_bf16_dma_kernel(GemmBf16Group grp)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t dlds[];
    const int prob = bf16_product_of_block(grp);
    const GemmBf16Args &g = grp.g[prob];
    int tn, tm;
    if (!bf16_tile_of_block(g, (int)blockIdx.x - grp.block0[prob], tn, tm)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1, wm = wave >> 1;
    const int r = lane & 31, c = lane >> 5;
    const int n0 = tn * GD_N, m0 = tm * GD_M;
    const uint32_t lds0 = lds_address(dlds);

    // DMA roles: one instruction fills 8 rows x 128 bytes (lane l: row l / 8, slot l % 8 holding global
    // column slot ^ ((row >> 1) & 7)); wavefront w fills rows 32 w .. 32 w + 31 of P and of Q: 4 + 4 instructions
    const char *pbase = reinterpret_cast<const char *>(g.P + (int64_t)n0 * g.ldp);
    const char *qbase = reinterpret_cast<const char *>(g.Q + (int64_t)m0 * g.ldq);
    uint32_t poff[4], qoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 32 * wave + 8 * i + (lane >> 3);
        const int col = (lane & 7) ^ ((row >> 1) & 7);
        int n = n0 + row;
        n = (n < g.N ? n : g.N - 1) - n0;
        poff[i] = (uint32_t)(((int64_t)n * g.ldp + col * 8) * 2);
        int m = m0 + row;
        m = (m < g.M ? m : g.M - 1) - m0;
        qoff[i] = (uint32_t)(((int64_t)m * g.ldq + col * 8) * 2);
    }
    auto dma_stage = [&](int kt, int stage) {
        const char *pb = pbase + (int64_t)kt * (GD_K * 2), *qb = qbase + (int64_t)kt * (GD_K * 2);
        const uint32_t dp = lds0 + stage * GD_STAGE + wave * 4096, dq = dp + GD_N * GD_K * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_dma16(pb, poff[i], dp + i * 1024);
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_dma16(qb, qoff[i], dq + i * 1024);
    };
    // LDS read addresses: row * 128 + 16 * ((2u + c) ^ ((row >> 1) & 7)); (row >> 1) & 7 = (r >> 1) & 7 for every
    // tile of the wavefront, so one lane address per u and operand, tiles and stages are immediate offsets.  (With
    // row & 7 as the swizzle, rows r and r + 8 of a 16-lane group met in the same banks: four conflict cycles per read.)
    uint32_t pa[4], qa[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int slot = (2 * u + c) ^ ((r >> 1) & 7);
        pa[u] = lds0 + (wn * 128 + r) * 128 + 16 * slot;
        qa[u] = lds0 + GD_N * GD_K * 2 + (wm * 64 + r) * 128 + 16 * slot;
    }
    typedef __attribute__((address_space(3))) const v8bf *lds_v8bf;

    v16f acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    auto multiply_stage = [&](const int stage) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v8bf pf[4], qf[2];
#pragma unroll
            for (int a = 0; a < 4; ++a) pf[a] = *(lds_v8bf)(uintptr_t)(pa[u] + stage * GD_STAGE + a * 32 * 128);
#pragma unroll
            for (int b = 0; b < 2; ++b) qf[b] = *(lds_v8bf)(uintptr_t)(qa[u] + stage * GD_STAGE + b * 32 * 128);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[a], qf[b], acc[a][b], 0, 0, 0);
        }
    };
    // step kt reads stage kt & 1 while the DMA fills the other one with step kt + 1 (past the end the last
    // step is fetched again into a stage nobody reads any more); the barrier at the end of a step publishes
    // the landed stage and frees the one just read.  Stage numbers are literals: two steps per loop trip.
    const int nk = g.K / GD_K;
    auto step = [&](const int kt, const int stage) {
        dma_stage(kt + 1 < nk ? kt + 1 : nk - 1, stage ^ 1);
        multiply_stage(stage);
        SBN_WAIT_VMCNT(0);
        __syncthreads();
    };
    dma_stage(0, 0);
    SBN_WAIT_VMCNT(0);
    __syncthreads();
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
        step(kt, 0);
        step(kt + 1, 1);
    }
    if (kt < nk) step(kt, 0);

    bf16_wave_epilogue<2>(g, acc, n0 + wn * 128, m0 + wm * 64, lane);
}

GemmBf16Args make_bf16_args(const uint16_t *P, int64_t ldp, int N, const uint16_t *Q, int64_t ldq, int M, int K, uint16_t *C,
                            int64_t ldc, const float *alpha, int accumulate)
{
    GemmBf16Args g;
    g.P = P; g.Q = Q; g.C = C; g.alpha = alpha; g.ldp = ldp; g.ldq = ldq; g.ldc = ldc;
    g.N = N; g.M = M; g.K = K; g.accumulate = accumulate;
    g.tiles_n = (int)ceil_div(N, GB_N);   // for the register-prefetch kernel; the launcher recounts for the DMA kernel
    g.tiles_m = (int)ceil_div(M, GB_M);
    g.mask = nullptr;
    g.mask_wpr = 0;
    return g;
}

// one launch for one or two products; the one with the longer contraction goes first
// Products of one launch, longest contraction first: the long tiles start at once and the short ones fill
// the multiprocessors they leave idle.
sbn_status launch_gemm_bf16(int count, const GemmBf16Args *args, hipStream_t stream)
{
    for (int first = 0; first < count; first += GB_GROUP_MAX) {
        GemmBf16Group grp;
        grp.count = count - first < GB_GROUP_MAX ? count - first : GB_GROUP_MAX;
        int order[GB_GROUP_MAX];
        for (int i = 0; i < grp.count; ++i) order[i] = first + i;
        std::stable_sort(order, order + grp.count, [&](int a, int b) { return args[a].K > args[b].K; });
        // the DMA kernel takes whole 64-k stages and 16-byte aligned rows; anything else takes the register-prefetch kernel
        bool dma = true;
        for (int i = 0; i < grp.count; ++i) {
            const GemmBf16Args &a = args[order[i]];
            dma = dma && a.K % GD_K == 0 && a.ldp % 8 == 0 && a.ldq % 8 == 0 && aligned(a.P, 16) && aligned(a.Q, 16);
        }
        int blocks = 0;
        for (int i = 0; i < grp.count; ++i) {
            grp.g[i] = args[order[i]];
            if (dma) {
                grp.g[i].tiles_n = (int)ceil_div(grp.g[i].N, GD_N);
                grp.g[i].tiles_m = (int)ceil_div(grp.g[i].M, GD_M);
            }
            grp.block0[i] = blocks;
            blocks += (grp.g[i].tiles_n * grp.g[i].tiles_m + 7) / 8 * 8;   // eight equal shares, one per XCD
        }
        for (int i = grp.count; i <= GB_GROUP_MAX; ++i) grp.block0[i] = blocks;
        for (int i = grp.count; i < GB_GROUP_MAX; ++i) grp.g[i] = grp.g[0];
        if (dma) {
            static thread_local bool raised = false;
            if (!raised) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bf16_dma_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, GD_LDS);
                if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute"); return SBN_EHIP; }
                raised = true;
            }
            hipLaunchKernelGGL(gemm_bf16_dma_kernel, dim3(blocks), dim3(512), GD_LDS, stream, grp);
            sbn_status st = check_launch("gemm_bf16_dma_kernel");
            if (st != SBN_OK) return st;
        } else {
            hipLaunchKernelGGL(gemm_bf16_nt_kernel, dim3(blocks), dim3(256), 0, stream, grp);
            sbn_status st = check_launch("gemm_bf16_nt_kernel");
            if (st != SBN_OK) return st;
        }
    }
    return SBN_OK;
}

inline int64_t pad8(int64_t x) { return (x + 7) / 8 * 8; }

}  // namespace

size_t backward_workspace_bytes(int64_t tokens, int64_t d_out, int64_t d_in)
{
    // W_eff^T bf16 [d_in, pad8(d_out)] + int8 W_eff (generic patterns) + (dY/s_x)^T bf16 [d_out, pad8(tokens)]
    // + xq^T bf16 [d_in, pad8(tokens)]
    // + the mask bit plane of the gradient-masked variant
    return align_up((size_t)d_in * pad8(d_out) * 2, 256) + align_up((size_t)d_out * d_in, 256) +
           align_up((size_t)d_out * pad8(tokens) * 2, 256) + align_up((size_t)d_in * pad8(tokens) * 2, 256) +
           align_up((size_t)d_out * ((d_in + 31) / 32) * 4, 256);
}

// Backward products of `count` layers in one pass: the layout kernels of every layer, then ONE matrix-multiply
// launch (per GB_GROUP_MAX products) over all dW and dX tiles.  Layers that share their quantized input (Q/K/V,
// up/gate) share its transpose.
sbn_status launch_backward_grouped(int count, const BackwardItem *items, const Pattern &pat, int flags, hipStream_t stream)
{
    const int accumulate = (flags & SBN_BWD_ACCUMULATE) != 0;
    std::vector<GemmBf16Args> products;
    std::vector<const uint16_t *> xt_of(count, nullptr);
    products.reserve(2 * count);
    sbn_status st;
    for (int i = 0; i < count; ++i) {
        const BackwardItem &it = items[i];
        const int64_t tokens = it.tokens, d_in = it.d_in, d_out = it.d_out;
        uint8_t *ws = static_cast<uint8_t *>(it.workspace);
        uint16_t *wt = reinterpret_cast<uint16_t *>(ws);
        ws += align_up((size_t)d_in * pad8(d_out) * 2, 256);
        int8_t *w8 = reinterpret_cast<int8_t *>(ws);
        ws += align_up((size_t)d_out * d_in, 256);
        uint16_t *dyt = reinterpret_cast<uint16_t *>(ws);
        ws += align_up((size_t)d_out * pad8(tokens) * 2, 256);
        uint16_t *xt = reinterpret_cast<uint16_t *>(ws);
        ws += align_up((size_t)d_in * pad8(tokens) * 2, 256);
        uint32_t *mask_bits = reinterpret_cast<uint32_t *>(ws);
        const uint16_t *dy = static_cast<const uint16_t *>(it.dY);

        if (it.dX) {
            const int64_t ldw = pad8(d_out);
            if (pat.N == 2 && pat.M == 4 && d_in % CHUNK == 0) {
                dim3 grid((unsigned)(d_in / CHUNK), (unsigned)ceil_div(d_out, 64));
                hipLaunchKernelGGL(unpack_transpose_kernel, grid, dim3(256), 0, stream, static_cast<const uint8_t *>(it.packed),
                                   (int)d_out, (int)d_in, wt, ldw);
                st = check_launch("unpack_transpose_kernel");
            } else {
                st = launch_expand_groups(it.packed, d_out, d_in, pat, w8, stream);
                if (st != SBN_OK) return st;
                dim3 grid((unsigned)ceil_div(d_in, 64), (unsigned)ceil_div(d_out, 64));
                hipLaunchKernelGGL(transpose_i8_kernel, grid, dim3(256), 0, stream, w8, d_out, d_in, wt, ldw);
                st = check_launch("transpose_i8_kernel");
            }
            if (st != SBN_OK) return st;
            // dX[t, k] = gamma * sum_o dY[t, o] * W_eff^T[k, o]
            products.push_back(make_bf16_args(wt, ldw, (int)d_in, dy, d_out, (int)tokens, (int)d_out, static_cast<uint16_t *>(it.dX),
                                              d_in, it.gamma, 0));
        }
        if (it.dW) {
            const int64_t ldt = pad8(tokens);
            {
                dim3 grid((unsigned)ceil_div(d_out, 64), (unsigned)ceil_div(tokens, 64));
                hipLaunchKernelGGL(transpose_scale_dy_kernel, grid, dim3(256), 0, stream, dy, it.sx, tokens, d_out, dyt, ldt);
                st = check_launch("transpose_scale_dy_kernel");
                if (st != SBN_OK) return st;
            }
            const uint16_t *xts = nullptr;   // an earlier layer of the call already transposed the same activations
            for (int j = 0; j < i && !xts; ++j)
                if (xt_of[j] && items[j].xq == it.xq && items[j].tokens == tokens && items[j].d_in == d_in) xts = xt_of[j];
            if (!xts) {
                dim3 grid((unsigned)ceil_div(d_in, 64), (unsigned)ceil_div(tokens, 64));
                hipLaunchKernelGGL(transpose_i8_kernel, grid, dim3(256), 0, stream, it.xq, tokens, d_in, xt, ldt);
                st = check_launch("transpose_i8_kernel");
                if (st != SBN_OK) return st;
                xts = xt;
            }
            xt_of[i] = xts;
            // dW[o, k] = sum_t (dY/s_x)^T[o, t] * xq^T[k, t]; both operands are zero for t in [tokens, ldt)
            GemmBf16Args a = make_bf16_args(xts, ldt, (int)d_in, dyt, ldt, (int)d_out, (int)ldt, static_cast<uint16_t *>(it.dW), d_in,
                                            nullptr, accumulate);
            if (flags & SBN_BWD_MASK_DW) {
                // ablation variant: only the weights of the current mask receive the new gradient term
                st = launch_mask_bitplane(it.packed, d_out, d_in, pat, mask_bits, stream);
                if (st != SBN_OK) return st;
                a.mask = mask_bits;
                a.mask_wpr = (int)((d_in + 31) / 32);
            }
            products.push_back(a);
        }
    }
    // all products are independent of each other (dX reads W_eff^T and dY, dW reads the two transposes)
    return launch_gemm_bf16((int)products.size(), products.data(), stream);
}

sbn_status launch_backward(const void *dY, int64_t tokens, int64_t d_in, int64_t d_out, const Pattern &pat,
                           const void *packed, const float *gamma, const int8_t *xq, const float *sx, void *dX,
                           void *dW, int flags, void *workspace, size_t ws_bytes, hipStream_t stream)
{
    (void)ws_bytes;
    BackwardItem it{dY, tokens, d_in, d_out, packed, gamma, xq, sx, dX, dW, workspace};
    return launch_backward_grouped(1, &it, pat, flags, stream);
}

}  // namespace sbn
