// Prefill / training GEMM of the sparse ternary linear layer on CDNA4 int8 matrix cores (2:4).
//   acc[t, o] = sum_k W_eff[o, k] * xq[t, k],   Y = acc * gamma / s_x[t] (+ bias)
// Section 2.2 (forward-pass equation).  Two paths:
//   sparse  v_smfmac_i32_32x32x64_i8: the packed weights ARE the compressed A operand (code word ->
//           16 int8 values, index word -> the instruction's index register), tokens are B;
//   dense   v_mfma_i32_32x32x32_i8 on W_eff expanded to int8 with explicit zeros: the in-run
//           comparison a dense ternary layer would run.
#include "sbn_internal.hpp"
#include "sbn_mfma.hpp"

namespace sbn {

namespace {

constexpr int BO = 256;        // output rows (of W) per block
constexpr int BT = 128;        // tokens per block
constexpr int KSTEP = 128;     // input features per main-loop iteration = one packed chunk
constexpr int LDS_ROW = KSTEP + 16;   // padded row of the token tile: 16-byte reads of 32 rows hit distinct banks

struct GemmArgs {
    const int8_t *xq;
    const float *sx;
    const uint8_t *packed;   // sparse path
    const int8_t *w_dense;   // dense path
    const float *gamma;
    const float *bias;
    float *Y;
    int32_t *acc_out;
    int tokens, d_in, d_out;
    int tiles_o, tiles_t;
};

// blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles (row tile
// fastest) so the blocks sharing an L2 reuse the same token tile
__device__ __forceinline__ void tile_of_block(const GemmArgs &g, int &to, int &tt)
{
    const int nb = g.tiles_o * g.tiles_t;
    int id = blockIdx.x;
    if ((nb & 7) == 0) id = (id & 7) * (nb >> 3) + (id >> 3);
    to = id % g.tiles_o;
    tt = id / g.tiles_o;
}

__device__ __forceinline__ void store_tile(const GemmArgs &g, const v16i &acc, int o_base, int t, float scale)
{
    // lane holds token t and rows o_base + 8*(i/4) + i%4  (o_base already includes 4*(lane/32))
    if (t >= g.tokens) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int o = o_base + 8 * q;
        if (o + 3 < g.d_out && (g.d_out & 3) == 0) {
            float4 y;
            y.x = (float)acc[4 * q + 0] * scale;
            y.y = (float)acc[4 * q + 1] * scale;
            y.z = (float)acc[4 * q + 2] * scale;
            y.w = (float)acc[4 * q + 3] * scale;
            if (g.bias) {
                const float4 b = *reinterpret_cast<const float4 *>(g.bias + o);
                y.x += b.x; y.y += b.y; y.z += b.z; y.w += b.w;
            }
            *reinterpret_cast<float4 *>(g.Y + (int64_t)t * g.d_out + o) = y;
            if (g.acc_out)
                *reinterpret_cast<int4 *>(g.acc_out + (int64_t)t * g.d_out + o) =
                    make_int4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (o + i < g.d_out) {
                    float y = (float)acc[4 * q + i] * scale;
                    if (g.bias) y += g.bias[o + i];
                    g.Y[(int64_t)t * g.d_out + o + i] = y;
                    if (g.acc_out) g.acc_out[(int64_t)t * g.d_out + o + i] = acc[4 * q + i];
                }
            }
        }
    }
}

// ---- sparse path --------------------------------------------------------------------------------
// 4 wavefronts as 2 (rows) x 2 (tokens); each owns 128 rows x 64 tokens = 4 x 2 tiles of 32x32.
// Per iteration (one 128-weight chunk) a lane (row r = lane % 32, half c = lane / 32) loads, for
// each of its four row tiles, index words 2c, 2c+1 and code words 2c, 2c+1 of its row's chunk
// (two 8-byte loads) straight from global memory; sub-step u = 0, 1 uses word 2c + u, i.e. the
// lane supplies weights [64c + 32u, +32) of the chunk.  The token tile goes through LDS.
__global__ void __launch_bounds__(256, 2) gemm_smfmac_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) int8_t lds[2][BT * LDS_ROW];
    int to, tt;
    tile_of_block(g, to, tt);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wo = wave & 1, wt = wave >> 1;
    const int r = lane & 31, c = lane >> 5;
    const int K = g.d_in, nchunks = K / KSTEP;
    const int o0 = to * BO + wo * 128, t0 = tt * BT;

    // global -> LDS copy of the token tile: thread i moves 16 bytes of row i/8 (+32 per pass)
    const int cp_row = tid >> 3, cp_col = (tid & 7) * 16;
    const int8_t *xsrc[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int t = t0 + cp_row + 32 * p;
        t = t < g.tokens ? t : g.tokens - 1;
        xsrc[p] = g.xq + (int64_t)t * K + cp_col;
    }
    // packed rows of the four row tiles
    const uint8_t *wsrc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        int o = o0 + 32 * a + r;
        o = o < g.d_out ? o : g.d_out - 1;
        wsrc[a] = g.packed + (int64_t)o * nchunks * 32 + 8 * c;
    }

    v16i acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0;

    uint4 xreg[4];
    uint2 ireg[4], creg[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) xreg[p] = *reinterpret_cast<const uint4 *>(xsrc[p]);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        ireg[a] = *reinterpret_cast<const uint2 *>(wsrc[a]);
        creg[a] = *reinterpret_cast<const uint2 *>(wsrc[a] + 16);
    }
#pragma unroll
    for (int p = 0; p < 4; ++p)
        *reinterpret_cast<uint4 *>(&lds[0][(cp_row + 32 * p) * LDS_ROW + cp_col]) = xreg[p];
    __syncthreads();

    for (int kc = 0; kc < nchunks; ++kc) {
        const int cur = kc & 1;
        uint2 icur[4], ccur[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) { icur[a] = ireg[a]; ccur[a] = creg[a]; }
        if (kc + 1 < nchunks) {
#pragma unroll
            for (int p = 0; p < 4; ++p) xreg[p] = *reinterpret_cast<const uint4 *>(xsrc[p] + (kc + 1) * KSTEP);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                ireg[a] = *reinterpret_cast<const uint2 *>(wsrc[a] + (int64_t)(kc + 1) * 32);
                creg[a] = *reinterpret_cast<const uint2 *>(wsrc[a] + (int64_t)(kc + 1) * 32 + 16);
            }
        }
        const int8_t *bt = &lds[cur][0];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            v8i bfrag[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int8_t *p = bt + (wt * 64 + 32 * b + r) * LDS_ROW + 32 * u + 16 * c;
                const uint4 lo = *reinterpret_cast<const uint4 *>(p);
                const uint4 hi = *reinterpret_cast<const uint4 *>(p + 64);
                bfrag[b] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const v4i av = expand_codes(u ? ccur[a].y : ccur[a].x);
                const int iv = (int)(u ? icur[a].y : icur[a].x);
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, bfrag[b], acc[a][b], iv, 0, 0);
            }
        }
        if (kc + 1 < nchunks) {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                *reinterpret_cast<uint4 *>(&lds[cur ^ 1][(cp_row + 32 * p) * LDS_ROW + cp_col]) = xreg[p];
        }
        __syncthreads();
    }

    const float gam = *g.gamma;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int t = t0 + wt * 64 + 32 * b + r;
        const float scale = t < g.tokens ? __fdiv_rn(gam, g.sx[t]) : 0.0f;
#pragma unroll
        for (int a = 0; a < 4; ++a) store_tile(g, acc[a][b], o0 + 32 * a + 4 * c, t, scale);
    }
}

// ---- dense comparison path ---------------------------------------------------------------------
// packed -> int8 W_eff with explicit zeros, one thread per group of four weights
__global__ void __launch_bounds__(256) expand_dense_kernel(const uint8_t *__restrict__ packed, int8_t *__restrict__ w,
                                                          int64_t ngroups)
{
    const int64_t gidx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gidx >= ngroups) return;
    const int64_t chunk = gidx >> 5;
    const int gi = (int)(gidx & 31), word = gi >> 3, t = gi & 7;
    const uint32_t *cw = reinterpret_cast<const uint32_t *>(packed + chunk * 32);
    const uint32_t nib = (cw[word] >> (4 * t)) & 0xfu;
    const uint32_t codes = cw[4 + word];
    uint32_t out = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int v = 2 * t + h;
        const uint32_t code = (codes >> (8 * (v & 3) + 2 * (v >> 2))) & 3u;
        const uint32_t byte = code == 1u ? 0x01u : code == 3u ? 0xffu : 0u;
        const uint32_t pos = h ? (nib >> 2) : (nib & 3u);
        out |= byte << (8 * pos);
    }
    reinterpret_cast<uint32_t *>(w)[gidx] = out;
}

// Same tiling as the sparse kernel; A fragments are 16 dense int8 per lane read from global
// memory (lane (r, c) supplies weights [64c + 16u, +16) of the chunk in sub-step u = 0..3).
__global__ void __launch_bounds__(256, 2) gemm_dense_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) int8_t lds[2][BT * LDS_ROW];
    int to, tt;
    tile_of_block(g, to, tt);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wo = wave & 1, wt = wave >> 1;
    const int r = lane & 31, c = lane >> 5;
    const int K = g.d_in, nchunks = K / KSTEP;
    const int o0 = to * BO + wo * 128, t0 = tt * BT;

    const int cp_row = tid >> 3, cp_col = (tid & 7) * 16;
    const int8_t *xsrc[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int t = t0 + cp_row + 32 * p;
        t = t < g.tokens ? t : g.tokens - 1;
        xsrc[p] = g.xq + (int64_t)t * K + cp_col;
    }
    const int8_t *wsrc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        int o = o0 + 32 * a + r;
        o = o < g.d_out ? o : g.d_out - 1;
        wsrc[a] = g.w_dense + (int64_t)o * K + 64 * c;
    }

    v16i acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0;

    uint4 xreg[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) xreg[p] = *reinterpret_cast<const uint4 *>(xsrc[p]);
#pragma unroll
    for (int p = 0; p < 4; ++p)
        *reinterpret_cast<uint4 *>(&lds[0][(cp_row + 32 * p) * LDS_ROW + cp_col]) = xreg[p];
    __syncthreads();

    for (int kc = 0; kc < nchunks; ++kc) {
        const int cur = kc & 1;
        if (kc + 1 < nchunks) {
#pragma unroll
            for (int p = 0; p < 4; ++p) xreg[p] = *reinterpret_cast<const uint4 *>(xsrc[p] + (kc + 1) * KSTEP);
        }
        const int8_t *bt = &lds[cur][0];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v4i afrag[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const uint4 w = *reinterpret_cast<const uint4 *>(wsrc[a] + (int64_t)kc * KSTEP + 16 * u);
                afrag[a] = v4i{(int)w.x, (int)w.y, (int)w.z, (int)w.w};
            }
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const uint4 x = *reinterpret_cast<const uint4 *>(bt + (wt * 64 + 32 * b + r) * LDS_ROW + 64 * c + 16 * u);
                const v4i bfrag = v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afrag[a], bfrag, acc[a][b], 0, 0, 0);
            }
        }
        if (kc + 1 < nchunks) {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                *reinterpret_cast<uint4 *>(&lds[cur ^ 1][(cp_row + 32 * p) * LDS_ROW + cp_col]) = xreg[p];
        }
        __syncthreads();
    }

    const float gam = *g.gamma;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int t = t0 + wt * 64 + 32 * b + r;
        const float scale = t < g.tokens ? __fdiv_rn(gam, g.sx[t]) : 0.0f;
#pragma unroll
        for (int a = 0; a < 4; ++a) store_tile(g, acc[a][b], o0 + 32 * a + 4 * c, t, scale);
    }
}

GemmArgs make_args(const LinearItem &it)
{
    GemmArgs g;
    g.xq = it.xq; g.sx = it.sx; g.packed = static_cast<const uint8_t *>(it.packed); g.w_dense = nullptr;
    g.gamma = it.gamma; g.bias = it.bias; g.Y = it.Y; g.acc_out = it.acc_out;
    g.tokens = (int)it.tokens; g.d_in = (int)it.d_in; g.d_out = (int)it.d_out;
    g.tiles_o = (int)ceil_div(it.d_out, BO);
    g.tiles_t = (int)ceil_div(it.tokens, BT);
    return g;
}

}  // namespace

sbn_status launch_gemm_smfmac(const LinearItem &it, hipStream_t stream)
{
    GemmArgs g = make_args(it);
    hipLaunchKernelGGL(gemm_smfmac_kernel, dim3(g.tiles_o * g.tiles_t), dim3(256), 0, stream, g);
    return check_launch("gemm_smfmac_kernel");
}

sbn_status launch_gemm_dense(const LinearItem &it, int8_t *w_dense, hipStream_t stream)
{
    const int64_t ngroups = it.d_out * it.d_in / 4;
    hipLaunchKernelGGL(expand_dense_kernel, dim3((unsigned)ceil_div(ngroups, 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t *>(it.packed), w_dense, ngroups);
    sbn_status st = check_launch("expand_dense_kernel");
    if (st != SBN_OK) return st;
    GemmArgs g = make_args(it);
    g.w_dense = w_dense;
    hipLaunchKernelGGL(gemm_dense_kernel, dim3(g.tiles_o * g.tiles_t), dim3(256), 0, stream, g);
    return check_launch("gemm_dense_kernel");
}

}  // namespace sbn
