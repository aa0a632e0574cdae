// Forward of the N:M-sparse ternary linear layer for decode batches of 17 .. 64 tokens (Section 2.2 forward-pass
// equation; Section 3.2 measures decoding at batch sizes from 64 up): few enough tokens that a layer is bound by
// the one pass over its packed weights, too many for the activations of all tokens to stay in LDS.
//
// Persistent blocks of eight wavefronts, one per multiprocessor.  The rows of all problems of a launch are cut into
// strips of 128 * RT rows; a block takes a contiguous run of strips.  Inside a strip wavefront w owns the rows
// 16 * RT * w .. + 16 * RT - 1 and all tokens (TT token tiles of 16: the columns of v_smfmac_i32_16x16x128_i8), and
// the block walks the input dimension in super-steps of 512 weights, all wavefronts together:
//   weights      straight from HBM into registers, a queue of DEPTH super-steps per wavefront (16-byte loads, a
//                wavefront reads 128 contiguous bytes per row and super-step); the queue runs on across strip and
//                problem boundaries, so the stream never drains;
//   activations  the int8 rows of the super-step (16 * TT tokens x 512) in LDS, double-buffered: the tile of the next
//                super-step is fetched (from L2) into registers while the current one is multiplied, written to the
//                other buffer, one barrier per super-step;
//   outputs      at the end of a strip the accumulators are rescaled (gamma / s_x) into an LDS staging area
//                [token][row] and leave as whole token rows of the strip (512 * RT contiguous bytes per store
//                instruction), not as 64-byte pieces per lane group.
// The weights are read in the 2:4 operand form (index word = the instruction's index register) or as dense 2-bit
// codes (DENSE: the packed form of N = M, and of any other pattern after conversion) on v_mfma_i32_16x16x64_i8.
#include <algorithm>

#include "sbn_internal.hpp"
#include "sbn_mfma.hpp"

namespace sbn {

namespace {

struct BatchItem {
    const int8_t *xq;        // int8 [tokens, d_in]
    const float *sx;         // fp32 [tokens]
    const uint8_t *packed;
    const float *gamma;
    float *Y;                // fp32 [tokens, d_out]
    int d_in, d_out, tokens;
    int pad;
};
constexpr int BATCH_MAX = 56;
struct BatchTable {
    BatchItem it[BATCH_MAX];
    int strip0[64 + 1];      // first strip of each problem; entries past the last problem hold the total
    int count;
    int share, share_rem;    // strips per block: the first share_rem blocks take share + 1
    int pad;
};
static_assert(sizeof(BatchTable) <= 4096 && sizeof(BatchTable) % 8 == 0, "the table travels as a kernel argument");

constexpr int BNW = 8;              // wavefronts per block
constexpr int XP = 512 + 16;        // bytes between the token rows of an activation tile in LDS (16 rows 16 bytes apart in the banks)

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
template <typename T> __device__ __forceinline__ T *uni(T *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    typedef T __attribute__((address_space(1))) *global_ptr;   // stays a global (not a flat) access
    return (T *)(global_ptr)(((uint64_t)hi << 32) | lo);
}

// Position in a block's work: strip f (counted over all problems), super-step ks of it, and what follows from them.
struct Cursor {
    int f, ks;
    int item, first;         // problem of strip f and that problem's first strip
    int nchunks, nsuper, d_out, d_in, tokens;
    const uint8_t *packed;
    const int8_t *xq;
};

template <int TT, int RT, int DEPTH, bool DENSE>
__global__ void __launch_bounds__(64 * BNW) gemv_batch_kernel(BatchTable tab_arg)
{
    constexpr int SR = 128 * RT;                 // rows of a strip
    constexpr int XBUF = 16 * TT * XP;           // bytes of one activation tile
    constexpr int YP = SR + 4;                   // floats between the token rows of the output staging area
    constexpr int XVEC = 16 * TT * 32 / (64 * BNW);   // 16-byte vectors of a tile per thread
    static_assert(16 * TT * 32 % (64 * BNW) == 0, "a tile is staged by the whole block in equal parts");
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];   // [2][XBUF] activation tiles, then [16 * TT][YP] floats
    float *ystg = reinterpret_cast<float *>(lds + 2 * XBUF);
    __shared__ __attribute__((aligned(16))) BatchTable tab;
    __shared__ float sx_lds[16 * TT];
    __shared__ float gamma_lds;
    {
        (void)tab_arg;
        const uint2 *src = (const uint2 *)__builtin_amdgcn_kernarg_segment_ptr();   // the table is the only argument
        uint2 *dst = reinterpret_cast<uint2 *>(&tab);
        for (int i = threadIdx.x; i < (int)(sizeof(BatchTable) / 8); i += 64 * BNW) dst[i] = src[i];
        __syncthreads();
    }
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, c4 = lane >> 4;
    const uint32_t ones = vgpr_ones();
    const int share = uni(tab.share), share_rem = uni(tab.share_rem);
    const int b0 = share * (int)blockIdx.x + ((int)blockIdx.x < share_rem ? (int)blockIdx.x : share_rem);
    const int b1 = b0 + share + ((int)blockIdx.x < share_rem ? 1 : 0);
    if (b0 >= b1) return;
    const int bound = tab.strip0[1 + lane];

    auto enter_item = [&](Cursor &c) {   // c.item set: everything that follows from the problem
        const BatchItem &src = tab.it[c.item];
        c.first = uni(tab.strip0[c.item]);
        c.d_in = uni(src.d_in); c.d_out = uni(src.d_out); c.tokens = uni(src.tokens);
        c.packed = uni(src.packed); c.xq = uni(src.xq);
        c.nchunks = c.d_in / CHUNK;
        c.nsuper = (c.nchunks + 3) >> 2;
    };
    // one super-step on; past the block's last super-step the cursor stays where it is (what is fetched there is ignored)
    auto advance = [&](Cursor &c) {
        if (c.ks + 1 < c.nsuper) { ++c.ks; return; }
        if (c.f + 1 >= b1) return;
        ++c.f;
        c.ks = 0;
        if (c.f >= uni(tab.strip0[c.item + 1])) {
            do ++c.item; while (c.f >= uni(tab.strip0[c.item + 1]));
            enter_item(c);
        }
    };
    Cursor ld;   // where the weight queue is filled
    ld.f = b0; ld.ks = 0;
    ld.item = __builtin_popcountll(__ballot(bound <= b0));   // as many problems end at or before the block's first strip
    enter_item(ld);
    Cursor cp = ld;   // where the arithmetic is

    // the lane's packed rows of the strip being loaded
    const uint8_t *prow[RT];
    auto locate = [&](const Cursor &c) {
#pragma unroll
        for (int a = 0; a < RT; ++a) {
            int row = (c.f - c.first) * SR + wave * 16 * RT + 16 * a + r;
            row = row < c.d_out ? row : c.d_out - 1;
            prow[a] = c.packed + (int64_t)row * c.nchunks * 32;
        }
    };
    locate(ld);
    uint4 qi[DEPTH][RT], qc[DEPTH][RT];
    auto issue = [&](uint4(&ib)[RT], uint4(&cb)[RT]) {
        int ch = 4 * ld.ks + c4;
        ch = ch < ld.nchunks ? ch : ld.nchunks - 1;
#pragma unroll
        for (int a = 0; a < RT; ++a) {
            const uint8_t *p = prow[a] + (uint32_t)ch * 32;
            ib[a] = *reinterpret_cast<const uint4 *>(p);
            cb[a] = *reinterpret_cast<const uint4 *>(p + 16);
        }
        const int f_before = ld.f;
        advance(ld);
        if (ld.f != f_before) locate(ld);
    };
    // the activation tile of a position: thread v of the block fetches the 16-byte vectors v, v + 512, ... of
    // [16 * TT tokens][512 bytes]; rows past the problem's tokens and columns past its input dimension are zero
    auto fetch_tile = [&](const Cursor &c, uint4(&xv)[XVEC]) {
#pragma unroll
        for (int i = 0; i < XVEC; ++i) {
            const int v = (int)threadIdx.x + 64 * BNW * i, row = v >> 5, col = 512 * c.ks + 16 * (v & 31);
            const bool ok = row < c.tokens && col < c.d_in;
            const uint4 q = *reinterpret_cast<const uint4 *>(c.xq + (ok ? (int64_t)row * c.d_in + col : 0));
            xv[i] = ok ? q : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tile = [&](int8_t *buf, const uint4(&xv)[XVEC]) {
#pragma unroll
        for (int i = 0; i < XVEC; ++i) {
            const int v = (int)threadIdx.x + 64 * BNW * i;
            *reinterpret_cast<uint4 *>(buf + (v >> 5) * XP + 16 * (v & 31)) = xv[i];
        }
    };
    // s_x of the problem's tokens and its gamma, for the epilogues of its strips: through LDS, so that an epilogue
    // issues no load from memory (loads complete in order: waiting for one would drain the weight queue)
    auto stage_scales = [&](const Cursor &c) {
        if ((int)threadIdx.x < 16 * TT) {
            const float *sx = uni(tab.it[c.item].sx);
            sx_lds[threadIdx.x] = (int)threadIdx.x < c.tokens ? sx[threadIdx.x] : 1.0f;
        } else if ((int)threadIdx.x == 16 * TT) {
            gamma_lds = *uni(tab.it[c.item].gamma);
        }
    };

    // Activation tiles are requested DEPTH super-steps ahead as well, into registers, and written to LDS one super-step
    // ahead.  Loads complete in the order they were issued: a tile requested only one super-step ahead would be the
    // youngest load but one when it is needed, and waiting for it would wait for the whole weight queue too.
    uint4 xs[DEPTH][XVEC];
    Cursor cf = cp;   // where the activation tiles are requested
    {
        uint4 x0[XVEC];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (d == 0) fetch_tile(cf, x0);
            else fetch_tile(cf, xs[d]);
            advance(cf);
            issue(qi[d], qc[d]);
        }
        stage_scales(cp);
        store_tile(lds, x0);
        __syncthreads();
    }

    v4i acc[RT][TT];
#pragma unroll
    for (int a = 0; a < RT; ++a)
#pragma unroll
        for (int t = 0; t < TT; ++t) acc[a][t] = v4i{0, 0, 0, 0};
    const int boff = DENSE ? 128 * c4 : 128 * (c4 >> 1) + 16 * (c4 & 1);
    int parity = 0;
    bool done = false;
    while (!done) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (done) break;
            uint4 ic[RT], cc[RT];
#pragma unroll
            for (int a = 0; a < RT; ++a) { ic[a] = qi[d][a]; cc[a] = qc[d][a]; }
            Cursor nx = cp;   // where the arithmetic goes next
            advance(nx);
            const bool last = nx.f == cp.f && nx.ks == cp.ks;   // the block's last super-step
            fetch_tile(cf, xs[d]);
            advance(cf);
            issue(qi[d], qc[d]);
            if (4 * cp.ks + 4 > cp.nchunks) {   // the last super-step of a ragged input dimension (the same for the whole block)
                if (4 * cp.ks + c4 >= cp.nchunks) {   // chunks past its end
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        cc[a] = make_uint4(0, 0, 0, 0);
                        if constexpr (DENSE) ic[a] = make_uint4(0, 0, 0, 0);   // all eight words are codes
                    }
                }
            }
            const int8_t *xt = lds + parity * XBUF + r * XP + boff;
            if constexpr (DENSE) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    v4i a4[RT];
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        const uint4 &half = j < 4 ? ic[a] : cc[a];
                        const uint32_t cw = (j & 3) == 0 ? half.x : (j & 3) == 1 ? half.y : (j & 3) == 2 ? half.z : half.w;
                        a4[a] = expand_codes(cw, ones);
                    }
#pragma unroll
                    for (int t = 0; t < TT; ++t) {
                        const v4i b = *reinterpret_cast<const v4i *>(xt + 16 * t * XP + 16 * j);
#pragma unroll
                        for (int a = 0; a < RT; ++a) acc[a][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a4[a], b, acc[a][t], 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    v4i a4[RT];
                    uint32_t iw[RT];
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        const uint32_t cw = j == 0 ? cc[a].x : j == 1 ? cc[a].y : j == 2 ? cc[a].z : cc[a].w;
                        iw[a] = j == 0 ? ic[a].x : j == 1 ? ic[a].y : j == 2 ? ic[a].z : ic[a].w;
                        a4[a] = expand_codes(cw, ones);
                    }
#pragma unroll
                    for (int t = 0; t < TT; ++t) {
                        const uint4 blo = *reinterpret_cast<const uint4 *>(xt + 16 * t * XP + 32 * j);
                        const uint4 bhi = *reinterpret_cast<const uint4 *>(xt + 16 * t * XP + 32 * j + 256);
                        const v8i b = {(int)blo.x, (int)blo.y, (int)blo.z, (int)blo.w, (int)bhi.x, (int)bhi.y, (int)bhi.z, (int)bhi.w};
#pragma unroll
                        for (int a = 0; a < RT; ++a)
                            acc[a][t] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a4[a], b, acc[a][t], (int)iw[a], 0, 0);
                    }
                }
            }
            store_tile(lds + (parity ^ 1) * XBUF, xs[(d + 1) % DEPTH]);
            __syncthreads();   // the next tile is in place, and nobody reads the current one any more
            parity ^= 1;
            if (cp.ks == cp.nsuper - 1) {
                // strip complete: lane holds token 16 t + r, rows 4 c4 + i of each of its row tiles
                const float g = gamma_lds;
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const float scale = __fdiv_rn(g, sx_lds[16 * t + r]);
#pragma unroll
                    for (int a = 0; a < RT; ++a) {
                        const v4f y = {(float)acc[a][t][0] * scale, (float)acc[a][t][1] * scale, (float)acc[a][t][2] * scale,
                                       (float)acc[a][t][3] * scale};
                        *reinterpret_cast<v4f *>(&ystg[(16 * t + r) * YP + wave * 16 * RT + 16 * a + 4 * c4]) = y;
                        acc[a][t] = v4i{0, 0, 0, 0};
                    }
                }
                __syncthreads();
                float *Y = uni(tab.it[cp.item].Y);
                const int row = (cp.f - cp.first) * SR + 4 * lane;
                if (4 * lane < SR && row < cp.d_out) {   // d_out is a multiple of four (host check)
                    for (int t = wave; t < cp.tokens; t += BNW) {
                        const v4f y = *reinterpret_cast<const v4f *>(&ystg[t * YP + 4 * lane]);
                        // streaming store: Y is not read again here and should not displace the weight stream in L2
                        __builtin_nontemporal_store(y, reinterpret_cast<v4f *>(Y + (int64_t)t * cp.d_out + row));
                    }
                }
                if (!last && nx.item != cp.item) {
                    __syncthreads();   // every lane has taken its scales of the finished problem
                    stage_scales(nx);  // visible after the barrier of the next super-step, long before the next epilogue
                }
            }
            done = last;
            cp = nx;
        }
    }
}

}  // namespace

// tokens <= 64, d_out % 4 == 0, d_in % 128 == 0, activations quantized; the problems of a launch share a token-tile count
bool gemv_batch_takes(const LinearItem &it)
{
    return it.tokens <= 64 && it.d_out % 4 == 0 && it.d_in % CHUNK == 0 && it.d_in <= (1 << 24) && !it.bias && !it.acc_out;
}

template <int TT, int RT, bool DENSE>
static sbn_status launch_batch_as(const BatchTable &tab, int blocks, hipStream_t stream)
{
    constexpr int DEPTH = TT * RT >= 8 ? 3 : 4;   // what the register file holds: a queue slot is 8 RT registers, a tile in flight 4 TT
    constexpr size_t lds = 2 * 16 * TT * XP + 16 * TT * (128 * RT + 4) * sizeof(float);
    static thread_local bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemv_batch_kernel<TT, RT, DEPTH, DENSE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute"); return SBN_EHIP; }
        raised = true;
    }
    hipLaunchKernelGGL((gemv_batch_kernel<TT, RT, DEPTH, DENSE>), dim3(blocks), dim3(64 * BNW), lds, stream, tab);
    return check_launch("gemv_batch_kernel");
}

sbn_status launch_gemv_batch(int count, const LinearItem *items, bool dense_codes, hipStream_t stream)
{
    for (int first = 0; first < count;) {
        // a launch: consecutive problems with the same number of token tiles (two up to 32 tokens, four up to 64)
        const int tt = items[first].tokens <= 32 ? 2 : 4;
        int n = 1;
        while (first + n < count && n < BATCH_MAX && (items[first + n].tokens <= 32 ? 2 : 4) == tt) ++n;
        // strips of 256 rows when those fill the device, of 128 rows otherwise
        int64_t wide = 0;
        for (int i = 0; i < n; ++i) wide += ceil_div(items[first + i].d_out, 256);
        const int rt = wide >= device_cus() ? 2 : 1;
        BatchTable tab;
        int s = 0;
        for (int i = 0; i < n; ++i) {
            const LinearItem &li = items[first + i];
            BatchItem &b = tab.it[i];
            b.xq = li.xq; b.sx = li.sx; b.packed = static_cast<const uint8_t *>(li.packed); b.gamma = li.gamma; b.Y = li.Y;
            b.d_in = (int)li.d_in; b.d_out = (int)li.d_out; b.tokens = (int)li.tokens; b.pad = 0;
            tab.strip0[i] = s;
            s += (int)ceil_div(li.d_out, 128 * rt);
        }
        for (int i = n; i <= 64; ++i) tab.strip0[i] = s;
        tab.count = n;
        const int blocks = s < device_cus() ? s : device_cus();
        tab.share = s / blocks;
        tab.share_rem = s % blocks;
        tab.pad = 0;
        sbn_status st;
        if (dense_codes) {
            st = tt == 2 ? (rt == 2 ? launch_batch_as<2, 2, true>(tab, blocks, stream) : launch_batch_as<2, 1, true>(tab, blocks, stream))
                         : (rt == 2 ? launch_batch_as<4, 2, true>(tab, blocks, stream) : launch_batch_as<4, 1, true>(tab, blocks, stream));
        } else {
            st = tt == 2 ? (rt == 2 ? launch_batch_as<2, 2, false>(tab, blocks, stream) : launch_batch_as<2, 1, false>(tab, blocks, stream))
                         : (rt == 2 ? launch_batch_as<4, 2, false>(tab, blocks, stream) : launch_batch_as<4, 1, false>(tab, blocks, stream));
        }
        if (st != SBN_OK) return st;
        first += n;
    }
    return SBN_OK;
}

}  // namespace sbn
