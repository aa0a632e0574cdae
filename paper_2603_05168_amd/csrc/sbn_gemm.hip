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

// A grouped launch covers the tiles of up to GEMM_GROUP_MAX problems: problem p owns the blocks
// [block0[p], block0[p+1]); every block0 is a multiple of 8 so that a problem's block i still runs on
// XCD i % 8 (blocks beyond a problem's last tile exit at once).  Problems that share tokens run
// back to back: the tail of one fills the machine together with the head of the next.
constexpr int GEMM_GROUP_MAX = 8;
struct GemmGroup {
    GemmArgs g[GEMM_GROUP_MAX];
    int block0[GEMM_GROUP_MAX + 1];
    int count;
};

// Blocks are dealt round-robin to the 8 XCDs, each with its own 4 MB L2.  XCD x takes the token
// tiles [x, x+1) * tiles_t/8 and walks them in groups of four: inside a group the token tile is the
// fastest index, then the row tile.  The 64 blocks an XCD runs at a time then share four token tiles
// (1.3 MB, resident for the whole group) while the packed weights stream through its L2 once per
// group, instead of every row tile being re-fetched for every token tile (measured: L2 miss traffic
// 15x the unique input bytes with the row tile fastest).
__device__ __forceinline__ void tile_of_block(const GemmArgs &g, int id, int &to, int &tt)
{
    const int tpx = g.tiles_t >> 3;   // token tiles per XCD
    if ((g.tiles_t & 7) == 0 && (tpx % 4 == 0 || tpx < 4)) {
        const int tg = tpx < 4 ? tpx : 4;
        const int x = id & 7, j = id >> 3;
        const int group = j / (g.tiles_o * tg), rem = j % (g.tiles_o * tg);
        to = rem / tg;
        tt = x * tpx + group * tg + rem % tg;
    } else {
        to = id % g.tiles_o;
        tt = id / g.tiles_o;
    }
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

// Epilogue of both GEMM kernels.  A wavefront owns RA row tiles x TB token tiles of 32x32; a lane
// holds one token and rows 8q + 4c + i of each row tile, so a direct store would put only 32
// contiguous bytes per token into each instruction (measured: 1.5x the algorithmic write traffic).
// The accumulators are rescaled, transposed through the now idle LDS ring (32 tokens x 32*RA rows of
// fp32 per wavefront and pass) and leave as whole rows of 128*RA bytes.  Ragged row edges and the
// int32 accumulator output take the plain per-lane stores.
//   orow = first output row of the wavefront, tok0 = its first token
template <int RA, int TB>
__device__ __forceinline__ void block_epilogue(const GemmArgs &g, v16i (&acc)[RA][TB], const float (&sxv)[TB + 1],
                                               int8_t *lds, int o0, int orow, int tok0, int wave, int lane)
{
    const int r = lane & 31, c = lane >> 5;
    const bool fast_store = (g.d_out & 3) == 0 && o0 + BO <= g.d_out && !g.acc_out;
    if (fast_store) {
        constexpr int EROW = 128 * RA + 16;     // bytes per staged token row (padded)
        constexpr int LPR = 8 * RA;             // lanes (float4) per token row
        constexpr int RPI = 64 / LPR;           // token rows per store instruction
        int8_t *const est = lds + wave * (32 * EROW);
        __syncthreads();   // every wavefront has left the main loop: the ring can be overwritten
        v4f bias4 = {0.f, 0.f, 0.f, 0.f};
        if (g.bias) bias4 = *reinterpret_cast<const v4f *>(g.bias + orow + 4 * (lane % LPR));
        const int tokens = g.tokens;
        const int64_t d_out = g.d_out;
        const bool all_tokens = tok0 + 32 * TB <= tokens;
        float *const ybase = g.Y + (int64_t)(tok0 + lane / LPR) * d_out + orow + 4 * (lane % LPR);
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            const float scale = __fdiv_rn(sxv[TB], sxv[b]);
#pragma unroll
            for (int a = 0; a < RA; ++a)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float4 y;
                    y.x = (float)acc[a][b][4 * q + 0] * scale;
                    y.y = (float)acc[a][b][4 * q + 1] * scale;
                    y.z = (float)acc[a][b][4 * q + 2] * scale;
                    y.w = (float)acc[a][b][4 * q + 3] * scale;
                    *reinterpret_cast<float4 *>(est + r * EROW + (32 * a + 8 * q + 4 * c) * 4) = y;
                }
            // the wavefront reads back what it wrote itself (its LDS operations complete in order):
            // all reads of the pass first, then the stores, so that the LDS latency is paid once
            v4f yv[32 / RPI];
#pragma unroll
            for (int j = 0; j < 32 / RPI; ++j)
                yv[j] = *reinterpret_cast<const v4f *>(est + (RPI * j + lane / LPR) * EROW + (lane % LPR) * 16);
#pragma unroll
            for (int j = 0; j < 32 / RPI; ++j) {
                yv[j] += bias4;
                // streaming store: Y is not read again here and must not push the operands out of L2
                if (all_tokens || tok0 + 32 * b + RPI * j + lane / LPR < tokens)
                    __builtin_nontemporal_store(yv[j], reinterpret_cast<v4f *>(ybase + (int64_t)(32 * b + RPI * j) * d_out));
            }
        }
        return;
    }
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const int t = tok0 + 32 * b + r;
#pragma unroll
        for (int a = 0; a < RA; ++a) store_tile(g, acc[a][b], orow + 32 * a + 4 * c, t, __fdiv_rn(sxv[TB], sxv[b]));
    }
}

// gamma and s_x[t] of the TB tokens a lane holds (token tile b: tok0 + 32 b + lane % 32), fetched
// before the first DMA so that they are long there when the epilogue divides them (a chain of
// dependent global loads at the start of the epilogue otherwise); absent tokens read the last token
template <int TB>
__device__ __forceinline__ void load_scales(const GemmArgs &g, int tok0, int lane, float (&sxv)[TB + 1])
{
    sxv[TB] = *g.gamma;
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const int t = tok0 + 32 * b + (lane & 31);
        sxv[b] = g.sx[t < g.tokens ? t : g.tokens - 1];
    }
}

// ---- sparse path --------------------------------------------------------------------------------
// 4 wavefronts, one per 64 rows of the block; each owns 64 rows x 128 tokens = 2 x 4 tiles of 32x32,
// so one code expansion (VALU) feeds four matrix instructions.
// Both operands reach LDS through LDS-DMA loads (lane l of a wavefront deposits its 16 bytes at
// base + 16*l), so no staging registers are needed and every load instruction reads whole cache lines:
//   tokens   128 tokens x 128 int8 per iteration, ring of 3 stages; one instruction fills 8 token
//            rows of 128 bytes; the 16-byte column a lane fetches is XOR-swizzled with
//            (row >> 1) & 7 so that 16-byte reads of 16 consecutive rows fall in distinct banks;
//   weights  256 rows x 64 bytes (two 32-byte chunks = two iterations) per refill, ring of 2 slots;
//            one instruction fills 16 rows; 16-byte granules swizzled with (row >> 2) & 3.
// A lane (row r = lane % 32, half c = lane / 32) reads index words 2c, 2c+1 and code words 2c, 2c+1
// of its row's chunk (two 8-byte LDS reads per row tile); sub-step u = 0, 1 uses word 2c + u, i.e.
// the lane supplies weights [64c + 32u, +32) of the chunk.
constexpr int STAGES = 3;
constexpr int WSLOT_BYTES = BO * 64;      // 16 KB: two chunks of every row of the block
constexpr int RA = 2;                     // row tiles per wavefront
constexpr int TB = BT / 32;               // token tiles per wavefront: all of the block's

__global__ void __launch_bounds__(256, 2) gemm_smfmac_kernel(GemmGroup grp)
{
    int prob = 0;
    while (prob + 1 < grp.count && (int)blockIdx.x >= grp.block0[prob + 1]) ++prob;
    const GemmArgs &g = grp.g[prob];
    const int local_id = blockIdx.x - grp.block0[prob];
    if (local_id >= g.tiles_o * g.tiles_t) return;   // padding block
    constexpr int NWAVES = 4;
    constexpr int STAGE_BYTES = BT * KSTEP;      // 16 KB
    constexpr int NDT = BT / 8 / NWAVES;         // token DMA instructions per wavefront and stage
    constexpr int NDW = 16 / NWAVES;             // weight DMA instructions per wavefront and pair
    static_assert(NDT == TB, "one token DMA instruction is issued under each matrix instruction of a row tile");
    __shared__ __attribute__((aligned(1024))) int8_t lds[STAGES * STAGE_BYTES + 2 * WSLOT_BYTES];
    const uint32_t lds0 = lds_address(lds), wlds0 = lds0 + STAGES * STAGE_BYTES;
    int to, tt;
    tile_of_block(g, local_id, to, tt);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, c = lane >> 5;
    const int K = g.d_in, nchunks = K / KSTEP, npairs = (nchunks + 1) / 2;
    const int o0 = to * BO, t0 = tt * BT;

    // DMA sources as uniform base + 32-bit lane offset, so the per-iteration advance is scalar arithmetic.
    // tokens: instruction i (0..NDT-1) of this wavefront fills tile rows (NDT*wave + i)*8 .. +7
    const int8_t *const xbase = g.xq + (int64_t)t0 * K;
    uint32_t xoff[NDT];
#pragma unroll
    for (int i = 0; i < NDT; ++i) {
        const int row = (NDT * wave + i) * 8 + (lane >> 3);
        const int t = t0 + row < g.tokens ? row : g.tokens - 1 - t0;
        xoff[i] = (uint32_t)t * (uint32_t)K + 16u * ((lane & 7) ^ ((row >> 1) & 7));
    }
    auto dma_tokens = [&](int kc, int stage) {
        const int8_t *src = xbase + (int64_t)kc * KSTEP;
        const uint32_t dst = lds0 + stage * STAGE_BYTES + wave * (NDT * 1024);
#pragma unroll
        for (int i = 0; i < NDT; ++i) lds_dma16(src, xoff[i], dst + i * 1024);
    };
    // weights: instruction i (0..NDW-1) of this wavefront fills block rows (NDW*wave + i)*16 .. +15
    const uint8_t *const wbase = g.packed + (int64_t)o0 * nchunks * 32;
    uint32_t woff[NDW];
    bool wclip[NDW];
    const bool odd_tail = (nchunks & 1) != 0;   // the last pair then holds one chunk: its second half is never read
#pragma unroll
    for (int i = 0; i < NDW; ++i) {
        const int row = (NDW * wave + i) * 16 + (lane >> 2);
        const int o = o0 + row < g.d_out ? row : g.d_out - 1 - o0;
        const int gran = (lane & 3) ^ ((row >> 2) & 3);
        woff[i] = (uint32_t)o * (uint32_t)(nchunks * 32) + 16u * gran;
        wclip[i] = odd_tail && gran >= 2;
    }
    auto dma_weights = [&](int pair, int slot) {
        const uint8_t *src = wbase + (int64_t)pair * 64;
        const uint32_t dst = wlds0 + slot * WSLOT_BYTES + wave * (NDW * 1024);
        const bool last = pair == npairs - 1;
#pragma unroll
        for (int i = 0; i < NDW; ++i) {
            // granules 2, 3 of a clipped pair lie past the row: fetch granule 0/1 again instead (never read)
            const uint32_t off = (last && wclip[i]) ? woff[i] - 32u : woff[i];
            lds_dma16(src, off, dst + i * 1024);
        }
    };
    // LDS read addresses, swizzles folded in.  tokens: row * 128 + 16 * (chunk16 ^ ((row >> 1) & 7));
    // the row's swizzle does not depend on the token tile (32 b), so tile and ring stage are immediate
    // offsets of four lane addresses.  weights: row * 64 + 16 * (granule ^ ((row >> 2) & 3)) + 8c,
    // eight lane addresses that are moved to the other slot once per pair.
    uint32_t b_lo[2], b_hi[2];   // [sub-step]
    {
        const int sw = (r >> 1) & 7;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            b_lo[u] = lds0 + r * KSTEP + 16 * ((2 * u + c) ^ sw);
            b_hi[u] = lds0 + r * KSTEP + 16 * ((4 + 2 * u + c) ^ sw);
        }
    }
    uint32_t a_idx[2][RA], a_code[2][RA];   // [chunk of the pair][row tile], in the slot of the pair being read
#pragma unroll
    for (int a = 0; a < RA; ++a) {
        const int row = wave * (32 * RA) + 32 * a + r, sw = (row >> 2) & 3;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            a_idx[h][a] = wlds0 + row * 64 + 8 * c + 16 * ((2 * h) ^ sw);
            a_code[h][a] = wlds0 + row * 64 + 8 * c + 16 * ((2 * h + 1) ^ sw);
        }
    }
    typedef __attribute__((address_space(3))) const v4i *lds_v4i;
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) const v2u *lds_u2;
    const uint32_t ones = vgpr_ones();

    v16i acc[RA][TB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0;

    // Software pipeline, one barrier per iteration placed between its two sub-steps:
    //   sub-step 0 of iteration kc   compute (kc, 0); the LDS reads of the tokens of (kc, 1) go out
    //                                under its first matrix instructions;
    //   middle                       wait for token stage kc+1 (and, for odd kc, the weight pair of
    //                                kc+1), barrier.  Every wavefront now holds all of stage kc in
    //                                registers, so its slot can take token stage kc+3 and, for odd
    //                                kc, the slot of pair (kc-1)/2 can take pair (kc+1)/2 + 1;
    //   sub-step 1                   compute (kc, 1); under its matrix instructions go those DMA
    //                                instructions and the LDS reads of the weights and tokens of (kc+1, 0).
    // A wavefront issues at most one instruction every few cycles, so what is placed between matrix
    // instructions is free while the matrix pipe is busy, and a block of other instructions after
    // them leaves the pipe idle: the source order is the intended issue order and a scheduling
    // barrier after every matrix instruction keeps it.  The DMA is unconditional (past the end it
    // fetches the last chunk again into a slot nobody reads), so the loop body has no branches and
    // the wait counts are the same every iteration; they rely on vector-memory operations of a
    // wavefront completing in issue order (tokens are issued before weights).
    float sxv[TB + 1];
    load_scales<TB>(g, t0, lane, sxv);
    // prologue in an order that leaves the ring in the state the loop's wait counts assume: behind
    // token stage 1 only token stage 2 and weight pair 1 are younger
    dma_weights(0, 0);
    dma_tokens(0, 0);
    dma_tokens(nchunks > 1 ? 1 : 0, 1);
    dma_tokens(nchunks > 2 ? 2 : nchunks - 1, 2);
    dma_weights(npairs > 1 ? 1 : 0, 1);

    v2u icur[RA], ccur[RA], inext[RA], cnext[RA];
    v8i bq[2][TB];
    auto read_weights = [&](const int h, v2u (&iv)[RA], v2u (&cv)[RA]) {
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            iv[a] = *(lds_u2)(uintptr_t)a_idx[h][a];
            cv[a] = *(lds_u2)(uintptr_t)a_code[h][a];
        }
    };
    auto token_read = [&](const int stage, const int u, const int b, v8i &bf) {
        bf.lo = *(lds_v4i)(uintptr_t)(b_lo[u] + stage * STAGE_BYTES + 32 * b * KSTEP);
        bf.hi = *(lds_v4i)(uintptr_t)(b_hi[u] + stage * STAGE_BYTES + 32 * b * KSTEP);
    };
    auto mma_row = [&](const int u, const int a, const v8i (&bf)[TB], auto &&between) {
        const int iv = (int)(u ? icur[a].y : icur[a].x);
        const v4i av = expand_codes(u ? ccur[a].y : ccur[a].x, ones);
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, bf[b], acc[a][b], iv, 0, 0);
            between(b);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    SBN_WAIT_VMCNT(NDW + 2 * NDT);   // weight pair 0 and token stage 0 are in; the three younger groups may fly
    __syncthreads();
    read_weights(0, icur, ccur);
#pragma unroll
    for (int b = 0; b < TB; ++b) token_read(0, 0, b, bq[0][b]);
    // one iteration that has a successor; stage = kc % 3 and h = kc & 1 are literals at every call
    auto iteration = [&](const int kc, const int stage, const int h) {
        mma_row(0, 0, bq[0], [&](const int b) { token_read(stage, 1, b, bq[1][b]); });
        mma_row(0, 1, bq[0], [&](const int) {});
        if (h == 0) SBN_WAIT_VMCNT(NDT + NDW); else SBN_WAIT_VMCNT(NDT);   // what the previous iteration issued may still fly
        __syncthreads();
        if (h == 1) {   // the reads below start a new pair: move the lane addresses to its slot
            const uint32_t delta = (((kc + 1) >> 1) & 1) ? (uint32_t)WSLOT_BYTES : (uint32_t)-WSLOT_BYTES;
#pragma unroll
            for (int a = 0; a < RA; ++a) {
                a_idx[0][a] += delta; a_idx[1][a] += delta; a_code[0][a] += delta; a_code[1][a] += delta;
            }
        }
        read_weights(h ^ 1, inext, cnext);
        __builtin_amdgcn_sched_barrier(0);
        const int kt = kc + 3 < nchunks ? kc + 3 : nchunks - 1;
        const int8_t *tsrc = xbase + (int64_t)kt * KSTEP;
        const uint32_t tdst = lds0 + stage * STAGE_BYTES + wave * (NDT * 1024);
        mma_row(1, 0, bq[1], [&](const int b) { lds_dma16(tsrc, xoff[b], tdst + b * 1024); });
        if (h == 1) {
            const int pw = (kc + 1) / 2 + 1;
            dma_weights(pw < npairs ? pw : npairs - 1, pw & 1);
        }
        mma_row(1, 1, bq[1], [&](const int b) { token_read(stage == 2 ? 0 : stage + 1, 0, b, bq[0][b]); });
#pragma unroll
        for (int a = 0; a < RA; ++a) { icur[a] = inext[a]; ccur[a] = cnext[a]; }
    };
    const int nsteady = nchunks - 1;   // iterations with a successor
    int kc = 0;
    for (; kc + 6 <= nsteady; kc += 6) {
        iteration(kc, 0, 0);
        iteration(kc + 1, 1, 1);
        iteration(kc + 2, 2, 0);
        iteration(kc + 3, 0, 1);
        iteration(kc + 4, 1, 0);
        iteration(kc + 5, 2, 1);
    }
    // up to five more, selected so that stage and h stay literals (kc is a multiple of 6 here)
    if (kc < nsteady) { iteration(kc, 0, 0); ++kc; }
    if (kc < nsteady) { iteration(kc, 1, 1); ++kc; }
    if (kc < nsteady) { iteration(kc, 2, 0); ++kc; }
    if (kc < nsteady) { iteration(kc, 0, 1); ++kc; }
    if (kc < nsteady) { iteration(kc, 1, 0); ++kc; }
    // last chunk: nothing left to fetch
    {
        const int stage = kc % STAGES;
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            bq[1][b].lo = *(lds_v4i)(uintptr_t)(b_lo[1] + stage * STAGE_BYTES + 32 * b * KSTEP);
            bq[1][b].hi = *(lds_v4i)(uintptr_t)(b_hi[1] + stage * STAGE_BYTES + 32 * b * KSTEP);
        }
        mma_row(0, 0, bq[0], [&](const int) {});
        mma_row(0, 1, bq[0], [&](const int) {});
        mma_row(1, 0, bq[1], [&](const int) {});
        mma_row(1, 1, bq[1], [&](const int) {});
    }
    SBN_WAIT_VMCNT(0);   // surplus DMA of the last iterations must not land in the epilogue's staging area

    block_epilogue<RA, TB>(g, acc, sxv, lds, o0, o0 + wave * (32 * RA), t0, wave, lane);
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

// Same block and wave shapes as the sparse kernel and the same LDS-DMA machinery, so that the two
// paths differ only in what the matrix instruction is fed: dense int8 rows with explicit zeros
// (no index register, no code expansion) into v_mfma_i32_32x32x32_i8, twice as many of them.
// Stage = 64 k of the 256 weight rows and 128 token rows (64-byte rows, 24 KB), ring of 3 stages;
// one DMA instruction fills 16 rows, 16-byte granules swizzled with (row >> 2) & 3.
constexpr int DK = 64;
constexpr int DSTAGE = (BO + BT) * DK;   // 24 KB

__global__ void __launch_bounds__(256, 2) gemm_dense_kernel(GemmArgs g)
{
    __shared__ __attribute__((aligned(1024))) int8_t lds[STAGES * DSTAGE];
    const uint32_t lds0 = lds_address(lds);
    int to, tt;
    tile_of_block(g, blockIdx.x, to, tt);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wo = wave & 1, wt = wave >> 1;
    const int r = lane & 31, c = lane >> 5;
    const int K = g.d_in, nk = K / DK;
    const int o0 = to * BO, t0 = tt * BT;

    const int8_t *const wbase = g.w_dense + (int64_t)o0 * K;
    const int8_t *const xbase = g.xq + (int64_t)t0 * K;
    uint32_t woff[4], xoff[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (4 * wave + i) * 16 + (lane >> 2);
        const int o = o0 + row < g.d_out ? row : g.d_out - 1 - o0;
        woff[i] = (uint32_t)o * (uint32_t)K + 16u * ((lane & 3) ^ ((row >> 2) & 3));
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = (2 * wave + i) * 16 + (lane >> 2);
        const int t = t0 + row < g.tokens ? row : g.tokens - 1 - t0;
        xoff[i] = (uint32_t)t * (uint32_t)K + 16u * ((lane & 3) ^ ((row >> 2) & 3));
    }
    // lane (r, c) supplies k = 32u + 16c + 0..15 of the stage = granule 2u + c, for both operands;
    // row tile and ring stage are immediate offsets of the lane addresses below
    typedef __attribute__((address_space(3))) const v4i *lds_v4i;
    uint32_t aaddr[2], baddr[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int sw = (r >> 2) & 3;   // (row >> 2) & 3 with row = 32 a + r + a multiple of 64
        aaddr[u] = lds0 + (wo * 128 + r) * DK + 16 * ((2 * u + c) ^ sw);
        baddr[u] = lds0 + BO * DK + (wt * 64 + r) * DK + 16 * ((2 * u + c) ^ sw);
    }

    v16i acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0;

    float sxv[3];
    load_scales<2>(g, t0 + wt * 64, lane, sxv);
    // Same software pipeline as the sparse kernel: ring of 3 stages, one barrier per iteration
    // between its two sub-steps, the DMA of stage kt+3 and the LDS reads of the next sub-step issued
    // between the matrix instructions, unconditional clamped DMA, stage as a literal.
    auto dma_one = [&](int kt, int stage, const int i) {   // i = 0..5: four weight and two token instructions
        const uint32_t dst = lds0 + stage * DSTAGE;
        if (i < 4) lds_dma16(wbase + (int64_t)kt * DK, woff[i], dst + (4 * wave + i) * 1024);
        else lds_dma16(xbase + (int64_t)kt * DK, xoff[i - 4], dst + BO * DK + (2 * wave + i - 4) * 1024);
    };
    auto dma = [&](int kt, int stage) {
#pragma unroll
        for (int i = 0; i < 6; ++i) dma_one(kt, stage, i);
    };
    v4i af[2][4], bf[2][2];
    auto read_a = [&](const int stage, const int u, const int a) {
        af[u][a] = *(lds_v4i)(uintptr_t)(aaddr[u] + stage * DSTAGE + 32 * a * DK);
    };
    auto read_b = [&](const int stage, const int u, const int b) {
        bf[u][b] = *(lds_v4i)(uintptr_t)(baddr[u] + stage * DSTAGE + 32 * b * DK);
    };
    auto mma = [&](const int u, const int a, const int b) {
        acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[u][a], bf[u][b], acc[a][b], 0, 0, 0);
    };
    dma(0, 0);
    dma(nk > 1 ? 1 : 0, 1);
    dma(nk > 2 ? 2 : nk - 1, 2);
    SBN_WAIT_VMCNT(12);   // stage 0 is in
    __syncthreads();
#pragma unroll
    for (int a = 0; a < 4; ++a) read_a(0, 0, a);
#pragma unroll
    for (int b = 0; b < 2; ++b) read_b(0, 0, b);
    auto iteration = [&](const int kt, const int stage) {   // stage = kt % 3 as a literal
        // sub-step 0; the six reads of sub-step 1 go out under its first matrix instructions
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            mma(0, i >> 1, i & 1);
            if (i < 4) read_a(stage, 1, i);
            else if (i < 6) read_b(stage, 1, i - 4);
            __builtin_amdgcn_sched_barrier(0);
        }
        SBN_WAIT_VMCNT(6);   // stage kt+1 is in; stage kt+2 may fly
        __syncthreads();
        const int kf = kt + 3 < nk ? kt + 3 : nk - 1;
        const int nstage = stage == 2 ? 0 : stage + 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            mma(1, i >> 1, i & 1);
            if (i < 6) dma_one(kf, stage, i);
            if (i >= 2 && i < 6) read_a(nstage, 0, i - 2);
            else if (i >= 6) read_b(nstage, 0, i - 6);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    const int nsteady = nk - 1;
    int kt = 0;
    for (; kt + 3 <= nsteady; kt += 3) {
        iteration(kt, 0);
        iteration(kt + 1, 1);
        iteration(kt + 2, 2);
    }
    if (kt < nsteady) { iteration(kt, 0); ++kt; }
    if (kt < nsteady) { iteration(kt, 1); ++kt; }
    {
        const int stage = kt % STAGES;
#pragma unroll
        for (int a = 0; a < 4; ++a) af[1][a] = *(lds_v4i)(uintptr_t)(aaddr[1] + stage * DSTAGE + 32 * a * DK);
#pragma unroll
        for (int b = 0; b < 2; ++b) bf[1][b] = *(lds_v4i)(uintptr_t)(baddr[1] + stage * DSTAGE + 32 * b * DK);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i) mma(u, i >> 1, i & 1);
    }
    SBN_WAIT_VMCNT(0);   // surplus DMA of the last iterations must not land in the epilogue's staging area
    block_epilogue<4, 2>(g, acc, sxv, lds, o0, o0 + wo * 128, t0 + wt * 64, wave, lane);
}

GemmArgs make_args(const LinearItem &it, int block_tokens = BT)
{
    GemmArgs g;
    g.xq = it.xq; g.sx = it.sx; g.packed = static_cast<const uint8_t *>(it.packed); g.w_dense = nullptr;
    g.gamma = it.gamma; g.bias = it.bias; g.Y = it.Y; g.acc_out = it.acc_out;
    g.tokens = (int)it.tokens; g.d_in = (int)it.d_in; g.d_out = (int)it.d_out;
    g.tiles_o = (int)ceil_div(it.d_out, BO);
    g.tiles_t = (int)ceil_div(it.tokens, block_tokens);
    return g;
}

}  // namespace

sbn_status launch_gemm_smfmac(int count, const LinearItem *items, hipStream_t stream)
{
    for (int first = 0; first < count; first += GEMM_GROUP_MAX) {
        GemmGroup grp;
        grp.count = count - first < GEMM_GROUP_MAX ? count - first : GEMM_GROUP_MAX;
        int blocks = 0;
        for (int i = 0; i < grp.count; ++i) {
            grp.g[i] = make_args(items[first + i]);
            grp.block0[i] = blocks;
            blocks += (grp.g[i].tiles_o * grp.g[i].tiles_t + 7) & ~7;
        }
        grp.block0[grp.count] = blocks;
        hipLaunchKernelGGL(gemm_smfmac_kernel, dim3(blocks), dim3(256), 0, stream, grp);
        sbn_status st = check_launch("gemm_smfmac_kernel");
        if (st != SBN_OK) return st;
    }
    return SBN_OK;
}

sbn_status launch_gemm_dense(const LinearItem &it, const Pattern &pat, int8_t *w_dense, hipStream_t stream)
{
    sbn_status st;
    if (pat.N == 2 && pat.M == 4 && it.d_in % CHUNK == 0) {
        const int64_t ngroups = it.d_out * it.d_in / 4;
        hipLaunchKernelGGL(expand_dense_kernel, dim3((unsigned)ceil_div(ngroups, 256)), dim3(256), 0, stream,
                           static_cast<const uint8_t *>(it.packed), w_dense, ngroups);
        st = check_launch("expand_dense_kernel");
    } else {
        // any other pattern (6:8, 2:8, 1:4, ...): the format-generic group decoder writes the same int8 W_eff
        st = launch_expand_groups(it.packed, it.d_out, it.d_in, pat, w_dense, stream);
    }
    if (st != SBN_OK) return st;
    GemmArgs g = make_args(it);
    g.w_dense = w_dense;
    hipLaunchKernelGGL(gemm_dense_kernel, dim3(g.tiles_o * g.tiles_t), dim3(256), 0, stream, g);
    return check_launch("gemm_dense_kernel");
}

}  // namespace sbn
