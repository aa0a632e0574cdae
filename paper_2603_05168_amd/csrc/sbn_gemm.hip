// Prefill / training GEMM of the sparse ternary linear layer on CDNA4 int8 matrix cores (2:4).
//   acc[t, o] = sum_k W_eff[o, k] * xq[t, k],   Y = acc * gamma / s_x[t] (+ bias)
// Section 2.2 (forward-pass equation).  Two paths:
//   sparse  v_smfmac_i32_32x32x64_i8: the packed weights ARE the compressed A operand (code word ->
//           16 int8 values, index word -> the instruction's index register), tokens are B;
//   dense   v_mfma_i32_32x32x32_i8 on W_eff expanded to int8 with explicit zeros: the in-run
//           comparison a dense ternary layer would run.
#include <algorithm>
#include <vector>

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

// A launch of the sparse kernel covers up to GEMM_GROUP_MAX problems with a work list, or up to GEMM_GROUP_WIDE
// problems of few tokens each (decode batches), whose work is dealt by row tile (see gemm_smfmac_kernel).
constexpr int GEMM_GROUP_MAX = 8, GEMM_GROUP_WIDE = 32;
template <int NP>
struct GemmGroupT {
    GemmArgs g[NP];
    int count;
};
using GemmGroup = GemmGroupT<GEMM_GROUP_MAX>;
using GemmGroupWide = GemmGroupT<GEMM_GROUP_WIDE>;

// Work list of a launch of the sparse kernel, made on the host: block b runs the pieces piece[b * per_block + i],
// i < per_block, up to the first empty one (width 0).  A piece = (problem, row tile of 512, first token unit of 32 tokens,
// width in units 1 .. 4).  per_block == 0: no list, the kernel splits the units by formula.
// per_block < 0: no list either, the problems have few tokens and the pieces are (problem, row tile, four token units),
// -per_block of them in all, dealt to the blocks in contiguous runs.
constexpr int PIECE_TABLE_MAX = 768;
template <int NE>
struct PieceTableT {
    int per_block;
    uint32_t piece[NE];   // bits [2:0] width, [15:3] first unit, [24:16] row tile, [27:25] problem
};
using PieceTable = PieceTableT<PIECE_TABLE_MAX>;
using PieceTableNone = PieceTableT<1>;
static_assert(sizeof(GemmGroup) + sizeof(PieceTable) <= 4000, "both travel as kernel arguments");
static_assert(sizeof(GemmGroupWide) + sizeof(PieceTableNone) <= 4000, "both travel as kernel arguments");

// Tile order of the dense comparison kernel.
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
// One persistent block of eight wavefronts per multiprocessor; block tile 512 rows x 128 tokens.  Wavefront w owns the
// rows 64 w .. 64 w + 63 (two row tiles of 32) and all tokens of the piece (TB = 1 .. 4 token tiles of 32), so one code
// expansion (nine vector instructions) feeds TB matrix instructions: measured on this part, up to four vector
// instructions per matrix instruction hide under it, more cost their full time.  The two wavefronts of a SIMD cover
// each other's waits.  Per 128-k step the wavefronts read 144 KB of operand fragments from LDS and the DMA deposits
// 32 KB; measured with a microbenchmark, reads (475 bytes/ns) and deposits (105 bytes/ns from L2) overlap, so it is
// the deposit path that is scarce: a step's 32 KB are 0.3 us of it against 0.5 us of matrix work.  Against two
// independent blocks of 256 x 128 the shared token tile saves a third of those bytes (256 instead of 384 bytes per
// matrix instruction).
// Both operands reach LDS through LDS-DMA loads (lane l of a wavefront deposits its 16 bytes at base + 16*l), so no
// staging registers are needed and every load instruction reads whole cache lines:
//   tokens   128 tokens x 128 int8 per stage, ring of NST stages; one instruction fills 8 token rows of 128 bytes; the
//            16-byte column a lane fetches is XOR-swizzled with (row >> 1) & 7 so that 16-byte reads of 16
//            consecutive rows fall in distinct banks;
//   weights  512 rows x 64 bytes (two 32-byte chunks = two iterations) per pair slot, ring of NWP slots; one instruction
//            fills 16 rows; 16-byte granules swizzled with (row >> 2) & 3.
// A lane (row r = lane % 32, half c = lane / 32) reads index words 2c, 2c+1 and code words 2c, 2c+1 of its row's chunk
// (two 8-byte LDS reads per row tile); sub-step u = 0, 1 uses word 2c + u, i.e. the lane supplies weights
// [64c + 32u, +32) of the chunk.
// Pieces follow one another without draining the pipeline: when the main loop of a piece ends, the first stages of the
// block's next piece are requested BEFORE the epilogue of the finished one runs, and the epilogue transposes through a
// staging area of its own, so the ring is never idle.
namespace sp {

constexpr int ROWS = 512;                      // rows of W per block tile
constexpr int NW = 8;                          // wavefronts
constexpr int RA = 2;                          // row tiles per wavefront
constexpr int NST = 3;                         // token stages (16 KB each)
constexpr int NWP = 2;                         // weight pair slots (32 KB each)
constexpr int TSTAGE = 128 * KSTEP;
constexpr int WPAIR = ROWS * 64;
constexpr int RING_BYTES = NST * TSTAGE + NWP * WPAIR;
// epilogue staging, one area per wavefront: 16 tokens x (64 rows of fp32 + 16 bytes of padding)
constexpr int STG_TOKENS = 16;
constexpr int EROW = 128 * RA + 16;
constexpr int STG_WAVE = STG_TOKENS * EROW;
// per-token scales of a piece (128 floats), fetched by DMA with its first stages; two areas, used alternately, because
// the scales of the next piece arrive while the epilogue of the current one still reads its own
constexpr int SCALES_OFF = RING_BYTES + NW * STG_WAVE;
constexpr int LDS_BYTES = SCALES_OFF + 2 * 512;
static_assert(LDS_BYTES <= 160 * 1024, "ring, staging and scales share the multiprocessor's LDS");
constexpr int NDW = 32 / NW;                   // weight DMA instructions per wavefront and pair (16 rows each)
constexpr int token_dma(int TB) { return (4 * TB + NW - 1) / NW; }   // token DMA instructions per wavefront and stage (8 rows each)
constexpr int cmin(int a, int b) { return a < b ? a : b; }

// Bookkeeping of the DMA ring at compile time.  Iteration j (negative j = the prologue) issues, in this order,
// weight pair (j - 1) / 2 + NWP if j is odd (NDW instructions), then token stage j + NST (NDT instructions); items with
// a negative number do not exist.  Returns how many DMA instructions of a wavefront are issued after the given item
// in iterations jlo .. jhi: the count a wait for that item may leave outstanding (the loads of a wavefront complete
// in issue order).
constexpr int issued_after(int NDT, int jlo, int jhi, bool want_pair, int id)
{
    int n = -1;
    for (int j = jlo; j <= jhi; ++j) {
        if (j & 1) {
            const int pid = (j - 1) / 2 + NWP;
            if (pid >= 0) {
                if (n >= 0) n += NDW;
                else if (want_pair && pid == id) n = 0;
            }
        }
        const int sid = j + NST;
        if (sid >= 0) {
            if (n >= 0) n += NDT;
            else if (!want_pair && sid == id) n = 0;
        }
    }
    return n;
}
constexpr int LEAD = NST > 2 * NWP - 1 ? NST : 2 * NWP - 1;          // prologue iterations -LEAD .. -1

// What a wavefront needs to issue the DMA of one piece: uniform bases and 32-bit lane offsets (the per-iteration
// advance is scalar arithmetic).  Token instruction i of wavefront w fills tile rows (NDT w + i) 8 .. + 7, weight
// instruction i fills block rows (NDW w + i) 16 .. + 15.
template <int NDT>
struct PieceDma {
    const int8_t *xbase;
    const uint8_t *wbase;
    uint32_t xoff[NDT], woff[NDW];
    uint32_t wclip;            // bit i: instruction i fetches granules 2, 3 of its rows, which do not exist in an odd last pair
    int nchunks, npairs;
};

template <int NDT>
__device__ __forceinline__ void dma_setup(PieceDma<NDT> &d, const GemmArgs &g, int to, int t0, int tb, int wave, int lane)
{
    const int K = g.d_in;
    d.nchunks = K / KSTEP;
    d.npairs = (d.nchunks + 1) / 2;
    d.xbase = g.xq + (int64_t)t0 * K;
#pragma unroll
    for (int i = 0; i < NDT; ++i) {
        int row = (NDT * wave + i) * 8 + (lane >> 3);
        const int sw = (row >> 1) & 7;
        row = row < 32 * tb ? row : 32 * tb - 1;                      // rows past the piece: its last row again (never read)
        const int t = t0 + row < g.tokens ? row : g.tokens - 1 - t0;   // tokens past the matrix: its last token again
        d.xoff[i] = (uint32_t)t * (uint32_t)K + 16u * ((lane & 7) ^ sw);
    }
    const int o0 = to * ROWS;
    d.wbase = g.packed + (int64_t)o0 * d.nchunks * 32;
    const bool odd_tail = (d.nchunks & 1) != 0;
    d.wclip = 0;
#pragma unroll
    for (int i = 0; i < NDW; ++i) {
        const int row = (NDW * wave + i) * 16 + (lane >> 2);
        const int o = o0 + row < g.d_out ? row : g.d_out - 1 - o0;     // rows past the matrix: its last row again
        const int gran = (lane & 3) ^ ((row >> 2) & 3);
        d.woff[i] = (uint32_t)o * (uint32_t)(d.nchunks * 32) + 16u * gran;
        if (odd_tail && gran >= 2) d.wclip |= 1u << i;
    }
}

// stages and pairs past the end are fetched again from the last one (into a slot nobody reads): the DMA is
// unconditional, so that the wait counts are the same in every iteration
template <int NDT>
__device__ __forceinline__ void dma_token(const PieceDma<NDT> &d, uint32_t lds0, int wave, int kc, int slot, int i)
{
    kc = kc < d.nchunks ? kc : d.nchunks - 1;
    lds_dma16(d.xbase + (int64_t)kc * KSTEP, d.xoff[i], lds0 + slot * TSTAGE + wave * (NDT * 1024) + i * 1024);
}

template <int NDT>
__device__ __forceinline__ void dma_weight(const PieceDma<NDT> &d, uint32_t lds0, int wave, int pair, int slot, int i)
{
    pair = pair < d.npairs ? pair : d.npairs - 1;
    // granules 2, 3 of a clipped pair lie past the row: fetch granule 0/1 again instead (never read)
    const uint32_t off = (pair == d.npairs - 1 && ((d.wclip >> i) & 1u)) ? d.woff[i] - 32u : d.woff[i];
    lds_dma16(d.wbase + (int64_t)pair * 64, off, lds0 + NST * TSTAGE + slot * WPAIR + wave * (NDW * 1024) + i * 1024);
}

// the items of iterations -LEAD .. -1, in the order the wait counts assume
template <int NDT>
__device__ __forceinline__ void dma_prologue(const PieceDma<NDT> &d, uint32_t lds0, int wave)
{
#pragma unroll
    for (int j = -LEAD; j <= -1; ++j) {
        if ((j & 1) && (j - 1) / 2 + NWP >= 0) {
#pragma unroll
            for (int i = 0; i < NDW; ++i) dma_weight(d, lds0, wave, (j - 1) / 2 + NWP, ((j - 1) / 2 + NWP) % NWP, i);
        }
        if (j + NST >= 0) {
#pragma unroll
            for (int i = 0; i < NDT; ++i) dma_token(d, lds0, wave, j + NST, (j + NST) % NST, i);
        }
    }
}

// A piece of the work list: (problem, row tile, first token, width in token tiles); width 0 = none.
struct Piece {
    int prob, to, t0, tb;
    int parity;   // which of the two scale areas the piece uses
};

// requests the first stages of a piece (called with the ring idle: before the first piece and between the main loop
// and the epilogue of the piece before)
template <class Group>
__device__ __forceinline__ void piece_prologue(const Group &grp, const Piece &p, int8_t *lds, int wave, int lane)
{
    const uint32_t lds0 = lds_address(lds);
    const GemmArgs &g = grp.g[p.prob];
    // s_x of the piece's tokens, by the first wavefront and in front of everything else: the oldest request of the
    // piece, so every wait for a stage covers it and no wait count changes
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int t = p.t0 + 64 * i + lane;
            lds_dma4(g.sx, 4u * (uint32_t)(t < g.tokens ? t : g.tokens - 1), lds0 + SCALES_OFF + 512 * p.parity + 256 * i);
        }
    }
    if (token_dma(p.tb) == 2) {
        PieceDma<2> d;
        dma_setup(d, g, p.to, p.t0, p.tb, wave, lane);
        dma_prologue(d, lds0, wave);
    } else {
        PieceDma<1> d;
        dma_setup(d, g, p.to, p.t0, p.tb, wave, lane);
        dma_prologue(d, lds0, wave);
    }
}

// Main loop and epilogue of one piece whose prologue is already in flight: rows [512 to, +512) of W against tokens
// [t0, t0 + 32 TB), the whole input dimension.  LIVE = false: a wavefront whose rows lie past the matrix (ragged last
// row tile) only moves data and keeps the barriers.
template <int TB, bool LIVE, bool DENSE, class Group>
__device__ __forceinline__ void piece_body(const Group &grp, const Piece &p, const Piece &next, int8_t *lds, const int wave,
                                           int lane)
{
    // everything derived from the lane number is computed anew for every piece: hoisted out of the loop over pieces,
    // the lane addresses of all instantiations would be live at once and spill
    asm volatile("" : "+v"(lane));
    constexpr int NDT = token_dma(TB);
    constexpr int WAIT_TOP = cmin(issued_after(NDT, -LEAD, -1, false, 0), issued_after(NDT, -LEAD, -1, true, 0));
    // in the middle of iteration kc: token stage kc + 1 and, for odd kc, weight pair (kc + 1) / 2 must have landed
    constexpr int WAIT_EVEN = issued_after(NDT, -LEAD, 99, false, 101);
    constexpr int WAIT_ODD = cmin(issued_after(NDT, -LEAD, 100, false, 102), issued_after(NDT, -LEAD, 100, true, 51));
    static_assert(WAIT_TOP >= 0 && WAIT_EVEN >= 0 && WAIT_ODD >= 0 && WAIT_TOP < 64 && WAIT_EVEN < 64 && WAIT_ODD < 64,
                  "ring bookkeeping");
    const GemmArgs &g = grp.g[p.prob];
    const int to = p.to, t0 = p.t0;
    const uint32_t lds0 = lds_address(lds), wlds0 = lds0 + NST * TSTAGE;
    const int r = lane & 31, c = lane >> 5;
    const int nchunks = g.d_in / KSTEP;
    const int o0 = to * ROWS;
    PieceDma<NDT> d;
    dma_setup(d, g, to, t0, TB, wave, lane);

    // ---- LDS read addresses (swizzles as in the DMA patterns above)
    uint32_t b_lo[2], b_hi[2];   // [sub-step]; the token tile is an immediate offset, the ring slot a scalar
    {
        const int sw = (r >> 1) & 7;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            b_lo[u] = lds0 + r * KSTEP + 16 * ((2 * u + c) ^ sw);
            b_hi[u] = lds0 + r * KSTEP + 16 * ((4 + 2 * u + c) ^ sw);
        }
    }
    // [chunk of the pair][row tile], slot 0.  2:4: index words 2c, 2c+1 and code words 2c, 2c+1 of the chunk (8 bytes
    // each); dense codes: words 4c .. 4c+3 of the chunk's eight code words (a_idx alone, 16 bytes)
    uint32_t a_idx[2][RA], a_code[2][RA];
#pragma unroll
    for (int a = 0; a < RA; ++a) {
        const int row = wave * (32 * RA) + 32 * a + r, sw = (row >> 2) & 3;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if constexpr (DENSE) {
                a_idx[h][a] = wlds0 + row * 64 + 16 * ((2 * h + c) ^ sw);
                a_code[h][a] = 0;
            } else {
                a_idx[h][a] = wlds0 + row * 64 + 8 * c + 16 * ((2 * h) ^ sw);
                a_code[h][a] = wlds0 + row * 64 + 8 * c + 16 * ((2 * h + 1) ^ sw);
            }
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

    // 2:4: (icur, ccur) = the lane's two index and two code words of the current chunk; dense codes: its four code words
    v2u icur[RA], ccur[RA], inext[RA], cnext[RA];
    v8i bq[2][TB];
    auto read_weights = [&](const int slot, const int h, const int a, v2u (&iv)[RA], v2u (&cv)[RA]) {
        if constexpr (DENSE) {
            typedef unsigned v4u __attribute__((ext_vector_type(4)));
            const v4u w = *(__attribute__((address_space(3))) const v4u *)(uintptr_t)(a_idx[h][a] + slot * WPAIR);
            iv[a] = v2u{w.x, w.y};
            cv[a] = v2u{w.z, w.w};
        } else {
            iv[a] = *(lds_u2)(uintptr_t)(a_idx[h][a] + slot * WPAIR);
            cv[a] = *(lds_u2)(uintptr_t)(a_code[h][a] + slot * WPAIR);
        }
    };
    auto token_read = [&](const int slot, const int u, const int b, v8i &bf) {
        bf.lo = *(lds_v4i)(uintptr_t)(b_lo[u] + slot * TSTAGE + 32 * b * KSTEP);
        bf.hi = *(lds_v4i)(uintptr_t)(b_hi[u] + slot * TSTAGE + 32 * b * KSTEP);
    };
    // One sub-step: RA x TB matrix instructions; side(s) is issued after instruction s (s = 0 .. RA * TB - 1).  A
    // wavefront issues at most one instruction every few cycles, so what is placed between matrix instructions is free
    // while the matrix pipe is busy, and a block of other instructions after them leaves the pipe idle: the source order
    // is the intended issue order and a scheduling barrier after every matrix instruction keeps it.
    // Dense codes: every group of four weights is the sum of a 2:4 group holding its positions 0, 1 and one holding its
    // positions 2, 3, so the same B fragment feeds two sparse instructions with constant index words.
    constexpr int NSLOT = (DENSE ? 2 : 1) * RA * TB;
    auto substep = [&](const int u, const v8i (&bf)[TB], auto &&side) {
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            if constexpr (LIVE && DENSE) {
                v4i a01, a23;   // sub-step u covers the lane's code words 2u, 2u + 1
                expand_dense_codes(u ? ccur[a].x : icur[a].x, u ? ccur[a].y : icur[a].y, a01, a23);
#pragma unroll
                for (int b = 0; b < TB; ++b) {
                    acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(a01, bf[b], acc[a][b], 0x44444444, 0, 0);
                    side(2 * a * TB + b);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int b = 0; b < TB; ++b) {
                    acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(a23, bf[b], acc[a][b], (int)0xeeeeeeeeu, 0, 0);
                    side((2 * a + 1) * TB + b);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else if constexpr (LIVE) {
                const int iv = (int)(u ? icur[a].y : icur[a].x);
                const v4i av = expand_codes(u ? ccur[a].y : ccur[a].x, ones);
#pragma unroll
                for (int b = 0; b < TB; ++b) {
                    acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, bf[b], acc[a][b], iv, 0, 0);
                    side(a * TB + b);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int s = 0; s < NSLOT / RA; ++s) side(a * (NSLOT / RA) + s);
            }
        }
    };

    // Weight pair 0 and token stage 0 are in; what was requested after them may fly.  The count is of ALL outstanding
    // vector-memory operations: loads complete in issue order among themselves, but stores (the epilogue of the piece
    // before, issued after this piece's first requests) may be acknowledged before older loads, so they cannot be
    // granted as outstanding - with at most WAIT_TOP operations of any kind in flight, at most WAIT_TOP loads are.
    SBN_WAIT_VMCNT(WAIT_TOP);
    __syncthreads();
    if constexpr (LIVE) {
#pragma unroll
        for (int a = 0; a < RA; ++a) read_weights(0, 0, a, icur, ccur);
#pragma unroll
        for (int b = 0; b < TB; ++b) token_read(0, 0, b, bq[0][b]);
    }
    // One iteration that has a successor; ts = kc % NST and ps = (kc / 2) % NWP are scalars, h = kc & 1 is a literal.
    //   sub-step 0   compute (kc, first half); the token fragments of the second half are read under it
    //   middle       wait for token stage kc + 1 (odd kc: and weight pair (kc + 1) / 2), barrier: every wavefront
    //                now holds all of stage kc in registers, so its slot takes stage kc + NST, and for odd kc the
    //                slot of pair kc / 2 takes pair kc / 2 + NWP
    //   sub-step 1   compute (kc, second half); under it go the DMA instructions, the weight words of chunk kc + 1
    //                and the token fragments of (kc + 1, first half), one per matrix instruction
    // The wait counts hold the outstanding DMA of this wavefront only; stores of the epilogue before that are still in
    // flight in the first iterations make a wait longer, never shorter.
    auto iteration = [&](const int kc, const int ts, const int ps, const int h) {
        substep(0, bq[0], [&](const int s) {
            if constexpr (LIVE) { if (s < TB) token_read(ts, 1, s, bq[1][s]); }
        });
        if (h == 0) SBN_WAIT_VMCNT(WAIT_EVEN); else SBN_WAIT_VMCNT(WAIT_ODD);
        __syncthreads();
        const int nts = ts + 1 == NST ? 0 : ts + 1;                         // slot of token stage kc + 1
        const int nps = h == 1 ? (ps + 1 == NWP ? 0 : ps + 1) : ps;         // slot of the pair of chunk kc + 1
        substep(1, bq[1], [&](const int s) {
            // side operations in issue order: weight DMA (odd kc), token DMA, weight words, token fragments;
            // operation k goes to slot k, the last slot takes what is left over
            constexpr int NOPS = NDW + NDT + RA + TB;
#pragma unroll
            for (int k = 0; k < NOPS; ++k) {
                if ((k < NSLOT ? k : NSLOT - 1) != s) continue;
                if (k < NDW) { if (h == 1) dma_weight(d, lds0, wave, kc / 2 + NWP, ps, k); }
                else if (k < NDW + NDT) dma_token(d, lds0, wave, kc + NST, ts, k - NDW);
                else if constexpr (LIVE) {
                    if (k < NDW + NDT + RA) read_weights(nps, h ^ 1, k - NDW - NDT, inext, cnext);
                    else token_read(nts, 0, k - NDW - NDT - RA, bq[0][k - NDW - NDT - RA]);
                }
            }
        });
        if constexpr (LIVE) {
#pragma unroll
            for (int a = 0; a < RA; ++a) { icur[a] = inext[a]; ccur[a] = cnext[a]; }
        }
    };
    const int nsteady = nchunks - 1;   // iterations with a successor
    int kc = 0, ts = 0, ps = 0;
    for (; kc + 2 <= nsteady; kc += 2) {
        iteration(kc, ts, ps, 0);
        ts = ts + 1 == NST ? 0 : ts + 1;
        iteration(kc + 1, ts, ps, 1);
        ts = ts + 1 == NST ? 0 : ts + 1;
        ps = ps + 1 == NWP ? 0 : ps + 1;
    }
    if (kc < nsteady) {
        iteration(kc, ts, ps, 0);
        ts = ts + 1 == NST ? 0 : ts + 1;
    }
    // last chunk: nothing left to fetch
    {
        if constexpr (LIVE) {
#pragma unroll
            for (int b = 0; b < TB; ++b) token_read(ts, 1, b, bq[1][b]);
        }
        substep(0, bq[0], [&](const int) {});
        substep(1, bq[1], [&](const int) {});
    }
    __syncthreads();     // every wavefront has read the last stage: the ring can take the next piece
    // The surplus DMA of the last iterations is still in flight: it lands in ring slots that nobody reads any more and
    // that the same wavefront's later requests overwrite in issue order; the staging area lies outside the ring.
    if (next.tb > 0) piece_prologue(grp, next, lds, wave, lane);

    // ---- epilogue: rescale, transpose through the wavefront's staging area (16 tokens x 64 rows of fp32 per pass) and
    // write whole rows of 256 bytes with streaming stores (Y is not read again here and must not push the operands out
    // of L2; per-lane stores of 32 contiguous bytes measured 1.5x the write traffic); ragged edges and the int32
    // accumulator output store per lane
    // The epilogue issues no vector loads: one would make the compiler wait for everything outstanding, the requests
    // for the next piece included.  gamma is a scalar load, the s_x of the piece came into LDS with its first stages.
    if constexpr (LIVE) {
        float sxv[TB + 1];
        sxv[TB] = *g.gamma;
#pragma unroll
        for (int b = 0; b < TB; ++b) sxv[b] = *reinterpret_cast<const float *>(lds + SCALES_OFF + 512 * p.parity + 4 * (32 * b + r));
        const int orow = o0 + wave * (32 * RA);
        const bool fast_store = (g.d_out & 3) == 0 && orow + 32 * RA <= g.d_out && !g.acc_out;
        if (fast_store) {
            constexpr int LPR = 8 * RA;              // lanes (16 bytes each) per token row
            constexpr int RPI = 64 / LPR;            // token rows per store instruction
            int8_t *const est = lds + RING_BYTES + wave * STG_WAVE;
            const int tokens = g.tokens;
            const int64_t d_out = g.d_out;
            const bool all_tokens = t0 + 32 * TB <= tokens;
            const bool has_bias = g.bias != nullptr;
            v4f bias4 = {0.f, 0.f, 0.f, 0.f};
            if (has_bias) bias4 = *reinterpret_cast<const v4f *>(g.bias + orow + 4 * (lane % LPR));
            float *const ybase = g.Y + (int64_t)(t0 + lane / LPR) * d_out + orow + 4 * (lane % LPR);
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                const float scale = __fdiv_rn(sxv[TB], sxv[b]);
#pragma unroll
                for (int half = 0; half < 32 / STG_TOKENS; ++half) {
                    // the lanes that hold tokens 16 half .. + 15 of the tile stage their 32 values
                    if ((r >> 4) == half) {
#pragma unroll
                        for (int a = 0; a < RA; ++a)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const v4f y = {(float)acc[a][b][4 * q + 0] * scale, (float)acc[a][b][4 * q + 1] * scale,
                                               (float)acc[a][b][4 * q + 2] * scale, (float)acc[a][b][4 * q + 3] * scale};
                                *reinterpret_cast<v4f *>(est + (r & 15) * EROW + (32 * a + 8 * q + 4 * c) * 4) = y;
                            }
                    }
                    asm volatile("" ::: "memory");   // the reads below are of what the lanes above have just written
                    // the wavefront reads back what it wrote itself (its LDS operations complete in order):
                    // all reads of the pass first, then the stores, so that the LDS latency is paid once
                    v4f yv[STG_TOKENS / RPI];
#pragma unroll
                    for (int j = 0; j < STG_TOKENS / RPI; ++j)
                        yv[j] = *reinterpret_cast<const v4f *>(est + (RPI * j + lane / LPR) * EROW + (lane % LPR) * 16);
#pragma unroll
                    for (int j = 0; j < STG_TOKENS / RPI; ++j) {
                        if (has_bias) yv[j] += bias4;
                        const int trow = 32 * b + STG_TOKENS * half + RPI * j;
                        if (all_tokens || t0 + trow + lane / LPR < tokens)
                            __builtin_nontemporal_store(yv[j], reinterpret_cast<v4f *>(ybase + (int64_t)trow * d_out));
                    }
                    asm volatile("" ::: "memory");   // the next pass overwrites the staging area only after these reads
                }
            }
        } else if (orow < g.d_out) {
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                const int t = t0 + 32 * b + r;
#pragma unroll
                for (int a = 0; a < RA; ++a) store_tile(g, acc[a][b], orow + 32 * a + 4 * c, t, __fdiv_rn(sxv[TB], sxv[b]));
            }
        }
    }
}

template <int TB, bool DENSE, class Group>
__device__ __forceinline__ void piece_live(const Group &grp, const Piece &p, const Piece &next, int8_t *lds, int wave, int lane)
{
    const bool live = p.to * ROWS + wave * (32 * RA) < grp.g[p.prob].d_out;   // a ragged last row tile leaves whole wavefronts idle
    if (live) piece_body<TB, true, DENSE>(grp, p, next, lds, wave, lane);
    else piece_body<TB, false, DENSE>(grp, p, next, lds, wave, lane);
}

template <bool DENSE, class Group>
__device__ __forceinline__ void piece_run(const Group &grp, const Piece &p, const Piece &next, int8_t *lds, int wave, int lane)
{
    if (p.tb == 4) piece_live<4, DENSE>(grp, p, next, lds, wave, lane);
    else if (p.tb == 3) piece_live<3, DENSE>(grp, p, next, lds, wave, lane);
    else if (p.tb == 2) piece_live<2, DENSE>(grp, p, next, lds, wave, lane);
    else piece_live<1, DENSE>(grp, p, next, lds, wave, lane);
}

}  // namespace sp

// The work of a launch is counted in units of 512 rows x 32 tokens.  Blocks go round-robin to the 8 XCDs (each with
// its own 4 MB L2); XCD x owns the token units [x, x + 1) * ceil(units / 8) of every problem, cut into groups of 16
// units (512 tokens: their int8 activations stay in its L2 while the packed weights stream through once per group).
// A strip = (problem, group, row tile).  Launches small enough for a work list (made on the host, see
// make_piece_table) run the pieces listed for each block; larger ones give every block of an XCD a consecutive run of
// the XCD's units in the order strip, unit (the same number of units each, +-1), cut into pieces of at most four units
// that do not cross a strip.
// DENSE = the weights are dense 2-bit codes (the stored form of N = M, or any pattern converted to it) instead of 2:4.
template <bool DENSE, class Group, class Table>
__global__ void __launch_bounds__(64 * sp::NW) gemm_smfmac_kernel(Group grp, Table tab)
{
    __shared__ __attribute__((aligned(1024))) int8_t lds[sp::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const sp::Piece none{0, 0, 0, 0, 0};
    if constexpr (sizeof(Table) == sizeof(PieceTableNone)) {
        // Decode batches (every problem at most 16 token units): a piece = (problem, row tile, a share of the token
        // units of at most tab.piece[0] = 4, 2 or 1: the widest that still gives every multiprocessor a piece), in that
        // order, -per_block pieces in all; block b runs a contiguous run of them, so the pieces of a row tile that has
        // more than one follow each other on one multiprocessor while its weights are still in L2.  Dealing token
        // units to XCDs, as below, would leave most XCDs without work here.
        const int P = -tab.per_block, nbk = (int)gridDim.x, b = (int)blockIdx.x, wmax = (int)tab.piece[0];
        const int q = P / nbk, rem = P % nbk;
        int f = b * q + (b < rem ? b : rem);
        const int end = f + q + (b < rem ? 1 : 0);
        int prob = 0, base = 0, parity = 0;
        auto piece_at = [&](int &f) {
            if (f >= end) return none;
            int units, groups;
            for (;;) {
                units = (grp.g[prob].tokens + 31) >> 5;
                groups = (units + wmax - 1) / wmax;
                const int cnt = ((grp.g[prob].d_out + sp::ROWS - 1) / sp::ROWS) * groups;
                if (f < base + cnt) break;
                base += cnt;
                ++prob;
            }
            const int local = f - base, to = local / groups, g = local % groups;
            const int wide = units / groups, more = units % groups;   // the first `more` shares hold one unit more
            ++f;
            parity ^= 1;
            return sp::Piece{prob, to, (g * wide + (g < more ? g : more)) * 32, wide + (g < more ? 1 : 0), parity};
        };
        sp::Piece cur = piece_at(f);
        if (cur.tb == 0) return;
        sp::piece_prologue(grp, cur, lds, wave, lane);
        while (cur.tb > 0) {
            const sp::Piece next = piece_at(f);
            sp::piece_run<DENSE>(grp, cur, next, lds, wave, lane);
            cur = next;
        }
        return;
    } else {
    if (tab.per_block > 0) {
        auto decode = [&](int i) {
            if (i >= tab.per_block) return none;
            const uint32_t pc = tab.piece[blockIdx.x * tab.per_block + i];
            return sp::Piece{(int)(pc >> 25), (int)((pc >> 16) & 0x1ff), (int)((pc >> 3) & 0x1fff) * 32, (int)(pc & 7), i & 1};
        };
        // the pieces of a block are listed without gaps: the first empty entry ends the list
        sp::Piece cur = decode(0);
        if (cur.tb == 0) return;
        sp::piece_prologue(grp, cur, lds, wave, lane);
        for (int i = 1; cur.tb > 0; ++i) {
            const sp::Piece next = decode(i);
            sp::piece_run<DENSE>(grp, cur, next, lds, wave, lane);
            cur = next;
        }
        return;
    }
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3, nb = gridDim.x >> 3;
    constexpr int GROUP_UNITS = 16;
    // units of problem p that XCD x owns: [x * upx, min((x + 1) * upx, units)), upx = ceil(units / 8)
    auto own_units = [&](int p, int &first) {
        const int units = (grp.g[p].tokens + 31) >> 5, upx = (units + 7) >> 3;
        first = x * upx;
        const int n = units - first;
        return n < 0 ? 0 : n < upx ? n : upx;
    };
    int total = 0;
    for (int p = 0; p < grp.count; ++p) {
        int first;
        total += (int)((grp.g[p].d_out + sp::ROWS - 1) / sp::ROWS) * own_units(p, first);
    }
    const int q = total / nb, rem = total % nb;
    int f = j * q + (j < rem ? j : rem);
    const int end = f + q + (j < rem ? 1 : 0);
    int prob = 0, group = 0, base = 0, parity = 0;
    // the piece that starts at flat unit f (f only grows, so the search for its strip resumes where it stopped)
    auto piece_at = [&](int &f) {
        if (f >= end) return none;
        int first, n, gsz, tiles_o;
        for (;;) {
            n = own_units(prob, first);
            tiles_o = (grp.g[prob].d_out + sp::ROWS - 1) / sp::ROWS;
            gsz = n - group * GROUP_UNITS;
            gsz = gsz > GROUP_UNITS ? GROUP_UNITS : gsz;
            const int cnt = gsz > 0 ? tiles_o * gsz : 0;
            if (gsz > 0 && f < base + cnt) break;
            base += cnt;
            if (gsz <= 0 || (group + 1) * GROUP_UNITS >= n) { ++prob; group = 0; } else ++group;
        }
        const int local = f - base;
        const int to = local / gsz, u = local % gsz;
        int w = gsz - u;
        w = w > 4 ? 4 : w;
        w = w > end - f ? end - f : w;
        f += w;
        parity ^= 1;
        return sp::Piece{prob, to, (first + group * GROUP_UNITS + u) * 32, w, parity};
    };
    sp::Piece cur = piece_at(f);
    if (cur.tb == 0) return;
    sp::piece_prologue(grp, cur, lds, wave, lane);
    while (cur.tb > 0) {
        const sp::Piece next = piece_at(f);
        sp::piece_run<DENSE>(grp, cur, next, lds, wave, lane);
        cur = next;
    }
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

// Same block and wave shapes as the sparse kernel and the same LDS-DMA machinery, so that the two
// paths differ only in what the matrix instruction is fed: dense int8 rows with explicit zeros
// (no index register, no code expansion) into v_mfma_i32_32x32x32_i8, twice as many of them.
// Stage = 64 k of the 256 weight rows and 128 token rows (64-byte rows, 24 KB), ring of 3 stages;
// one DMA instruction fills 16 rows, 16-byte granules swizzled with (row >> 2) & 3.
constexpr int STAGES = 3;
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

// Deals the work of a launch to the blocks (host side).  Per XCD: the strips (problem, token group of 16 units, row
// tile of 512) are cut into exactly m * nb pieces of at most four units, as even as the strip lengths allow (no block
// is left with single-unit crumbs: a piece of one unit pays nine vector instructions per matrix instruction).  The
// pieces stay in strip order and are dealt in m rounds of nb: the pieces that run at about the same time belong to a
// few neighbouring strips, whose weights and tokens fit the XCD's L2 together (dealt by width alone, across all strips,
// the same launch fetched 88 MB instead of 50 at 6912 x 2560 x 4096).  Inside a round the widest pieces go to the
// blocks with the least work so far, so every block ends up with the same number of units (+-1).  Odd XCDs run their
// rounds in reverse order, so that the chip's XCDs do not all reach their epilogues (bursts of Y stores) together.
// Returns blocks per XCD; leaves tab.per_block = 0 (formula split in the kernel) when the list would not fit.
static int make_piece_table(const GemmGroup &grp, PieceTable &tab)
{
    constexpr int GROUP_UNITS = 16;
    struct Strip { int prob, to, unit0, len, npieces; };
    static thread_local std::vector<Strip> strips;
    static thread_local std::vector<uint32_t> pieces;
    static thread_local std::vector<std::vector<uint32_t>> per_block;
    int nb = device_cus() / 8;
    nb = nb < 1 ? 1 : nb;
    int most = 0;   // units of the XCD with the most work
    for (int x = 0; x < 8; ++x) {
        int total = 0;
        for (int p = 0; p < grp.count; ++p) {
            const int units = (grp.g[p].tokens + 31) / 32, upx = (units + 7) / 8;
            const int n = units - x * upx;
            total += (int)ceil_div(grp.g[p].d_out, sp::ROWS) * (n < 0 ? 0 : n < upx ? n : upx);
        }
        most = total > most ? total : most;
    }
    nb = most < nb ? most : nb;
    nb = nb < 1 ? 1 : nb;
    const int m = (int)ceil_div(ceil_div(most, nb), 4);   // pieces per block: the busiest XCD's units per block, four at a time
    tab.per_block = 0;
    if (m * nb * 8 > PIECE_TABLE_MAX) return nb;
    for (int i = 0; i < m * nb * 8; ++i) tab.piece[i] = 0;
    per_block.resize(nb);
    for (int x = 0; x < 8; ++x) {
        strips.clear();
        int minpieces = 0;
        for (int p = 0; p < grp.count; ++p) {
            const int units = (grp.g[p].tokens + 31) / 32, upx = (units + 7) / 8;
            int n = units - x * upx;
            n = n < 0 ? 0 : n < upx ? n : upx;
            const int tiles_o = (int)ceil_div(grp.g[p].d_out, sp::ROWS);
            for (int g0 = 0; g0 < n; g0 += GROUP_UNITS)
                for (int to = 0; to < tiles_o; ++to) {
                    const int len = n - g0 < GROUP_UNITS ? n - g0 : GROUP_UNITS;
                    strips.push_back(Strip{p, to, x * upx + g0, len, (len + 3) / 4});
                    minpieces += (len + 3) / 4;
                }
        }
        if (strips.empty()) continue;
        // more pieces than the minimum: cut the strips with the widest pieces finer, one more piece at a time
        int extra = m * nb - minpieces;
        while (extra > 0) {
            int best = -1;
            for (size_t i = 0; i < strips.size(); ++i)
                if (strips[i].npieces < strips[i].len &&
                    (best < 0 || strips[i].len * strips[best].npieces > strips[best].len * strips[i].npieces))
                    best = (int)i;
            if (best < 0) break;
            ++strips[best].npieces;
            --extra;
        }
        pieces.clear();
        for (const Strip &st : strips) {
            int u = 0;
            for (int k = 0; k < st.npieces; ++k) {
                const int w = st.len / st.npieces + (k < st.len % st.npieces ? 1 : 0);
                pieces.push_back((uint32_t)w | ((uint32_t)(st.unit0 + u) << 3) | ((uint32_t)st.to << 16) | ((uint32_t)st.prob << 25));
                u += w;
            }
        }
        // Pieces stay in strip order: round i (the i-th piece of every block, roughly the same stretch of time) takes
        // the pieces [i * nb, (i + 1) * nb), i.e. a few neighbouring strips whose weights and tokens fit the XCD's L2
        // together.  Inside a round the widest pieces go to the blocks with the least work so far.
        for (int j = 0; j < nb; ++j) per_block[j].clear();
        static thread_local std::vector<int> load, by_load, by_width;
        load.assign(nb, 0);
        const int rounds = ((int)pieces.size() + nb - 1) / nb;
        if (rounds > m) return nb;   // cannot happen: the strips were cut into at most m * nb pieces
        for (int i = 0; i < rounds; ++i) {
            const int first = i * nb, n = (int)pieces.size() - first < nb ? (int)pieces.size() - first : nb;
            by_width.resize(n);
            for (int k = 0; k < n; ++k) by_width[k] = first + k;
            std::stable_sort(by_width.begin(), by_width.end(), [&](int a, int b) { return (pieces[a] & 7) > (pieces[b] & 7); });
            by_load.resize(nb);
            for (int j = 0; j < nb; ++j) by_load[j] = j;
            std::stable_sort(by_load.begin(), by_load.end(), [&](int a, int b) { return load[a] < load[b]; });
            for (int k = 0; k < n; ++k) {
                per_block[by_load[k]].push_back(pieces[by_width[k]]);
                load[by_load[k]] += (int)(pieces[by_width[k]] & 7);
            }
        }
        for (int j = 0; j < nb; ++j) {
            std::vector<uint32_t> &l = per_block[j];
            if (x & 1) std::reverse(l.begin(), l.end());   // odd XCDs run their rounds last to first
            for (size_t i = 0; i < l.size(); ++i) tab.piece[(size_t)(j * 8 + x) * m + i] = l[i];
        }
    }
    tab.per_block = m;
    return nb;
}

sbn_status launch_gemm_smfmac(int count, const LinearItem *items, bool dense_codes, hipStream_t stream)
{
    // problems of at most 16 token units (512 tokens: decode batches) are dealt by row tile, up to GEMM_GROUP_WIDE per launch
    // (2: at most 64 tokens and nothing but Y asked for: the streaming kernel for decode batches.  Also for a single
    // layer: with weights that come from HBM it measured 13.8 / 23.5 us at 32 tokens against 19.6 / 43.8 us on the
    // pieces below, 6912 x 2560 / 2560 x 6912; a piece streams its 512 rows through one multiprocessor's shallow ring)
    auto few_tokens = [&](int i) { return gemv_batch_takes(items[i]) ? 2 : items[i].tokens <= 16 * 32 ? 1 : 0; };
    for (int first = 0; first < count;) {
        const int few = few_tokens(first);
        const int most = few == 2 ? count : few ? GEMM_GROUP_WIDE : GEMM_GROUP_MAX;
        int n = 1;
        while (first + n < count && n < most && few_tokens(first + n) == few) ++n;
        if (few == 2) {
            sbn_status st = launch_gemv_batch(n, items + first, dense_codes, stream);
            if (st != SBN_OK) return st;
            first += n;
            continue;
        }
        if (few) {
            GemmGroupWide grp;
            grp.count = n;
            for (int i = 0; i < n; ++i) grp.g[i] = make_args(items[first + i]);
            // pieces of four token units feed the matrix pipe best; a launch with fewer pieces than multiprocessors (one
            // layer of a decode step) is cut finer, down to single units, so that its latency is that of a small piece
            int wmax = 4, pieces = 0;
            for (;; wmax >>= 1) {
                pieces = 0;
                for (int i = 0; i < n; ++i)
                    pieces += (int)ceil_div(items[first + i].d_out, sp::ROWS) * (int)ceil_div(ceil_div(items[first + i].tokens, 32), wmax);
                if (wmax == 1 || pieces >= device_cus()) break;
            }
            PieceTableNone tab;
            tab.per_block = -pieces;
            tab.piece[0] = (uint32_t)wmax;
            const int blocks = pieces < device_cus() ? pieces : device_cus();
            if (dense_codes) hipLaunchKernelGGL((gemm_smfmac_kernel<true, GemmGroupWide, PieceTableNone>), dim3(blocks), dim3(64 * sp::NW), 0, stream, grp, tab);
            else hipLaunchKernelGGL((gemm_smfmac_kernel<false, GemmGroupWide, PieceTableNone>), dim3(blocks), dim3(64 * sp::NW), 0, stream, grp, tab);
        } else {
            GemmGroup grp;
            grp.count = n;
            for (int i = 0; i < n; ++i) grp.g[i] = make_args(items[first + i]);
            static thread_local PieceTable tab;
            const int per_xcd = make_piece_table(grp, tab);
            if (dense_codes) hipLaunchKernelGGL((gemm_smfmac_kernel<true, GemmGroup, PieceTable>), dim3(8 * per_xcd), dim3(64 * sp::NW), 0, stream, grp, tab);
            else hipLaunchKernelGGL((gemm_smfmac_kernel<false, GemmGroup, PieceTable>), dim3(8 * per_xcd), dim3(64 * sp::NW), 0, stream, grp, tab);
        }
        sbn_status st = check_launch("gemm_smfmac_kernel");
        if (st != SBN_OK) return st;
        first += n;
    }
    return SBN_OK;
}

sbn_status launch_gemm_dense_expanded(const LinearItem &it, const int8_t *w_dense, hipStream_t stream)
{
    GemmArgs g = make_args(it);
    g.w_dense = w_dense;
    hipLaunchKernelGGL(gemm_dense_kernel, dim3(g.tiles_o * g.tiles_t), dim3(256), 0, stream, g);
    return check_launch("gemm_dense_kernel");
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
    return launch_gemm_dense_expanded(it, w_dense, stream);
}

}  // namespace sbn
