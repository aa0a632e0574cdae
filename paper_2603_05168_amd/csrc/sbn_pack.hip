// quantize_mask_pack: absmean scale, N:M magnitude mask, ternary codes, packed layout.
//
// bf16 matrices of whole chunks at 2:4, 1:4 or 2:8 take the single-read form: one persistent kernel
// (pack_stream_kernel, after a small clear of its counters) whose blocks keep units of 16384 weights
// in registers between the |w| sum and the packing (ranked and compacted while they wait for the
// threshold), so that W crosses HBM once.
// Everything else takes three enqueues per batch of up to PACK_MAX_ITEMS matrices:
//   1. absmean_partial_kernel  one block per 16384 weights, |w| summed in fp64 (every term exact)
//   2. absmean_finalize_kernel one block per matrix: fixed-order sum of the partials, gamma and
//                              the rounding threshold theta
//   3. pack_kernel             one block per 16 chunks (2048 weights): top-N per group, ternary
//                              codes, fields assembled in LDS, one coalesced store
// Section 2.1 (ternary quantizer), Section 2.2 (mask from latent weights, quantize then mask),
// Section 2.3 (the mask is recomputed every step, so this is a hot kernel).
#include <cstdlib>

#include "sbn_internal.hpp"

namespace sbn {

namespace {

struct PackTable {
    PackItem it[PACK_MAX_ITEMS];
    int sum_block0[PACK_MAX_ITEMS + 1];   // first absmean block of each matrix
    int pack_block0[PACK_MAX_ITEMS + 1];  // first pack block of each matrix
    int count;
};

// problem a block belongs to: largest i with prefix[i] <= block (binary search, scalar loads)
__device__ __forceinline__ int find_item(const int *prefix, int count, int block)
{
    int lo = 0, hi = count;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (block >= prefix[mid]) lo = mid; else hi = mid;
    }
    return lo;
}

// raw bits of one latent weight; magnitude compare happens on the integer pattern, which orders
// finite IEEE magnitudes exactly as the floats (and makes -0 tie with +0)
template <typename WT> struct Raw;
template <> struct Raw<float> {
    static constexpr uint32_t MAG = 0x7fffffffu;
    static constexpr int SIGN_SHIFT = 31;
    __device__ static uint32_t load(const float *p) { return __float_as_uint(*p); }
    __device__ static double abs_value(uint32_t raw) { return (double)__uint_as_float(raw & MAG); }
    __device__ static uint32_t threshold(float theta) { return __float_as_uint(theta); }
};
template <> struct Raw<uint16_t> {  // bf16
    static constexpr uint32_t MAG = 0x7fffu;
    static constexpr int SIGN_SHIFT = 15;
    __device__ static uint32_t load(const uint16_t *p) { return *p; }
    __device__ static double abs_value(uint32_t raw) { return (double)__uint_as_float((raw & MAG) << 16); }
    // smallest bf16 magnitude pattern whose value is >= theta
    __device__ static uint32_t threshold(float theta) { return (__float_as_uint(theta) + 0xffffu) >> 16; }
};

template <typename WT>
__device__ __forceinline__ void load8(const WT *p, bool vec, bool valid8, const bool valid[8], uint32_t raw[8])
{
    if (vec && valid8) {
        if constexpr (sizeof(WT) == 2) {
            uint4 v = *reinterpret_cast<const uint4 *>(p);
            raw[0] = v.x & 0xffffu; raw[1] = v.x >> 16;
            raw[2] = v.y & 0xffffu; raw[3] = v.y >> 16;
            raw[4] = v.z & 0xffffu; raw[5] = v.z >> 16;
            raw[6] = v.w & 0xffffu; raw[7] = v.w >> 16;
        } else {
            uint4 a = reinterpret_cast<const uint4 *>(p)[0];
            uint4 b = reinterpret_cast<const uint4 *>(p)[1];
            raw[0] = a.x; raw[1] = a.y; raw[2] = a.z; raw[3] = a.w;
            raw[4] = b.x; raw[5] = b.y; raw[6] = b.z; raw[7] = b.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) raw[j] = valid[j] ? Raw<WT>::load(p + j) : 0u;
    }
}

__device__ __forceinline__ double block_sum(double v, double *lds)
{
    const int tid = threadIdx.x;
    lds[tid] = v;
    __syncthreads();
#pragma unroll
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) lds[tid] += lds[tid + s];
        __syncthreads();
    }
    return lds[0];
}

// ---- pass 1: partial sums of |w| in fp64 ------------------------------------------------------
template <typename WT>
__global__ void __launch_bounds__(256) absmean_partial_kernel(PackTable tab, double *partials, int vec_ok)
{
    __shared__ double lds[256];
    const int item = find_item(tab.sum_block0, tab.count, blockIdx.x);
    const PackItem &it = tab.it[item];
    const int64_t lb = blockIdx.x - tab.sum_block0[item];
    const int64_t n = it.d_out * it.d_in;
    const WT *W = static_cast<const WT *>(it.W);
    const int64_t e0 = lb * PACK_SUM_ELEMS;
    double acc = 0.0;
    const bool flat = vec_ok && it.ld == it.d_in;
#pragma unroll
    for (int u = 0; u < PACK_SUM_ELEMS / (256 * 8); ++u) {
        const int64_t e = e0 + ((int64_t)u * 256 + threadIdx.x) * 8;
        if (e >= n) break;
        uint32_t raw[8];
        bool valid[8];
        if (flat) {
            // d_in % 8 == 0 here, so a vector never crosses the end of the matrix
            load8<WT>(W + e, true, true, valid, raw);
        } else {
            const WT *p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                valid[j] = e + j < n;
                const int64_t row = (e + j) / it.d_in, col = (e + j) % it.d_in;
                p[j] = W + row * it.ld + col;
                raw[j] = valid[j] ? Raw<WT>::load(p[j]) : 0u;
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += Raw<WT>::abs_value(raw[j]);
    }
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = total;
}

// ---- pass 2: gamma and the rounding threshold --------------------------------------------------
// theta is the smallest fp32 magnitude a with fl32(a / gamma) > 0.5.  Because fl32(a / gamma) is
// monotone in a, clip(round_half_even(w / gamma), -1, 1) != 0  <=>  |w| >= theta, so the pack
// kernel needs one integer compare per weight instead of a division.
// gamma and theta from the fp64 total of |w|
__device__ __forceinline__ float gamma_theta(double total, int64_t count, float &theta)
{
    float g = (float)(total / (double)count);
    g = g < 1e-5f ? 1e-5f : g;
    float a = 0.5f * g;
    while (!(__fdiv_rn(a, g) > 0.5f)) a = __uint_as_float(__float_as_uint(a) + 1u);
    theta = a;
    return g;
}

__global__ void __launch_bounds__(256) absmean_finalize_kernel(PackTable tab, const double *partials, float *theta)
{
    __shared__ double lds[256];
    const int item = blockIdx.x;
    const PackItem &it = tab.it[item];
    const int b0 = tab.sum_block0[item], b1 = tab.sum_block0[item + 1];
    double acc = 0.0;
    for (int b = b0 + threadIdx.x; b < b1; b += 256) acc += partials[b];
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        float a;
        *it.gamma = gamma_theta(total, it.d_out * it.d_in, a);
        theta[item] = a;
    }
}

// ---- pass 3: mask, codes, packed fields --------------------------------------------------------
// keep mask of 8 consecutive weights (8/M whole groups): element j is kept iff fewer than N
// elements of its group beat it, where an equal magnitude at a lower position beats it.
template <int N, int M>
__device__ __forceinline__ uint32_t keep_mask8(const uint32_t mag[8])
{
    if constexpr (N == M) {
        return 0xffu;
    } else {
        uint32_t keep = 0;
#pragma unroll
        for (int g = 0; g < 8 / M; ++g) {
#pragma unroll
            for (int j = 0; j < M; ++j) {
                int beaten = 0;
#pragma unroll
                for (int jj = 0; jj < M; ++jj) {
                    if (jj == j) continue;
                    const uint32_t a = mag[g * M + jj], me = mag[g * M + j];
                    beaten += (jj < j) ? (a >= me) : (a > me);
                }
                keep |= (uint32_t)(beaten < N) << (g * M + j);
            }
        }
        return keep;
    }
}

__device__ __forceinline__ void lds_or_merge(uint32_t *lds, int &cur_word, uint32_t &cur_bits, int word, uint32_t bits)
{
    if (word != cur_word) {
        if (cur_bits) atomicOr(&lds[cur_word], cur_bits);
        cur_word = word;
        cur_bits = 0;
    }
    cur_bits |= bits;
}

template <typename WT, int N, int M>
__global__ void __launch_bounds__(256) pack_kernel(PackTable tab, const float *theta, int vec_ok)
{
    constexpr int B = (N == M) ? 0 : (M == 2 ? 1 : M == 4 ? 2 : 3);
    constexpr int SLOTS = 128 * N / M;
    constexpr int IDX_BYTES = SLOTS * B / 8;
    constexpr int CB = IDX_BYTES + SLOTS / 4;   // chunk bytes
    constexpr int CNT = 8 * N / M;              // slots produced by one lane (8 weights)
    constexpr int LDS_WORDS = (16 * CB + 3) / 4 + 1;
    __shared__ uint32_t lds[LDS_WORDS];

    const int item = find_item(tab.pack_block0, tab.count, blockIdx.x);
    const PackItem &it = tab.it[item];
    const int64_t lb = blockIdx.x - tab.pack_block0[item];
    const int64_t nchunks = (it.d_in + CHUNK - 1) / CHUNK;
    const int64_t total_chunks = it.d_out * nchunks;
    const int tid = threadIdx.x;
    const int ql = tid >> 4;    // chunk within the block
    const int lane16 = tid & 15;  // 8-weight vector within the chunk
    const int64_t q = lb * 16 + ql;

    for (int w = tid; w < LDS_WORDS; w += 256) lds[w] = 0;
    __syncthreads();

    if (q < total_chunks) {
        const WT *W = static_cast<const WT *>(it.W);
        int64_t row, col;
        if (it.ld == it.d_in && (it.d_in % CHUNK) == 0) {
            row = 0;
            col = q * CHUNK + lane16 * 8;   // flat offset: rows are contiguous and chunk-aligned
        } else {
            row = q / nchunks;
            col = (q % nchunks) * CHUNK + lane16 * 8;
        }
        const int64_t row_end = (it.ld == it.d_in && (it.d_in % CHUNK) == 0) ? it.d_out * it.d_in : it.d_in;
        bool valid[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) valid[j] = col + j < row_end;
        uint32_t raw[8];
        load8<WT>(W + row * it.ld + col, vec_ok != 0, col + 8 <= row_end, valid, raw);

        const uint32_t th = Raw<WT>::threshold(theta[item]);
        uint32_t mag[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) mag[j] = raw[j] & Raw<WT>::MAG;
        const uint32_t keep = keep_mask8<N, M>(mag);

        // this lane's slots are s0 .. s0 + CNT - 1 of the chunk
        const int s0 = lane16 * CNT;
        const int idx_bit0 = ql * CB * 8;
        const int code_bit0 = (ql * CB + IDX_BYTES) * 8;
        int iw = -1, cw = -1;
        uint32_t ibits = 0, cbits = 0;
        int s = s0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if ((keep >> j) & 1u) {
                if constexpr (B > 0) {
                    const uint32_t pos_in_group = j % M;
                    const int p = idx_bit0 + s * B;
                    lds_or_merge(lds, iw, ibits, p >> 5, pos_in_group << (p & 31));
                    if ((p & 31) + B > 32)
                        lds_or_merge(lds, iw, ibits, (p >> 5) + 1, pos_in_group >> (32 - (p & 31)));
                }
                const uint32_t nz = mag[j] >= th;
                const uint32_t sign = (raw[j] >> Raw<WT>::SIGN_SHIFT) & 1u;
                const uint32_t code = nz ? (sign ? 3u : 1u) : 0u;
                const int v = s & 15;
                const int p = code_bit0 + 32 * (s >> 4) + 8 * (v & 3) + 2 * (v >> 2);
                lds_or_merge(lds, cw, cbits, p >> 5, code << (p & 31));
                ++s;
            }
        }
        if (ibits) atomicOr(&lds[iw], ibits);
        if (cbits) atomicOr(&lds[cw], cbits);
    }
    __syncthreads();

    // coalesced store of the block's chunks
    const int64_t chunks_here = (total_chunks - lb * 16) < 16 ? (total_chunks - lb * 16) : 16;
    const int bytes_here = (int)chunks_here * CB;
    uint8_t *out = it.packed + lb * 16 * CB;
    for (int w = tid; w * 4 < bytes_here; w += 256) {
        if (w * 4 + 4 <= bytes_here) {
            reinterpret_cast<uint32_t *>(out)[w] = lds[w];
        } else {
            for (int k = w * 4; k < bytes_here; ++k) out[k] = (uint8_t)(lds[w] >> (8 * (k & 3)));
        }
    }
}

// ---- fast pack kernels: bf16, rows contiguous, d_in % 128 == 0, patterns 2:4, 1:4, 2:8 ----------------
// A lane owns 8 consecutive weights (one 16-byte load).  Selection runs on integer keys
//     magnitude << 17 | (M - 1 - position in the group) << 2 | 1 << 1 | sign
// which are unique within a group, and the larger key is the larger magnitude or, among equals, the lower
// position, so max/min networks give the top-N with the tie rule built in.  A key is one rotation of the
// dword that holds its bf16 value (the magnitude lands in bits [17, 32), the sign in bit 0) plus one
// mask-and-or.  magnitude >= threshold is key >= threshold << 17, and the low two bits of a key, swapped,
// are the ternary code of its element when that element is nonzero (01 = +1, 11 = -1), so a selected
// key needs no look-up for its code.
// The words of a chunk are OR-reduced across lanes with DPP (a DPP row = 16 lanes = one chunk), the
// group leaders drop them into LDS, and the block stores its chunks with 16 bytes per thread.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_or_t(uint32_t x)
{
    return x | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}
// OR over aligned groups of 4, 8 or 16 lanes; every lane of the group ends with the result
template <int LANES> __device__ __forceinline__ uint32_t group_or(uint32_t x)
{
    x = dpp_or_t<0xB1>(x);                              // quad_perm [1,0,3,2]
    x = dpp_or_t<0x4E>(x);                              // quad_perm [2,3,0,1]
    if constexpr (LANES >= 8) x = dpp_or_t<0x141>(x);   // row_half_mirror: quad 0 <-> 1, 2 <-> 3
    if constexpr (LANES >= 16) x = dpp_or_t<0x140>(x);  // row_mirror: half 0 <-> 1
    return x;
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

template <int M> struct PackKey {
    static constexpr int SH = 17;                               // magnitude shift
    static constexpr uint32_t KEEP = 0xfffe0001u;               // magnitude and sign of a rotated dword
    static constexpr uint32_t POS = (uint32_t)(M - 1) << 2;     // position field
};

// keys of the eight bf16 values of a vector (four dwords, two values each)
template <int M>
__device__ __forceinline__ void make_keys(const uint4 &v, uint32_t (&key)[8])
{
    typedef PackKey<M> PK;
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t clo = ((uint32_t)(M - 1 - (2 * i) % M) << 2) | 2u, chi = ((uint32_t)(M - 1 - (2 * i + 1) % M) << 2) | 2u;
        key[2 * i] = (__builtin_rotateleft32(d[i], 17) & PK::KEEP) | clo;      // low half: magnitude bits [0, 15), sign bit 15
        key[2 * i + 1] = (__builtin_rotateleft32(d[i], 1) & PK::KEEP) | chi;   // high half: magnitude bits [16, 31), sign bit 31
    }
}

// the bf16 pattern (sign and magnitude) behind a key, in the low (raw_lo) or high (raw_hi) half of a dword
__device__ __forceinline__ uint32_t pair_of_keys(uint32_t klo, uint32_t khi)
{
    const uint32_t lo = __builtin_rotateleft32(klo, 15), hi = __builtin_rotateleft32(khi, 31);
    return (lo & 0xffffu) | (hi & 0xffff0000u);
}

// ternary codes of the two bf16 patterns of a dword, at bits [0, 2) and [16, 18): nonzero iff magnitude >=
// threshold, i.e. iff magnitude - (threshold - 1) does not saturate to 0.  thm1x2 = threshold - 1 in both halves.
__device__ __forceinline__ uint32_t pair_codes(uint32_t p, uint32_t thm1x2)
{
    // packed 16-bit saturating subtract and minimum, written out: the compiler splits the vector form into
    // two 16-bit compares and selects
    uint32_t over, nz;
    asm("v_pk_sub_u16 %0, %1, %2 clamp" : "=v"(over) : "v"(p & 0x7fff7fffu), "v"(thm1x2));
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(nz) : "v"(over), "v"(0x00010001u));
    return (((p >> 15) & nz) << 1) | nz;
}

struct Top2 { uint32_t first, second; };
// largest and second largest of four unique keys
__device__ __forceinline__ Top2 top2_of4(uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3)
{
    const uint32_t h01 = umax(k0, k1), l01 = umin(k0, k1), h23 = umax(k2, k3), l23 = umin(k2, k3);
    Top2 t;
    t.first = umax(h01, h23);
    t.second = umax(umin(h01, h23), umax(l01, l23));
    return t;
}

// the two keys ordered by position: lower position (= larger position field) first
template <int M>
__device__ __forceinline__ void by_position(const Top2 &t, uint32_t &klo, uint32_t &khi)
{
    const bool first_lo = (t.first & PackKey<M>::POS) > (t.second & PackKey<M>::POS);
    klo = first_lo ? t.first : t.second;
    khi = first_lo ? t.second : t.first;
}

// What the blocks of the single-read form share through the workspace: the partial sums (one slot per
// unit, preset to a pattern no sum can have, so that a slot's value is also the sign that the unit has
// arrived) and, per matrix, 32 ready words (unit lb polls word lb % 32: same-address device-scope accesses
// serialise, a single word per matrix cost 40 % of the sweep).  Every ready word has a 64-byte line of its own.
constexpr int PACK_SYNC_GROUPS = 32;
constexpr int PACK_SYNC_STRIDE = 16;                                       // words between two ready words
constexpr int PACK_SYNC_WORDS = PACK_SYNC_STRIDE * PACK_SYNC_GROUPS;       // per matrix
constexpr unsigned long long PACK_NO_PARTIAL = ~0ull;                      // a NaN pattern: sums of |w| are finite
struct PackSync {
    double *partials;     // one per block, as in the absmean pass
    float *theta;         // one per matrix
    unsigned *words;      // PACK_SYNC_WORDS per matrix, cleared before the launch (the partials are preset with them)
    int spin_limit;       // polls a block spends waiting for its ready word before it derives theta on its own
    uint32_t *unit_flips;  // when the launch counts mask flips: one slot per unit of the launch (every slot is written), else null
};
static_assert(sizeof(PackTable) + sizeof(PackSync) <= 4096, "both travel as kernel arguments");

constexpr int PACK_U = 8;   // 16-byte vectors per thread: a unit = 256 threads x 8 vectors = 128 chunks = 16384 weights

// the unit's weights into registers: thread (ql = tid / 16, l16 = tid % 16) takes vector l16 of chunk 16 u + ql
__device__ __forceinline__ void load_unit(const PackItem &it, int64_t lb, uint4 (&v)[PACK_U])
{
    const int64_t total_chunks = it.d_out * (it.d_in / CHUNK);
    const uint16_t *W = static_cast<const uint16_t *>(it.W);
    const int ql = threadIdx.x >> 4, l16 = threadIdx.x & 15;
#pragma unroll
    for (int u = 0; u < PACK_U; ++u) {
        const int64_t q = (lb * PACK_U + u) * 16 + ql;
        v[u] = q < total_chunks ? *reinterpret_cast<const uint4 *>(W + q * CHUNK + l16 * 8) : make_uint4(0, 0, 0, 0);
    }
}

// |w| of the eight bf16 values of a vector added to acc in element order (the order of the absmean pass)
__device__ __forceinline__ double abs8(const uint4 &d, double acc)
{
    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        // a bf16 value is the fp32 value with the same upper half; the absolute value is an operand modifier
        acc += (double)fabsf(__uint_as_float(w[k] << 16));
        acc += (double)fabsf(__uint_as_float(w[k] & 0xffff0000u));
    }
    return acc;
}

// What is left of a unit once its groups have been ranked, which needs no threshold: the bf16 patterns of
// the kept values, two per dword in position order, and one byte of index bits per vector (as they go into
// the index field).  18, 10 and 10 registers per thread for 2:4, 1:4 and 2:8 against 32 for the weights.
template <int N, int M> struct PackCompact {
    static constexpr int SEL = (N == 2 && M == 4) ? 2 * PACK_U : PACK_U;
    uint32_t sel[SEL];
    uint32_t idx[PACK_U / 4];
};

template <int N, int M>
__device__ __forceinline__ void select_unit(const uint4 (&v)[PACK_U], PackCompact<N, M> &c)
{
#pragma unroll
    for (int w = 0; w < PACK_U / 4; ++w) c.idx[w] = 0;
#pragma unroll
    for (int u = 0; u < PACK_U; ++u) {
        uint32_t key[8];
        make_keys<M>(v[u], key);
        uint32_t idxb;
        // position fields hold M - 1 - position: the index bits are inverted once they are assembled
        if constexpr (N == 2 && M == 4) {
            uint32_t klo[2], khi[2];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                by_position<M>(top2_of4(key[4 * g], key[4 * g + 1], key[4 * g + 2], key[4 * g + 3]), klo[g], khi[g]);
                c.sel[2 * u + g] = pair_of_keys(klo[g], khi[g]);
            }
            const uint32_t n0 = ((klo[0] >> 2) & 3u) | (khi[0] & 0xcu), n1 = ((klo[1] >> 2) & 3u) | (khi[1] & 0xcu);
            idxb = (n0 | (n1 << 4)) ^ 0xffu;
        } else if constexpr (N == 1 && M == 4) {
            const uint32_t t0 = umax(umax(key[0], key[1]), umax(key[2], key[3]));
            const uint32_t t1 = umax(umax(key[4], key[5]), umax(key[6], key[7]));
            c.sel[u] = pair_of_keys(t0, t1);
            idxb = (((t0 >> 2) & 3u) | (t1 & 0xcu)) ^ 0xfu;
        } else {   // 2:8
            const Top2 ta = top2_of4(key[0], key[1], key[2], key[3]);
            const Top2 tb = top2_of4(key[4], key[5], key[6], key[7]);
            Top2 t;
            t.first = umax(ta.first, tb.first);
            t.second = umax(umin(ta.first, tb.first), umax(ta.second, tb.second));
            uint32_t klo, khi;
            by_position<M>(t, klo, khi);
            c.sel[u] = pair_of_keys(klo, khi);
            idxb = (((klo >> 2) & 7u) | ((khi & 0x1cu) << 1)) ^ 0x3fu;   // two 3-bit positions
        }
        c.idx[u / 4] |= idxb << (8 * (u % 4));
    }
}

// Mask flips between the index fields of a new and an old packed form (mask flip rate equation of the ablation
// study): positions kept by exactly one of the two.  Both forms keep N positions per group, so a group flips
// 2 * (N - common) positions; the common ones are found by comparing the position fields, all groups of a word at once.
// 2:4, one index word = eight groups (nibble = pos0 | pos1 << 2, pos0 < pos1)
__device__ __forceinline__ uint32_t flips_2of4_word(uint32_t n, uint32_t o)
{
    const uint32_t x = n ^ o;
    const uint32_t same = ~(x | (x >> 1)) & 0x55555555u;                        // pos0 = pos0', pos1 = pos1'
    const uint32_t os = ((o & 0x33333333u) << 2) | ((o >> 2) & 0x33333333u);    // the old positions swapped
    const uint32_t y = n ^ os;
    const uint32_t cross = ~(y | (y >> 1)) & 0x55555555u;                       // pos0 = pos1', pos1 = pos0'
    return 32u - 2u * (uint32_t)(__popc(same) + __popc(cross));
}
// 1:4, one index word = sixteen groups of one 2-bit position
__device__ __forceinline__ uint32_t flips_1of4_word(uint32_t n, uint32_t o)
{
    const uint32_t x = n ^ o;
    return 2u * (uint32_t)__popc((x | (x >> 1)) & 0x55555555u);
}
// 2:8, half an index field = 48 bits = eight groups of two 3-bit positions (pos0 < pos1)
__device__ __forceinline__ uint32_t flips_2of8_half(uint64_t n, uint64_t o)
{
    constexpr uint64_t ONE = 0x249249249249ull;    // bit 0 of every 3-bit field
    constexpr uint64_t EVEN = 0x1c71c71c71c7ull;   // the first field of every group
    const uint64_t x = n ^ o;
    const uint64_t same = ~(x | (x >> 1) | (x >> 2)) & ONE;
    const uint64_t os = ((o & EVEN) << 3) | ((o >> 3) & EVEN);
    const uint64_t y = n ^ os;
    const uint64_t cross = ~(y | (y >> 1) | (y >> 2)) & ONE;
    return 32u - 2u * (uint32_t)(__popcll(same) + __popcll(cross));
}

// Codes of the compact unit with threshold th_val, fields assembled, and its 128 chunks (contiguous in the
// packed buffer) stored.  lds: PACK_U * 16 * CBW words of staging; ends with the block's stores issued, LDS
// free after the next barrier.
// FLIPS: the packed buffer still holds the matrix's previous packed form, which the unit replaces; the return value
// is the number of mask positions that differ between the two in this thread's share of the unit (thread t: half
// t % 2 of the index field of chunk t / 2).  The old index words are asked for first and have arrived before the
// barrier behind which the block's stores begin: no thread overwrites a word another thread has yet to read.
template <int N, int M, bool FLIPS>
__device__ __forceinline__ uint32_t finish_unit(const PackItem &it, const int64_t lb, const PackCompact<N, M> &c, const float th_val,
                                                uint32_t *lds)
{
    constexpr int U = PACK_U;
    constexpr int CBW = (M == 4 && N == 2) ? 8 : (M == 4 ? 4 : 5);   // dwords per chunk: 32, 16, 20 bytes
    const int64_t total_chunks = it.d_out * (it.d_in / CHUNK);
    const int tid = threadIdx.x, ql = tid >> 4, l16 = tid & 15;
    // the block's chunks are contiguous in the packed buffer
    const int64_t chunk0 = lb * U * 16;
    int64_t nch = total_chunks - chunk0;
    nch = nch > U * 16 ? U * 16 : nch;
    uint32_t *dst = reinterpret_cast<uint32_t *>(it.packed) + chunk0 * CBW;
    // index words of the old form: two words per thread (one at 1:4)
    constexpr int FW0 = (M == 4 && N == 2) ? 2 : 1;   // first word of half h is FW0 * h
    const bool fl_on = FLIPS && (tid >> 1) < nch;
    uint32_t old0 = 0, old1 = 0;
    if constexpr (FLIPS) {
        if (fl_on) {
            const uint32_t *po = dst + (tid >> 1) * CBW + FW0 * (tid & 1);
            old0 = po[0];
            if constexpr (!(M == 4 && N == 1)) old1 = po[1];
        }
    }
    // smallest bf16 magnitude pattern whose value is >= theta (at least 1: theta > 0), minus one, in both halves
    const uint32_t thm1x2 = (((__float_as_uint(th_val) + 0xffffu) >> 16) - 1u) * 0x10001u;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t *out = lds + (u * 16 + ql) * CBW;
        const uint32_t idxb = (c.idx[u / 4] >> (8 * (u % 4))) & 0xffu;
        if constexpr (N == 2 && M == 4) {
            // bytes 0 and 2 of each pair's codes -> the four code bytes of the vector
            const uint32_t codeb = __builtin_amdgcn_perm(pair_codes(c.sel[2 * u + 1], thm1x2), pair_codes(c.sel[2 * u], thm1x2), 0x06040200u);
            const int L = l16 & 3;
            const uint32_t idxw = group_or<4>(idxb << (8 * L));
            const uint32_t codew = group_or<4>(codeb << (2 * L));
            if (L == 0) {
                out[l16 >> 2] = idxw;
                out[4 + (l16 >> 2)] = codew;
            }
        } else {
            const uint32_t codeb = __builtin_amdgcn_perm(0u, pair_codes(c.sel[u], thm1x2), 0x0c0c0200u);
            const int L8 = l16 & 7;
            const uint32_t codew = group_or<8>(codeb << (16 * (L8 & 1) + 2 * (L8 >> 1)));
            if constexpr (M == 4) {
                const uint32_t idxw = group_or<8>(idxb << (4 * L8));
                if (L8 == 0) {
                    out[l16 >> 3] = idxw;
                    out[2 + (l16 >> 3)] = codew;
                }
            } else {
                // the pair of positions sits at bit 6 * l16 of the 96-bit index field
                const uint32_t off = 6u * (uint32_t)l16, w0 = off >> 5;
                const uint64_t bits = (uint64_t)idxb << (off & 31u);
                const uint32_t blo = (uint32_t)bits, bhi = (uint32_t)(bits >> 32);
                const uint32_t i0 = group_or<16>(w0 == 0 ? blo : 0u);
                const uint32_t i1 = group_or<16>((w0 == 1 ? blo : 0u) | (w0 == 0 ? bhi : 0u));
                const uint32_t i2 = group_or<16>((w0 == 2 ? blo : 0u) | (w0 == 1 ? bhi : 0u));
                if (l16 == 0) { out[0] = i0; out[1] = i1; out[2] = i2; }
                if (L8 == 0) out[3 + (l16 >> 3)] = codew;
            }
        }
    }
    if constexpr (FLIPS) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the old words are in registers: see above
    __syncthreads();
    uint32_t flips = 0;
    if constexpr (FLIPS) {
        if (fl_on) {
            const uint32_t *pn = lds + (tid >> 1) * CBW + FW0 * (tid & 1);
            if constexpr (M == 4 && N == 2) {
                flips = flips_2of4_word(pn[0], old0) + flips_2of4_word(pn[1], old1);
            } else if constexpr (M == 4) {
                flips = flips_1of4_word(pn[0], old0);
            } else {
                const bool up = tid & 1;   // bits [48, 96) of the field: the upper half of word 1 and word 2
                const uint64_t n48 = up ? (uint64_t)(pn[0] >> 16) | ((uint64_t)pn[1] << 16) : (uint64_t)pn[0] | ((uint64_t)(pn[1] & 0xffffu) << 32);
                const uint64_t o48 = up ? (uint64_t)(old0 >> 16) | ((uint64_t)old1 << 16) : (uint64_t)old0 | ((uint64_t)(old1 & 0xffffu) << 32);
                flips = flips_2of8_half(n48, o48);
            }
        }
    }
    const int ndw = (int)nch * CBW;
    for (int w = tid * 4; w < ndw; w += 1024) {
        if (w + 4 <= ndw) {
            *reinterpret_cast<uint4 *>(dst + w) = *reinterpret_cast<const uint4 *>(lds + w);
        } else {
            for (int k = w; k < ndw; ++k) dst[k] = lds[k];
        }
    }
    return flips;
}

// A unit's flip count goes to the unit's slot in the workspace (wavefront sums through LDS, one plain store), and a
// small kernel behind the pack kernel adds up the slots of every matrix in a fixed order.  One atomic per unit on a
// counter per matrix was tried first: the 145 000 atomics of the 210-matrix sweep queue up at the one L2 channel that
// holds the counters (about 6 ns each) and the sweep took 2.1 ms instead of 1.25.
// flips_wave_sum is called by all threads before the barrier that follows finish_unit, flips_commit after it;
// wave_flips is rewritten only behind the next unit's barriers.
__device__ __forceinline__ void flips_wave_sum(uint32_t flips, uint32_t *wave_flips)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) flips += (uint32_t)__shfl_xor((int)flips, o, 64);
    if ((threadIdx.x & 63) == 0) wave_flips[threadIdx.x >> 6] = flips;
}
__device__ __forceinline__ void flips_commit(const uint32_t *wave_flips, uint32_t *slot)
{
    if (threadIdx.x == 0) *slot = wave_flips[0] + wave_flips[1] + wave_flips[2] + wave_flips[3];
}

// one block per matrix: the flip counts of its units added up
__global__ void __launch_bounds__(256) pack_flips_sum_kernel(PackTable tab, const uint32_t *__restrict__ unit_flips,
                                                             unsigned long long *__restrict__ flips)
{
    __shared__ unsigned long long sums[256];
    const int lo = blockIdx.x;
    unsigned long long acc = 0;
    for (int g = tab.pack_block0[lo] + (int)threadIdx.x; g < tab.pack_block0[lo + 1]; g += 256) acc += unit_flips[g];
    sums[threadIdx.x] = acc;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if ((int)threadIdx.x < step) sums[threadIdx.x] += sums[threadIdx.x + step];
        __syncthreads();
    }
    if (threadIdx.x == 0) flips[lo] = sums[0];
}

// third kernel of the three-pass form: theta comes from the finalize kernel
template <int N, int M, bool FLIPS>
__global__ void __launch_bounds__(256) pack_fast_kernel(PackTable tab, const float *theta, uint32_t *unit_flips)
{
    constexpr int CBW = (M == 4 && N == 2) ? 8 : (M == 4 ? 4 : 5);
    __shared__ __attribute__((aligned(16))) uint32_t lds[PACK_U * 16 * CBW];
    __shared__ uint32_t wave_flips[4];
    const int lo = find_item(tab.pack_block0, tab.count, blockIdx.x);
    const PackItem &it = tab.it[lo];
    const int64_t lb = (int)blockIdx.x - tab.pack_block0[lo];
    uint4 v[PACK_U];
    load_unit(it, lb, v);
    PackCompact<N, M> c;
    select_unit<N, M>(v, c);
    const uint32_t fl = finish_unit<N, M, FLIPS>(it, lb, c, theta[lo], lds);
    if constexpr (FLIPS) {
        flips_wave_sum(fl, wave_flips);
        __syncthreads();
        flips_commit(wave_flips, unit_flips + blockIdx.x);
    }
}

// ---- single-read form ---------------------------------------------------------------------------
// Persistent blocks, as many as the device holds at once.  The units of the batch (16384 weights each,
// matrix after matrix) are dealt round-robin: block b takes units b, b + B, b + 2B, ...  For every unit a
// block loads the weights into registers and publishes their |w| sum (one store, fire and forget); the block
// that holds the matrix's first unit waits until every partial slot of the matrix is filled, adds them in
// the fixed order of the finalize kernel, derives gamma and theta and raises the matrix's ready words
// (they carry theta).  Ranking the groups needs no threshold, so a loaded unit is ranked at once and kept
// in its compact form (the kept values and their index bits: about half the registers); only the codes
// wait for theta.  A block has QD + 1 units in flight: QD compact ones wait for their matrices (the oldest
// is packed next), one more is loaded, summed and published BEFORE the block waits for the oldest - the
// hand-over of a matrix (four device-scope hops of about 1.5 us) runs under the loads of the following
// ones.  The smaller compact form also lets more blocks fit (2:4: six per SIMD instead of five).
// W crosses HBM once.
// Waits always end: a unit's matrix becomes ready once all its units are published; a block publishes
// every unit it holds before it waits, and the units of a matrix (at most as many as there are
// blocks: the host checks) all lie within one deal of the round-robin.  Take the block whose oldest unit
// has the smallest number x: every unit of x's matrix lies below x + B, so the block it belongs to
// already holds it, hence has published it; the same goes for the matrix's first unit, whose block finalizes.
// The wait is bounded all the same (the grid might
// not be fully resident when the device is shared): a block out of polls recomputes every partial of
// the matrix from HBM itself - same arithmetic, same order, same theta - and goes on.
template <int N, int M, int QD, int WAVES, bool FLIPS>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES))) pack_stream_kernel(PackTable tab, PackSync sync)
{
    constexpr int CBW = (M == 4 && N == 2) ? 8 : (M == 4 ? 4 : 5);
    __shared__ __attribute__((aligned(16))) uint32_t lds[PACK_U * 16 * CBW];
    __shared__ uint32_t wave_flips[4];
    __shared__ double red[256];
    __shared__ int role_s;      // 2: waited in vain
    __shared__ float th_s;
    const int tid = threadIdx.x;
    const int total_units = tab.pack_block0[tab.count];
    const int B = (int)gridDim.x;

    struct Unit { int lo; int64_t lb; };
    auto ready_words = [&](int lo) { return sync.words + (int64_t)lo * PACK_SYNC_WORDS; };
    auto unit_of = [&](int g) -> Unit {
        Unit un;
        un.lo = find_item(tab.pack_block0, tab.count, g);
        un.lb = g - tab.pack_block0[un.lo];
        return un;
    };
    // the |w| sum of a loaded unit into its partial slot
    auto publish = [&](const Unit &un, const uint4 (&v)[PACK_U]) {
        double acc = 0.0;
#pragma unroll
        for (int u = 0; u < PACK_U; ++u) acc = abs8(v[u], acc);
        const double mine = block_sum(acc, red);
        unsigned long long *const part_bits = reinterpret_cast<unsigned long long *>(sync.partials + tab.sum_block0[un.lo]);
        // Everything the blocks exchange (partials, ready words) moves through device-scope atomic accesses,
        // which are served where the eight L2s meet.  Release/acquire fences would do the same with a cache
        // write-back or invalidation each, a thousand per matrix (measured: 43 us per matrix).
        if (tid == 0)
            __hip_atomic_store(&part_bits[un.lb], (unsigned long long)__double_as_longlong(mine), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();   // red is free again
    };
    // theta of the unit's matrix: known, or polled from the group's ready word, or recomputed
    // theta of the unit's matrix.  The block that holds the matrix's first unit finalizes it: it waits until
    // every partial slot is filled, adds the partials in the finalize order, writes gamma and raises the
    // ready words; every other block polls its group's ready word.  Out of polls, either kind recomputes the
    // partials from HBM (the finalizing block still publishes the result).
    auto theta_of = [&](const Unit &un) -> float {
        const PackItem &it = tab.it[un.lo];
        const int nblk = tab.pack_block0[un.lo + 1] - tab.pack_block0[un.lo];
        const int ngroups = nblk < PACK_SYNC_GROUPS ? nblk : PACK_SYNC_GROUPS;
        const bool finalizer = un.lb == 0;
        unsigned *const rdy = ready_words(un.lo);
        const unsigned long long *const part_bits =
            reinterpret_cast<const unsigned long long *>(sync.partials + tab.sum_block0[un.lo]);
        if (tid == 0) role_s = 0;
        __syncthreads();
        double a2 = 0.0;   // finalizer: this thread's share of the partials, in the finalize order
        if (finalizer) {
            // a thread's slots are read FIN_BATCH at a time, all loads in flight together (a device-scope load
            // takes about 1.5 us); then the empty ones are polled
            constexpr int FIN_BATCH = 5;
            int spins = 0, ok = sync.spin_limit >= 0;
            for (int b0 = tid; b0 < nblk && ok; b0 += 256 * FIN_BATCH) {
                unsigned long long bits[FIN_BATCH];
#pragma unroll
                for (int j = 0; j < FIN_BATCH; ++j) {
                    const int b = b0 + 256 * j;
                    bits[j] = __hip_atomic_load(&part_bits[b < nblk ? b : b0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int j = 0; j < FIN_BATCH; ++j) {
                    const int b = b0 + 256 * j;
                    if (b >= nblk || !ok) continue;
                    while (bits[j] == PACK_NO_PARTIAL) {
                        if (++spins > sync.spin_limit) { ok = 0; break; }
                        __builtin_amdgcn_s_sleep(4);
                        bits[j] = __hip_atomic_load(&part_bits[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (ok) a2 += __longlong_as_double((long long)bits[j]);   // in the order b = tid, tid + 256, ...
                }
            }
            if (!ok) role_s = 2;   // several threads may write the same value
        } else if (tid == 0) {
            int spins = 0, ok = sync.spin_limit >= 0;
            unsigned word = 0u;
            while (ok && (word = __hip_atomic_load(&rdy[PACK_SYNC_STRIDE * (un.lb % PACK_SYNC_GROUPS)], __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT)) == 0u) {
                if (++spins > sync.spin_limit) ok = 0;
                else __builtin_amdgcn_s_sleep(4);
            }
            if (!ok) role_s = 2;
            th_s = __uint_as_float(word);
        }
        __syncthreads();
        const bool alone = role_s == 2;
        double total = 0.0;
        if (alone) {
            // every partial sum of the matrix from HBM, added up in the finalize order: thread b % 256 takes partial b
            const int64_t total_chunks = it.d_out * (it.d_in / CHUNK);
            const uint16_t *W = static_cast<const uint16_t *>(it.W);
            const int ql = tid >> 4, l16 = tid & 15;
            double a3 = 0.0;
            for (int b = 0; b < nblk; ++b) {
                double pa = 0.0;
#pragma unroll
                for (int u = 0; u < PACK_U; ++u) {
                    const int64_t q = ((int64_t)b * PACK_U + u) * 16 + ql;
                    if (q < total_chunks) pa = abs8(*reinterpret_cast<const uint4 *>(W + q * CHUNK + l16 * 8), pa);
                }
                const double pb = block_sum(pa, red);
                if ((b & 255) == tid) a3 += pb;
                __syncthreads();   // red is reused by the next round
            }
            total = block_sum(a3, red);
        } else if (finalizer) {
            total = block_sum(a2, red);
        }
        if (alone || finalizer) {
            if (tid == 0) {
                float th;
                const float g = gamma_theta(total, it.d_out * it.d_in, th);
                if (finalizer) {
                    *it.gamma = g;
                    sync.theta[un.lo] = th;
                }
                th_s = th;
            }
            __syncthreads();
            // the ready word of a group IS theta (its bit pattern is never zero: theta >= 0.5e-5)
            if (finalizer && tid < ngroups)
                __hip_atomic_store(&rdy[PACK_SYNC_STRIDE * tid], __float_as_uint(th_s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const float th = th_s;
        __syncthreads();   // th_s, role_s and red may be rewritten by what follows
        return th;
    };
    // A block has up to QD + 1 units in flight: the weights of the youngest in registers (loading), the QD
    // older ones ranked and compacted, waiting for their matrices' thresholds; q[0] is the oldest.
    uint4 raw[PACK_U];
    PackCompact<N, M> q[QD];
    Unit uq[QD];
    int queued = 0;
    auto push = [&](const Unit &un) {   // rank the loaded unit and queue it
#pragma unroll
        for (int i = 0; i < QD; ++i)
            if (queued == i) {   // one copy of the ranking code per slot: through a temporary the registers run out
                select_unit<N, M>(raw, q[i]);
                uq[i] = un;
            }
        ++queued;
    };
    int g = (int)blockIdx.x;
    for (int i = 0; i < QD && g < total_units; ++i, g += B) {
        const Unit un = unit_of(g);
        load_unit(tab.it[un.lo], un.lb, raw);
        publish(un, raw);
        push(un);
    }
    while (queued > 0) {
        const bool more = g < total_units;
        Unit un;
        if (more) {   // published before this block waits: no matrix waits for a block that itself waits
            un = unit_of(g);
            load_unit(tab.it[un.lo], un.lb, raw);
            publish(un, raw);
        }
        const float th = theta_of(uq[0]);
        const uint32_t fl = finish_unit<N, M, FLIPS>(tab.it[uq[0].lo], uq[0].lb, q[0], th, lds);
        if constexpr (FLIPS) flips_wave_sum(fl, wave_flips);
        __syncthreads();   // the staging area is free for the next unit
        if constexpr (FLIPS) flips_commit(wave_flips, sync.unit_flips + tab.pack_block0[uq[0].lo] + uq[0].lb);
#pragma unroll
        for (int i = 0; i + 1 < QD; ++i)
            if (i + 1 < queued) {
                q[i] = q[i + 1];
                uq[i] = uq[i + 1];
            }
        --queued;
        if (more) {
            push(un);
            g += B;
        }
    }
}

// ---- test hook: packed -> dense W_eff and mask --------------------------------------------------
__device__ __forceinline__ uint32_t get_bits(const uint8_t *field, int pos, int nbits)
{
    uint32_t v = 0;
    for (int i = 0; i < nbits; ++i) v |= (uint32_t)((field[(pos + i) >> 3] >> ((pos + i) & 7)) & 1u) << i;
    return v;
}

__global__ void __launch_bounds__(256) unpack_kernel(const uint8_t *packed, int64_t d_out, int64_t d_in, Pattern pat,
                                                     int8_t *W_eff, uint8_t *mask)
{
    const int64_t nchunks = (d_in + CHUNK - 1) / CHUNK;
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= d_out * nchunks) return;
    const int64_t row = q / nchunks, c = q % nchunks;
    for (int j = 0; j < CHUNK; ++j) {
        const int64_t col = c * CHUNK + j;
        if (col < d_in) {
            if (W_eff) W_eff[row * d_in + col] = 0;
            if (mask) mask[row * d_in + col] = 0;
        }
    }
    const uint8_t *idx_field = packed + q * pat.chunk_bytes;
    const uint8_t *code_field = idx_field + pat.idx_bytes;
    for (int s = 0; s < pat.slots; ++s) {
        const int g = s / pat.N;
        const int j = pat.b ? (int)get_bits(idx_field, s * pat.b, pat.b) : s % pat.N;
        const int v = s & 15;
        const uint32_t code = get_bits(code_field, 32 * (s >> 4) + 8 * (v & 3) + 2 * (v >> 2), 2);
        const int64_t col = c * CHUNK + g * pat.M + j;
        if (col >= d_in) continue;
        if (mask) mask[row * d_in + col] = 1;
        if (W_eff) W_eff[row * d_in + col] = code == 1u ? 1 : code == 3u ? -1 : 0;
    }
}

// packed -> int8 W_eff with explicit zeros for any pattern, one thread per group of M weights (the
// operand of the dense matrix path for patterns that have no sparse matrix instruction): the N slots
// of the group are decoded into an M-byte word and stored at once
__global__ void __launch_bounds__(256) expand_groups_kernel(const uint8_t *__restrict__ packed, int64_t d_out, int64_t d_in,
                                                            Pattern pat, int8_t *__restrict__ W_eff)
{
    const int64_t gpr = d_in / pat.M;   // groups per row
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= d_out * gpr) return;
    const int64_t row = gid / gpr;
    const int gr = (int)(gid % gpr);
    const int gpc = CHUNK / pat.M;      // groups per chunk
    const int64_t nchunks = (d_in + CHUNK - 1) / CHUNK;
    const int c = gr / gpc, g = gr % gpc;
    const uint8_t *idx_field = packed + (row * nchunks + c) * pat.chunk_bytes;
    const uint8_t *code_field = idx_field + pat.idx_bytes;
    uint64_t out = 0;
    for (int s = 0; s < pat.N; ++s) {
        const int slot = g * pat.N + s;
        int j = s;
        if (pat.b) {
            const int p = slot * pat.b;
            const uint32_t two = (uint32_t)idx_field[p >> 3] | ((uint32_t)idx_field[(p >> 3) + 1] << 8);   // the next byte is still inside the chunk
            j = (int)((two >> (p & 7)) & ((1u << pat.b) - 1u));
        }
        const int v = slot & 15;
        const int cp = 32 * (slot >> 4) + 8 * (v & 3) + 2 * (v >> 2);
        const uint32_t code = (code_field[cp >> 3] >> (cp & 7)) & 3u;
        const uint64_t byte = code == 1u ? 0x01u : code == 3u ? 0xffu : 0u;
        out |= byte << (8 * j);
    }
    int8_t *dst = W_eff + row * d_in + (int64_t)gr * pat.M;
    if (pat.M == 8) *reinterpret_cast<uint2 *>(dst) = make_uint2((uint32_t)out, (uint32_t)(out >> 32));
    else if (pat.M == 4) *reinterpret_cast<uint32_t *>(dst) = (uint32_t)out;
    else *reinterpret_cast<uint16_t *>(dst) = (uint16_t)out;
}

// Patterns that never keep more than two weights in an aligned group of four (1:2, 1:4, 2:4 itself,
// 1:8, 2:8) are instances of 2:4, so the sparse matrix instruction can run them.  This kernel rewrites
// such a packed matrix as the 2:4 operand form the sparse GEMM reads (32-byte chunks: four index
// words, four code words): one thread per 32 weights = one index word and one code word.  Groups
// with fewer than two kept weights get padding slots with code 0 (their index is irrelevant).
__global__ void __launch_bounds__(256) repack_2of4_kernel(const uint8_t *__restrict__ packed, int64_t d_out, int64_t d_in,
                                                          Pattern pat, uint8_t *__restrict__ out24)
{
    const int64_t nchunks = d_in / CHUNK;   // the caller guarantees whole chunks
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= d_out * nchunks * 4) return;
    const int64_t chunk = q >> 2;
    const int w = (int)(q & 3);             // which 32-weight quarter of the chunk
    const uint8_t *idx_field = packed + chunk * pat.chunk_bytes;
    const uint8_t *code_field = idx_field + pat.idx_bytes;
    // state of the eight target groups in registers: iw takes the positions as they arrive (low two bits
    // of nibble t first, then the high two), cw the codes at their final place, cntw two bits of count
    uint32_t iw = 0, cw = 0, cntw = 0;
    const int gps = 32 / pat.M;             // source groups in this quarter
    for (int gs = 0; gs < gps; ++gs) {
        const int g = w * gps + gs;
        for (int s = 0; s < pat.N; ++s) {
            const int slot = g * pat.N + s;
            int j = s;
            if (pat.b) {
                const int p = slot * pat.b;
                const uint32_t two = (uint32_t)idx_field[p >> 3] | ((uint32_t)idx_field[(p >> 3) + 1] << 8);
                j = (int)((two >> (p & 7)) & ((1u << pat.b) - 1u));
            }
            const int sv = slot & 15;
            const int cp = 32 * (slot >> 4) + 8 * (sv & 3) + 2 * (sv >> 2);
            const uint32_t c = (code_field[cp >> 3] >> (cp & 7)) & 3u;
            const int k = gs * pat.M + j;   // weight inside the quarter; slots of a group come in ascending index
            const int t = k >> 2;
            const uint32_t n = (cntw >> (2 * t)) & 3u;   // 0 or 1 for an instance of 2:4
            iw |= (uint32_t)(k & 3) << (4 * t + 2 * n);
            const int v = 2 * t + (int)n;   // value index inside the code word
            cw |= c << (8 * (v & 3) + 2 * (v >> 2));
            cntw += 1u << (2 * t);
        }
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t n = (cntw >> (2 * t)) & 3u;
        const uint32_t p0 = (iw >> (4 * t)) & 3u;
        if (n == 0) {
            iw |= 1u << (4 * t + 2);                           // positions (0, 1), both codes 0
        } else if (n == 1) {
            if (p0 < 3) {
                iw |= 3u << (4 * t + 2);                       // (p, 3): padding last
            } else {                                           // (0, 3): padding first, the kept value moves to the second slot
                const int v0 = 2 * t, v1 = 2 * t + 1;
                const uint32_t c = (cw >> (8 * (v0 & 3) + 2 * (v0 >> 2))) & 3u;
                cw &= ~(3u << (8 * (v0 & 3) + 2 * (v0 >> 2)));
                cw |= c << (8 * (v1 & 3) + 2 * (v1 >> 2));
                iw = (iw & ~(0xfu << (4 * t))) | (0xcu << (4 * t));
            }
        }
    }
    uint32_t *o = reinterpret_cast<uint32_t *>(out24 + chunk * 32);
    o[w] = iw;
    o[4 + w] = cw;
}

// ---- mask flips between two packed forms (ablation study, mask flip rate equation) ---------------
// one thread per group: the kept positions of both forms as M-bit sets, popcount of their XOR;
// block sums go to the workspace and are added in a fixed order by the finalize kernel
constexpr int FLIP_GROUPS_PER_THREAD = 8;

__device__ __forceinline__ uint32_t group_mask_bits(const uint8_t *idx_field, int g, const Pattern &pat)
{
    uint32_t m = 0;
    for (int s = 0; s < pat.N; ++s) {
        const int p = (g * pat.N + s) * pat.b;
        const uint32_t two = (uint32_t)idx_field[p >> 3] | ((uint32_t)idx_field[(p >> 3) + 1] << 8);   // next byte: still in the chunk
        m |= 1u << ((two >> (p & 7)) & ((1u << pat.b) - 1u));
    }
    return m;
}

// N:M mask as a bit plane: word (row, j) holds the mask of weights 32 j .. 32 j + 31 of the row (bit = position);
// one thread per word.  Rows are d_in / 32 words, rounded up (positions past d_in read as zero).
__global__ void __launch_bounds__(256) mask_bitplane_kernel(const uint8_t *__restrict__ packed, int64_t d_out, int64_t d_in,
                                                            Pattern pat, uint32_t *__restrict__ bits)
{
    const int64_t wpr = (d_in + 31) / 32;
    const int64_t wid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (wid >= d_out * wpr) return;
    const int64_t row = wid / wpr;
    const int j = (int)(wid % wpr);
    const int64_t nchunks = (d_in + CHUNK - 1) / CHUNK;
    const uint8_t *idx_field = packed + (row * nchunks + j / 4) * pat.chunk_bytes;
    const int gpw = 32 / pat.M;          // groups per word
    const int g0 = (j % 4) * gpw;        // first group of the word inside its chunk
    uint32_t word = 0;
    for (int gl = 0; gl < gpw; ++gl) {
        if ((int64_t)j * 32 + (int64_t)gl * pat.M >= d_in) break;
        const uint32_t gm = pat.b ? group_mask_bits(idx_field, g0 + gl, pat) : (1u << pat.M) - 1u;
        word |= gm << (gl * pat.M);
    }
    bits[wid] = word;
}

__global__ void __launch_bounds__(256) mask_flips_kernel(const uint8_t *__restrict__ pa, const uint8_t *__restrict__ pb,
                                                         int64_t d_out, int64_t d_in, Pattern pat,
                                                         unsigned long long *__restrict__ partial)
{
    __shared__ unsigned int wave_sum[4];
    const int64_t gpr = d_in / pat.M, total = d_out * gpr;
    const int gpc = CHUNK / pat.M;
    const int64_t nchunks = (d_in + CHUNK - 1) / CHUNK;
    unsigned int flips = 0;
    const int64_t base = ((int64_t)blockIdx.x * 256 + threadIdx.x) * FLIP_GROUPS_PER_THREAD;
    for (int i = 0; i < FLIP_GROUPS_PER_THREAD; ++i) {
        const int64_t gid = base + i;
        if (gid >= total) break;
        const int64_t row = gid / gpr;
        const int gr = (int)(gid % gpr);
        const int64_t off = (row * nchunks + gr / gpc) * pat.chunk_bytes;
        flips += __popc(group_mask_bits(pa + off, gr % gpc, pat) ^ group_mask_bits(pb + off, gr % gpc, pat));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) flips += __shfl_xor((int)flips, o, 64);
    if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = flips;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (unsigned long long)wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
}

__global__ void __launch_bounds__(256) mask_flips_finalize_kernel(const unsigned long long *__restrict__ partial, int64_t n,
                                                                  unsigned long long *__restrict__ out)
{
    __shared__ unsigned long long sums[256];
    unsigned long long s = 0;
    for (int64_t i = threadIdx.x; i < n; i += 256) s += partial[i];
    sums[threadIdx.x] = s;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if ((int)threadIdx.x < step) sums[threadIdx.x] += sums[threadIdx.x + step];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = sums[0];
}

template <typename WT>
sbn_status launch_pack_kernel(const PackTable &tab, int nblocks, const float *theta, int vec_ok, const Pattern &pat,
                              hipStream_t stream)
{
#define SBN_PACK_CASE(n, m)                                                                             \
    if (pat.N == n && pat.M == m) {                                                                     \
        hipLaunchKernelGGL((pack_kernel<WT, n, m>), dim3(nblocks), dim3(256), 0, stream, tab, theta, vec_ok); \
        return check_launch("pack_kernel");                                                             \
    }
    SBN_PACK_CASE(1, 2) SBN_PACK_CASE(2, 2)
    SBN_PACK_CASE(1, 4) SBN_PACK_CASE(2, 4) SBN_PACK_CASE(3, 4) SBN_PACK_CASE(4, 4)
    SBN_PACK_CASE(1, 8) SBN_PACK_CASE(2, 8) SBN_PACK_CASE(3, 8) SBN_PACK_CASE(4, 8)
    SBN_PACK_CASE(5, 8) SBN_PACK_CASE(6, 8) SBN_PACK_CASE(7, 8) SBN_PACK_CASE(8, 8)
#undef SBN_PACK_CASE
    return SBN_EUNSUPPORTED;
}

}  // namespace

size_t pack_workspace_bytes(int64_t count, int64_t d_out, int64_t d_in)
{
    const int64_t blocks = ceil_div(d_out * d_in, PACK_SUM_ELEMS);
    // partial sums, thresholds, ready words, and the per-unit flip counts of the flip-counting call
    return align_up((size_t)count * (size_t)blocks * sizeof(double), 256) + align_up((size_t)count * sizeof(float), 256) +
           align_up((size_t)count * PACK_SYNC_WORDS * sizeof(unsigned), 256) + align_up((size_t)count * (size_t)blocks * sizeof(uint32_t), 256);
}

__global__ void __launch_bounds__(256) pack_sync_clear_kernel(unsigned *words, int nwords, unsigned long long *partials, int npartials)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < nwords) words[i] = 0u;
    if (i < npartials) partials[i] = PACK_NO_PARTIAL;
}

// blocks of the single-read pack kernel the device holds at once = its grid (per instantiation, cached per thread)
// Compact units a block queues and wavefronts per SIMD of the single-read kernel, per pattern.  Measured
// (sweep of 210 matrices): 2:4 with (queue, wavefronts) = (1, 6) 1.27 ms, (2, 5) 1.39, (1, 7) 1.50 (spills);
// 1:4 / 2:8 with (2, 5) 1.11 / 1.27 ms, (3, 5) 1.12 / 1.31, (1, 7) 1.14 / 1.31, (2, 6) 1.17 / 1.36.
template <int N, int M> struct PackStreamShape {
    static constexpr int QD = (N == 2 && M == 4) ? 1 : 2;
    static constexpr int WAVES = (N == 2 && M == 4) ? 6 : 5;
};

template <int N, int M>
static void launch_pack_stream(int grid, hipStream_t stream, const PackTable &tab, const PackSync &sync)
{
    if (sync.unit_flips)
        hipLaunchKernelGGL((pack_stream_kernel<N, M, PackStreamShape<N, M>::QD, PackStreamShape<N, M>::WAVES, true>), dim3(grid), dim3(256), 0,
                           stream, tab, sync);
    else
        hipLaunchKernelGGL((pack_stream_kernel<N, M, PackStreamShape<N, M>::QD, PackStreamShape<N, M>::WAVES, false>), dim3(grid), dim3(256), 0,
                           stream, tab, sync);
}

template <int N, int M>
static void launch_pack_fast(int grid, hipStream_t stream, const PackTable &tab, const float *theta, uint32_t *unit_flips)
{
    if (unit_flips) hipLaunchKernelGGL((pack_fast_kernel<N, M, true>), dim3(grid), dim3(256), 0, stream, tab, theta, unit_flips);
    else hipLaunchKernelGGL((pack_fast_kernel<N, M, false>), dim3(grid), dim3(256), 0, stream, tab, theta, unit_flips);
}

template <int N, int M>
static int fused_capacity()
{
    static thread_local int cap = 0;
    if (cap == 0) {
        int per_cu = 0;
        // (the flip-counting instantiation has the same launch bounds, wavefronts per SIMD and LDS plus 16 bytes)
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pack_stream_kernel<N, M, PackStreamShape<N, M>::QD, PackStreamShape<N, M>::WAVES, true>, 256, 0) != hipSuccess) per_cu = 0;
        cap = per_cu > 0 ? per_cu * device_cus() : -1;
    }
    return cap;
}

// flips: null, or one counter per matrix: the packed buffers then hold the previous packed forms, which are replaced, and
// the counters receive the mask flips between the two (only in the forms that keep a unit's chunks in one block)
sbn_status launch_pack(int count, const PackItem *items, sbn_dtype wdt, const Pattern &pat, void *workspace,
                       size_t ws_bytes, hipStream_t stream, unsigned long long *flips)
{
    if (flips) {
        const bool fast_pattern = (pat.M == 4 && (pat.N == 1 || pat.N == 2)) || (pat.M == 8 && pat.N == 2);
        if (wdt != SBN_BF16 || !fast_pattern) return SBN_EUNSUPPORTED;
        for (int i = 0; i < count; ++i)
            if (items[i].ld != items[i].d_in || items[i].d_in % CHUNK != 0 || !aligned(items[i].W, 16)) return SBN_EUNSUPPORTED;
    }
    // workspace: [partials: one double per absmean block of every matrix][theta: one float per matrix]
    int64_t total_sum_blocks = 0;
    for (int i = 0; i < count; ++i) total_sum_blocks += ceil_div(items[i].d_out * items[i].d_in, PACK_SUM_ELEMS);
    // + [arrival counters and ready words of the single-read form: PACK_SYNC_WORDS per matrix]
    const size_t need = align_up((size_t)total_sum_blocks * sizeof(double), 256) + align_up((size_t)count * sizeof(float), 256) +
                        align_up((size_t)count * PACK_SYNC_WORDS * sizeof(unsigned), 256);
    // + [flip counts of the units of one launch, when flips are counted]
    if (ws_bytes < need + (flips ? align_up((size_t)total_sum_blocks * sizeof(uint32_t), 256) : 0)) return SBN_ESIZE;
    double *partials = static_cast<double *>(workspace);
    float *theta = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + align_up((size_t)total_sum_blocks * sizeof(double), 256));
    unsigned *sync_words = reinterpret_cast<unsigned *>(reinterpret_cast<uint8_t *>(theta) + align_up((size_t)count * sizeof(float), 256));
    uint32_t *unit_flips = flips ? reinterpret_cast<uint32_t *>(static_cast<uint8_t *>(workspace) + need) : nullptr;

    const size_t esz = wdt == SBN_BF16 ? 2 : 4;
    int64_t sum_base = 0;
    for (int first = 0; first < count; first += PACK_MAX_ITEMS) {
        const int n = count - first < PACK_MAX_ITEMS ? count - first : PACK_MAX_ITEMS;
        PackTable tab;
        tab.count = n;
        int vec_ok = 1;
        bool flat_ok = true;            // every matrix: contiguous rows of whole chunks, 16-byte aligned
        int fb[PACK_MAX_ITEMS + 1];     // block prefix of the fast pack kernel (128 chunks per block)
        int sb = 0, pb = 0;
        fb[0] = 0;
        for (int i = 0; i < n; ++i) {
            const PackItem &it = items[first + i];
            tab.it[i] = it;
            tab.sum_block0[i] = sb;
            tab.pack_block0[i] = pb;
            if (it.ld != it.d_in || it.d_in % CHUNK != 0 || !aligned(it.W, 16)) flat_ok = false;
            fb[i + 1] = fb[i] + (int)ceil_div(it.d_out * ceil_div(it.d_in, CHUNK), 128);
            sb += (int)ceil_div(it.d_out * it.d_in, PACK_SUM_ELEMS);
            pb += (int)ceil_div(it.d_out * ceil_div(it.d_in, CHUNK), 16);
            if (!aligned(it.W, 16) || (it.ld * esz) % 16 != 0 || it.d_in % 8 != 0) vec_ok = 0;
        }
        tab.sum_block0[n] = sb;
        tab.pack_block0[n] = pb;
        double *part = partials + sum_base;
        float *th = theta + first;
        const bool fast_pattern = (pat.M == 4 && (pat.N == 1 || pat.N == 2)) || (pat.M == 8 && pat.N == 2);
        const bool fast = wdt == SBN_BF16 && fast_pattern && flat_ok;
        sbn_status st = SBN_OK;
        // single-read form: persistent grid of as many blocks as the device holds; no matrix may have more units than that
        bool fused = fast;
        int cap = 0;
        if (fast) {
            cap = pat.M == 4 && pat.N == 2 ? fused_capacity<2, 4>() : pat.M == 4 ? fused_capacity<1, 4>() : fused_capacity<2, 8>();
            for (int i = 0; i < n; ++i) fused = fused && fb[i + 1] - fb[i] <= cap;
        }
        if (fused) {
            for (int i = 0; i < n; ++i) tab.pack_block0[i] = fb[i];
            tab.pack_block0[n] = fb[n];
            unsigned *words = sync_words + (size_t)PACK_SYNC_WORDS * first;
            const int nclear = n * PACK_SYNC_WORDS > sb ? n * PACK_SYNC_WORDS : sb;
            hipLaunchKernelGGL(pack_sync_clear_kernel, dim3((nclear + 255) / 256), dim3(256), 0, stream, words, n * PACK_SYNC_WORDS,
                               reinterpret_cast<unsigned long long *>(part), sb);
            st = check_launch("pack_sync_clear_kernel");
            if (st != SBN_OK) return st;
            PackSync sync{part, th, words, pack_spin_limit(), unit_flips};
            const int grid = fb[n] < cap ? fb[n] : cap;
            if (pat.M == 4 && pat.N == 2) launch_pack_stream<2, 4>(grid, stream, tab, sync);
            else if (pat.M == 4) launch_pack_stream<1, 4>(grid, stream, tab, sync);
            else launch_pack_stream<2, 8>(grid, stream, tab, sync);
            st = check_launch("pack_stream_kernel");
            if (st != SBN_OK) return st;
            if (flips) {
                hipLaunchKernelGGL(pack_flips_sum_kernel, dim3(n), dim3(256), 0, stream, tab, unit_flips, flips + first);
                st = check_launch("pack_flips_sum_kernel");
                if (st != SBN_OK) return st;
            }
            sum_base += sb;
            continue;
        }
        if (wdt == SBN_BF16)
            hipLaunchKernelGGL(absmean_partial_kernel<uint16_t>, dim3(sb), dim3(256), 0, stream, tab, part, vec_ok);
        else
            hipLaunchKernelGGL(absmean_partial_kernel<float>, dim3(sb), dim3(256), 0, stream, tab, part, vec_ok);
        st = check_launch("absmean_partial_kernel");
        if (st != SBN_OK) return st;
        hipLaunchKernelGGL(absmean_finalize_kernel, dim3(n), dim3(256), 0, stream, tab, part, th);
        st = check_launch("absmean_finalize_kernel");
        if (st != SBN_OK) return st;
        if (fast) {
            for (int i = 0; i < n; ++i) tab.pack_block0[i] = fb[i];
            tab.pack_block0[n] = fb[n];
            if (pat.M == 4 && pat.N == 2) launch_pack_fast<2, 4>(fb[n], stream, tab, th, unit_flips);
            else if (pat.M == 4) launch_pack_fast<1, 4>(fb[n], stream, tab, th, unit_flips);
            else launch_pack_fast<2, 8>(fb[n], stream, tab, th, unit_flips);
            st = check_launch("pack_fast_kernel");
            if (st == SBN_OK && flips) {
                hipLaunchKernelGGL(pack_flips_sum_kernel, dim3(n), dim3(256), 0, stream, tab, unit_flips, flips + first);
                st = check_launch("pack_flips_sum_kernel");
            }
        } else {
            st = wdt == SBN_BF16 ? launch_pack_kernel<uint16_t>(tab, pb, th, vec_ok, pat, stream)
                                 : launch_pack_kernel<float>(tab, pb, th, vec_ok, pat, stream);
        }
        if (st != SBN_OK) return st;
        sum_base += sb;
    }
    return SBN_OK;
}

sbn_status launch_unpack(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, int8_t *W_eff,
                         uint8_t *mask, hipStream_t stream)
{
    const int64_t total = d_out * ceil_div(d_in, CHUNK);
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t *>(packed), d_out, d_in, pat, W_eff, mask);
    return check_launch("unpack_kernel");
}

size_t mask_flips_workspace_bytes(int64_t d_out, int64_t d_in, int M)
{
    const int64_t groups = d_out * (d_in / M);
    return align_up((size_t)ceil_div(groups, 256 * FLIP_GROUPS_PER_THREAD) * sizeof(unsigned long long), 256);
}

sbn_status launch_mask_flips(const void *packed_a, const void *packed_b, int64_t d_out, int64_t d_in, const Pattern &pat,
                             uint64_t *flips_out, void *workspace, hipStream_t stream)
{
    unsigned long long *out = reinterpret_cast<unsigned long long *>(flips_out);
    unsigned long long *partial = static_cast<unsigned long long *>(workspace);
    if (pat.b == 0) {   // N == M: every position is kept in both forms
        hipLaunchKernelGGL(mask_flips_finalize_kernel, dim3(1), dim3(256), 0, stream, partial, (int64_t)0, out);
        return check_launch("mask_flips_finalize_kernel");
    }
    const int64_t nblocks = ceil_div(d_out * (d_in / pat.M), 256 * FLIP_GROUPS_PER_THREAD);
    hipLaunchKernelGGL(mask_flips_kernel, dim3((unsigned)nblocks), dim3(256), 0, stream, static_cast<const uint8_t *>(packed_a),
                       static_cast<const uint8_t *>(packed_b), d_out, d_in, pat, partial);
    sbn_status st = check_launch("mask_flips_kernel");
    if (st != SBN_OK) return st;
    hipLaunchKernelGGL(mask_flips_finalize_kernel, dim3(1), dim3(256), 0, stream, partial, nblocks, out);
    return check_launch("mask_flips_finalize_kernel");
}

sbn_status launch_repack_2of4(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, uint8_t *out24,
                              hipStream_t stream)
{
    const int64_t total = d_out * (d_in / CHUNK) * 4;
    hipLaunchKernelGGL(repack_2of4_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t *>(packed), d_out, d_in, pat, out24);
    return check_launch("repack_2of4_kernel");
}

// Any pattern -> dense 2-bit codes (the packed form of N = M: eight code words per 128-weight chunk,
// weight p of the chunk in word p / 16 at bits 8 * (p % 4) + 2 * ((p % 16) / 4)), zero codes at the
// dropped positions.  One thread per output word (16 weights = 16 / M groups).  Whole chunks only.
// PN, PM = the pattern as compile-time constants (bit positions become literals, the loops unroll), or 0, 0 = read it
// from pat
template <int PN, int PM>
__global__ void __launch_bounds__(256) repack_dense_codes_kernel(const uint8_t *__restrict__ packed, int64_t nwords, Pattern pat,
                                                                 uint32_t *__restrict__ out)
{
    const int64_t wid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (wid >= nwords) return;
    const int N = PN ? PN : pat.N, M = PM ? PM : pat.M;
    const int b = PM ? (PM == PN ? 0 : PM == 2 ? 1 : PM == 4 ? 2 : 3) : pat.b;
    const int64_t chunk = wid >> 3;
    const int w = (int)(wid & 7);
    const uint8_t *idx_field = packed + chunk * pat.chunk_bytes;
    const uint8_t *code_field = idx_field + pat.idx_bytes;
    const int gpw = 16 / M;   // groups per word
    const int slot0 = w * gpw * N;
    uint32_t word = 0;
#pragma unroll
    for (int gl = 0; gl < gpw; ++gl) {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int slot = slot0 + gl * N + n;
            int j = n;
            if (b) {
                const int p = slot * b;
                const uint32_t two = (uint32_t)idx_field[p >> 3] | ((uint32_t)idx_field[(p >> 3) + 1] << 8);   // the next byte is still inside the chunk
                j = (int)((two >> (p & 7)) & ((1u << b) - 1u));
            }
            const int sv = slot & 15;
            const int cp = 32 * (slot >> 4) + 8 * (sv & 3) + 2 * (sv >> 2);
            const uint32_t code = (code_field[cp >> 3] >> (cp & 7)) & 3u;
            const int v = gl * M + j;
            word |= code << (8 * (v & 3) + 2 * (v >> 2));
        }
    }
    out[wid] = word;
}

// 6:8, the paper's main pattern, with one thread per chunk: 60 bytes in as 15 words (36 bytes of 3-bit indices, 24 of
// codes), 32 bytes out; every bit position is a literal after unrolling, and no byte-sized loads are left.
__global__ void __launch_bounds__(256) repack_6of8_dense_codes_kernel(const uint8_t *__restrict__ packed, int64_t nchunks,
                                                                      uint4 *__restrict__ out)
{
    const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (chunk >= nchunks) return;
    const uint32_t *in = reinterpret_cast<const uint32_t *>(packed + chunk * 60);
    uint32_t d[16];
#pragma unroll
    for (int i = 0; i < 15; ++i) d[i] = in[i];
    d[15] = 0;
    uint32_t o[8];
#pragma unroll
    for (int w = 0; w < 8; ++w) {
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < 12; ++k) {   // the two groups of the word: slots 12 w .. 12 w + 11
            const int slot = 12 * w + k, p = 3 * slot;
            const uint32_t j = (p & 31) <= 29 ? (d[p >> 5] >> (p & 31)) & 7u
                                              : __funnelshift_r(d[p >> 5], d[(p >> 5) + 1], p & 31) & 7u;
            const int sv = slot & 15;
            const uint32_t code = (d[9 + (slot >> 4)] >> (8 * (sv & 3) + 2 * (sv >> 2))) & 3u;
            // weight v = 8 (k / 6) + j of the word sits at bits 8 (v % 4) + 2 (v / 4)
            word |= code << (8 * (j & 3u) + 2 * (j >> 2) + 4 * (k / 6));
        }
        o[w] = word;
    }
    out[2 * chunk] = make_uint4(o[0], o[1], o[2], o[3]);
    out[2 * chunk + 1] = make_uint4(o[4], o[5], o[6], o[7]);
}

sbn_status launch_mask_bitplane(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, uint32_t *bits,
                                hipStream_t stream)
{
    const int64_t words = d_out * ((d_in + 31) / 32);
    hipLaunchKernelGGL(mask_bitplane_kernel, dim3((unsigned)ceil_div(words, 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t *>(packed), d_out, d_in, pat, bits);
    return check_launch("mask_bitplane_kernel");
}

sbn_status launch_repack_dense_codes(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, uint8_t *out,
                                     hipStream_t stream)
{
    const int64_t nwords = d_out * (d_in / CHUNK) * 8;
    const dim3 grid((unsigned)ceil_div(nwords, 256));
    const uint8_t *in = static_cast<const uint8_t *>(packed);
    uint32_t *o = reinterpret_cast<uint32_t *>(out);
    if (pat.N == 6 && pat.M == 8)
        hipLaunchKernelGGL(repack_6of8_dense_codes_kernel, dim3((unsigned)ceil_div(nwords / 8, 256)), dim3(256), 0, stream, in,
                           nwords / 8, reinterpret_cast<uint4 *>(out));
    else hipLaunchKernelGGL((repack_dense_codes_kernel<0, 0>), grid, dim3(256), 0, stream, in, nwords, pat, o);
    return check_launch("repack_dense_codes_kernel");
}

sbn_status launch_expand_groups(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, int8_t *W_eff,
                                hipStream_t stream)
{
    const int64_t total = d_out * (d_in / pat.M);
    hipLaunchKernelGGL(expand_groups_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t *>(packed), d_out, d_in, pat, W_eff);
    return check_launch("expand_groups_kernel");
}

}  // namespace sbn
