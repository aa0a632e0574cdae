// Internal declarations shared by the translation units of libsbn (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sbn.h"

namespace sbn {

// Geometry of the packed layout for one N:M pattern (see include/sbn.h).
struct Pattern {
    int N, M;
    int b;            // index bits per slot (0 when N == M)
    int slots;        // slots per 128-weight chunk
    int idx_bytes;    // bytes of the index field of a chunk
    int code_bytes;   // bytes of the code field of a chunk
    int chunk_bytes;  // idx_bytes + code_bytes
};

inline bool make_pattern(int N, int M, Pattern &p)
{
    int b = M == 2 ? 1 : M == 4 ? 2 : M == 8 ? 3 : -1;
    if (b < 0 || N < 1 || N > M) return false;
    if (N == M) b = 0;
    p.N = N;
    p.M = M;
    p.b = b;
    p.slots = 128 * N / M;
    p.idx_bytes = p.slots * b / 8;
    p.code_bytes = p.slots / 4;
    p.chunk_bytes = p.idx_bytes + p.code_bytes;
    return true;
}

constexpr int CHUNK = 128;  // weights per chunk of the packed layout

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// error text of the last failed HIP call of this thread
void set_hip_error(hipError_t e, const char *what);
sbn_status check_launch(const char *what);

// ---- pack (sbn_pack.hip) --------------------------------------------------------------------
struct PackItem {
    const void *W;
    uint8_t *packed;
    float *gamma;
    int64_t d_out, d_in, ld;
};
constexpr int PACK_MAX_ITEMS = 70;     // matrices per launch (descriptor table travels as kernel argument: 4 KB at most)
constexpr int64_t PACK_SUM_ELEMS = 16384;  // elements reduced by one block of the absmean pass
size_t pack_workspace_bytes(int64_t count, int64_t d_out, int64_t d_in);
sbn_status launch_pack(int count, const PackItem *items, sbn_dtype wdt, const Pattern &pat,
                       void *workspace, size_t ws_bytes, hipStream_t stream, unsigned long long *flips = nullptr);
size_t mask_flips_workspace_bytes(int64_t d_out, int64_t d_in, int M);
sbn_status launch_mask_flips(const void *packed_a, const void *packed_b, int64_t d_out, int64_t d_in, const Pattern &pat,
                             uint64_t *flips_out, void *workspace, hipStream_t stream);
// N:M patterns that are instances of 2:4: at most two kept weights in every aligned group of four
inline bool embeds_in_2of4(const Pattern &p) { return (p.M == 2 && p.N == 1) || (p.M >= 4 && p.N <= 2); }
sbn_status launch_repack_2of4(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, uint8_t *out24,
                              hipStream_t stream);
// any pattern -> dense 2-bit codes (the packed form of N = M), explicit zero codes at the dropped positions
sbn_status launch_repack_dense_codes(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, uint8_t *out,
                                     hipStream_t stream);
// the N:M mask of a packed matrix as one bit per weight, rows of ceil(d_in / 32) words
sbn_status launch_mask_bitplane(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, uint32_t *bits,
                                hipStream_t stream);
sbn_status launch_expand_groups(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat, int8_t *W_eff,
                                hipStream_t stream);
sbn_status launch_unpack(const void *packed, int64_t d_out, int64_t d_in, const Pattern &pat,
                         int8_t *W_eff, uint8_t *mask, hipStream_t stream);

// ---- forward (sbn_linear.hip) ----------------------------------------------------------------
struct LinearItem {
    const void *X;        // bf16 [tokens, d_in]
    const void *packed;
    const float *gamma;
    const float *bias;    // may be null
    float *Y;
    int8_t *xq;           // int8 [tokens, d_in] (caller's buffer or workspace)
    float *sx;            // fp32 [tokens]
    int32_t *acc_out;     // may be null
    int64_t tokens, d_in, d_out;
    bool quantized = true;   // xq / sx already hold the quantized activations (false: launch_gemv derives them from X)
};
size_t linear_workspace_bytes(int64_t tokens, int64_t d_out, int64_t d_in);
sbn_status launch_act_quant(const void *X, int64_t tokens, int64_t d_in, int8_t *xq, float *sx,
                            hipStream_t stream);
sbn_status launch_rmsnorm_act_quant(const void *X, const float *gain, float eps, int64_t tokens, int64_t d_in, int8_t *xq,
                                    float *sx, void *xn, hipStream_t stream);
// how the decode kernels read the packed weights: the 2:4 operand form, dense 2-bit codes (N = M), or the 1:4
// packed form as stored (rewritten into sparse operands in registers)
enum GemvForm : int { GEMV_2OF4 = 0, GEMV_DENSE = 1, GEMV_1OF4 = 2 };
sbn_status launch_gemv(int count, const LinearItem *items, GemvForm form, hipStream_t stream);
// dense_codes: the weights are dense 2-bit codes (packed form of N = M) instead of the 2:4 form
sbn_status launch_gemm_smfmac(int count, const LinearItem *items, bool dense_codes, hipStream_t stream);
// decode batches (sbn_batch.hip): problems of at most 64 tokens without bias or accumulator output stream their weights
// once through a kernel of their own; launch_gemm_smfmac hands them over
bool gemv_batch_takes(const LinearItem &it);
sbn_status launch_gemv_batch(int count, const LinearItem *items, bool dense_codes, hipStream_t stream);
sbn_status launch_gemm_dense(const LinearItem &it, const Pattern &pat, int8_t *w_dense, hipStream_t stream);
sbn_status launch_gemm_dense_expanded(const LinearItem &it, const int8_t *w_dense, hipStream_t stream);
sbn_status launch_linear_generic(const LinearItem &it, const Pattern &pat, hipStream_t stream);

int device_cus();   // multiprocessors of the current device

// Bounds of the two bounded inter-block waits (streaming decode: flags of the fused quantizer; single-read pack:
// the matrix's ready word), in polls; negative = never wait.  Process-wide, changed only by the test hook
// sbn_test_set_spin_limits; the launchers read them once per launch.
constexpr int GEMV_SPIN_DEFAULT = 1 << 10;
constexpr int PACK_SPIN_DEFAULT = 1 << 12;
int gemv_spin_limit();
int pack_spin_limit();

// ---- backward (sbn_backward.hip) ---------------------------------------------------------------
size_t backward_workspace_bytes(int64_t tokens, int64_t d_out, int64_t d_in);
struct BackwardItem {
    const void *dY;
    int64_t tokens, d_in, d_out;
    const void *packed;
    const float *gamma;
    const int8_t *xq;
    const float *sx;
    void *dX, *dW;
    void *workspace;   // this layer's share, backward_workspace_bytes(tokens, d_out, d_in)
};
sbn_status launch_backward_grouped(int count, const BackwardItem *items, const Pattern &pat, int flags, hipStream_t stream);
sbn_status launch_backward(const void *dY, int64_t tokens, int64_t d_in, int64_t d_out,
                           const Pattern &pat, const void *packed, const float *gamma,
                           const int8_t *xq, const float *sx, void *dX, void *dW, int flags,
                           void *workspace, size_t ws_bytes, hipStream_t stream);

}  // namespace sbn
