// extern "C" entry points of libsbn: argument validation on the host, workspace carving, dispatch.
// Nothing here allocates or synchronises; every check happens before the first launch.
#include <atomic>
#include <climits>
#include <string>
#include <vector>

#include "sbn_internal.hpp"

namespace sbn {

static thread_local std::string g_last_error;

void set_hip_error(hipError_t e, const char *what)
{
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
}

sbn_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error(e, what);
        return SBN_EHIP;
    }
    return SBN_OK;
}

static std::atomic<int> g_gemv_spin{GEMV_SPIN_DEFAULT}, g_pack_spin{PACK_SPIN_DEFAULT};
int gemv_spin_limit() { return g_gemv_spin.load(std::memory_order_relaxed); }
int pack_spin_limit() { return g_pack_spin.load(std::memory_order_relaxed); }

static sbn_status check_shape(int64_t d_out, int64_t d_in, int N, int M, Pattern &pat)
{
    if (d_out <= 0 || d_in <= 0) return SBN_EINVAL;
    if (!make_pattern(N, M, pat)) return SBN_EINVAL;
    if (d_in % M != 0) return SBN_EINVAL;
    // index arithmetic in the kernels is 32-bit per matrix in a few places
    if (d_out * ceil_div(d_in, CHUNK) >= (int64_t)1 << 31) return SBN_EUNSUPPORTED;
    return SBN_OK;
}

static sbn_path resolve_path(sbn_path path, int64_t tokens, int64_t d_in, const Pattern &pat)
{
    if (path != SBN_PATH_AUTO) return path;
    const bool is24 = pat.N == 2 && pat.M == 4;
    // 2:4 and its instances (1:4, 2:8, ...: rewritten into the 2:4 operand form first) take the sparse instruction as
    // it is meant.  Every other pattern (the paper's 6:8 among them) has no sparse matrix instruction of its own on
    // this part: its weights run as dense 2-bit codes (N = M is stored that way, the rest is converted first), in
    // decode through the streaming kernel and beyond decode sizes through the same sparse instruction, issued twice
    // per group of four weights (positions 0, 1 and positions 2, 3 - the matrix-core time of a dense int8 product, at
    // a quarter of its weight bytes)
    if (d_in % CHUNK == 0) return tokens <= 16 ? SBN_PATH_GEMV : SBN_PATH_SMFMAC;
    return d_in % 64 == 0 ? SBN_PATH_DENSE_MFMA : SBN_PATH_GENERIC;
}

}  // namespace sbn

using namespace sbn;

extern "C" {

const char *sbn_last_error(void) { return g_last_error.c_str(); }

void sbn_test_set_spin_limits(int gemv_polls, int pack_polls)
{
    g_gemv_spin.store(gemv_polls == INT_MIN ? GEMV_SPIN_DEFAULT : gemv_polls, std::memory_order_relaxed);
    g_pack_spin.store(pack_polls == INT_MIN ? PACK_SPIN_DEFAULT : pack_polls, std::memory_order_relaxed);
}

sbn_status sbn_packed_bytes(int64_t d_out, int64_t d_in, int N, int M, size_t *bytes)
{
    Pattern pat;
    if (!bytes) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    *bytes = (size_t)d_out * (size_t)ceil_div(d_in, CHUNK) * (size_t)pat.chunk_bytes;
    return SBN_OK;
}

sbn_status sbn_workspace_bytes(sbn_op op, int64_t tokens, int64_t d_out, int64_t d_in, int N, int M, size_t *bytes)
{
    Pattern pat;
    if (!bytes || (tokens <= 0 && op != SBN_OP_MASK_FLIPS)) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    switch (op) {
    case SBN_OP_QUANTIZE_MASK_PACK: *bytes = pack_workspace_bytes(tokens, d_out, d_in); return SBN_OK;
    case SBN_OP_LINEAR: *bytes = linear_workspace_bytes(tokens, d_out, d_in); return SBN_OK;
    case SBN_OP_BACKWARD: *bytes = backward_workspace_bytes(tokens, d_out, d_in); return SBN_OK;
    case SBN_OP_MASK_FLIPS: *bytes = mask_flips_workspace_bytes(d_out, d_in, M); return SBN_OK;
    }
    return SBN_EINVAL;
}

sbn_status sbn_quantize_mask_pack(const void *W_latent, sbn_dtype wdt, int64_t d_out, int64_t d_in, int64_t ld_w,
                                  int N, int M, void *packed, float *gamma, void *workspace, size_t ws_bytes,
                                  void *stream)
{
    Pattern pat;
    if (!W_latent || !packed || !gamma || !workspace) return SBN_EINVAL;
    if (wdt != SBN_F32 && wdt != SBN_BF16) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    if (ld_w < d_in) return SBN_EINVAL;
    if (!aligned(packed, 16) || !aligned(gamma, 4) || !aligned(workspace, 256)) return SBN_EALIGN;
    if (!aligned(W_latent, wdt == SBN_BF16 ? 2 : 4)) return SBN_EALIGN;
    PackItem it{W_latent, static_cast<uint8_t *>(packed), gamma, d_out, d_in, ld_w};
    return launch_pack(1, &it, wdt, pat, workspace, ws_bytes, static_cast<hipStream_t>(stream));
}

sbn_status sbn_quantize_mask_pack_batched(int count, const void *const *W_latent, sbn_dtype wdt, const int64_t *d_out,
                                          const int64_t *d_in, int N, int M, void *const *packed,
                                          float *const *gamma, void *workspace, size_t ws_bytes, void *stream)
{
    if (count <= 0 || count > 4096 || !W_latent || !d_out || !d_in || !packed || !gamma || !workspace) return SBN_EINVAL;
    if (wdt != SBN_F32 && wdt != SBN_BF16) return SBN_EINVAL;
    if (!aligned(workspace, 256)) return SBN_EALIGN;
    Pattern pat;
    static thread_local std::vector<PackItem> tl_items;   // host-side descriptor list, reused between calls
    tl_items.resize(count);
    for (int i = 0; i < count; ++i) {
        if (!W_latent[i] || !packed[i] || !gamma[i]) return SBN_EINVAL;
        sbn_status st = check_shape(d_out[i], d_in[i], N, M, pat);
        if (st != SBN_OK) return st;
        if (!aligned(packed[i], 16) || !aligned(gamma[i], 4)) return SBN_EALIGN;
        if (!aligned(W_latent[i], wdt == SBN_BF16 ? 2 : 4)) return SBN_EALIGN;
        tl_items[i] = PackItem{W_latent[i], static_cast<uint8_t *>(packed[i]), gamma[i], d_out[i], d_in[i], d_in[i]};
    }
    return launch_pack(count, tl_items.data(), wdt, pat, workspace, ws_bytes, static_cast<hipStream_t>(stream));
}

sbn_status sbn_quantize_mask_pack_flips_batched(int count, const void *const *W_latent, sbn_dtype wdt, const int64_t *d_out,
                                                const int64_t *d_in, int N, int M, void *const *packed,
                                                float *const *gamma, uint64_t *flips_out, void *workspace, size_t ws_bytes,
                                                void *stream)
{
    if (count <= 0 || count > 4096 || !W_latent || !d_out || !d_in || !packed || !gamma || !flips_out || !workspace) return SBN_EINVAL;
    if (wdt != SBN_F32 && wdt != SBN_BF16) return SBN_EINVAL;
    if (!aligned(workspace, 256) || !aligned(flips_out, 8)) return SBN_EALIGN;
    Pattern pat;
    static thread_local std::vector<PackItem> tl_items;   // host-side descriptor list, reused between calls
    tl_items.resize(count);
    for (int i = 0; i < count; ++i) {
        if (!W_latent[i] || !packed[i] || !gamma[i]) return SBN_EINVAL;
        sbn_status st = check_shape(d_out[i], d_in[i], N, M, pat);
        if (st != SBN_OK) return st;
        if (!aligned(packed[i], 16) || !aligned(gamma[i], 4)) return SBN_EALIGN;
        if (!aligned(W_latent[i], 2)) return SBN_EALIGN;
        tl_items[i] = PackItem{W_latent[i], static_cast<uint8_t *>(packed[i]), gamma[i], d_out[i], d_in[i], d_in[i]};
    }
    return launch_pack(count, tl_items.data(), wdt, pat, workspace, ws_bytes, static_cast<hipStream_t>(stream),
                       reinterpret_cast<unsigned long long *>(flips_out));
}

sbn_status sbn_unpack(const void *packed, int64_t d_out, int64_t d_in, int N, int M, int8_t *W_eff, uint8_t *mask,
                      void *stream)
{
    Pattern pat;
    if (!packed || (!W_eff && !mask)) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    return launch_unpack(packed, d_out, d_in, pat, W_eff, mask, static_cast<hipStream_t>(stream));
}

sbn_status sbn_act_quant(const void *X, int64_t tokens, int64_t d_in, int8_t *xq, float *sx, void *stream)
{
    if (!X || !xq || !sx || tokens <= 0 || d_in <= 0) return SBN_EINVAL;
    if (d_in % 8 != 0) return SBN_EUNSUPPORTED;
    if (!aligned(X, 16) || !aligned(xq, 16) || !aligned(sx, 4)) return SBN_EALIGN;
    return launch_act_quant(X, tokens, d_in, xq, sx, static_cast<hipStream_t>(stream));
}

sbn_status sbn_rmsnorm_act_quant(const void *X, int64_t tokens, int64_t d_in, const float *gain, float eps, int8_t *xq, float *sx,
                                 void *xn_out, void *stream)
{
    if (!X || !xq || !sx || tokens <= 0 || d_in <= 0 || !(eps >= 0.0f)) return SBN_EINVAL;
    if (d_in % 8 != 0 || d_in > 16384) return SBN_EUNSUPPORTED;
    if (!aligned(X, 16) || !aligned(xq, 16) || !aligned(sx, 4) || (gain && !aligned(gain, 16)) || (xn_out && !aligned(xn_out, 16)))
        return SBN_EALIGN;
    return launch_rmsnorm_act_quant(X, gain, eps, tokens, d_in, xq, sx, xn_out, static_cast<hipStream_t>(stream));
}

// activations_only: the workspace holds the activation regions only (the entry point with the library's own scratch);
// paths that rewrite or expand the weights into the workspace are then refused
static sbn_status linear_one(const LinearItem &it_in, const Pattern &pat, sbn_path path, void *workspace,
                             size_t ws_bytes, hipStream_t stream, bool activations_only = false)
{
    LinearItem it = it_in;
    const bool is24 = pat.N == 2 && pat.M == 4;
    path = resolve_path(path, it.tokens, it.d_in, pat);
    const bool sparse_form = is24 || embeds_in_2of4(pat);   // runs on the sparse instruction (after a rewrite unless 2:4)
    const bool one4_decode = pat.N == 1 && pat.M == 4 && path == SBN_PATH_GEMV;   // the decode kernels read 1:4 as stored
    if (path == SBN_PATH_GEMV && it.tokens > 16) return SBN_EUNSUPPORTED;
    if ((path == SBN_PATH_GEMV || path == SBN_PATH_SMFMAC) && it.d_in % CHUNK != 0) return SBN_EUNSUPPORTED;
    if (path == SBN_PATH_DENSE_MFMA && it.d_in % 64 != 0) return SBN_EUNSUPPORTED;
    const size_t xq_bytes = align_up((size_t)it.tokens * it.d_in, 256);
    const size_t sx_bytes = align_up((size_t)it.tokens * sizeof(float), 256);
    if (activations_only) {
        const bool weights_as_stored = path == SBN_PATH_GENERIC ||
                                       ((path == SBN_PATH_SMFMAC || path == SBN_PATH_GEMV) && (is24 || pat.N == pat.M)) ||
                                       one4_decode;
        if (!weights_as_stored) return SBN_EUNSUPPORTED;
        if (ws_bytes < xq_bytes + sx_bytes) return SBN_ESIZE;
    } else if (ws_bytes < linear_workspace_bytes(it.tokens, it.d_out, it.d_in)) {
        return SBN_ESIZE;
    }
    // workspace: [xq int8 tokens*d_in][sx fp32 tokens][dense int8 W for the comparison path]
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    if (!it.xq) it.xq = reinterpret_cast<int8_t *>(ws);
    if (!it.sx) it.sx = reinterpret_cast<float *>(ws + xq_bytes);
    int8_t *w_dense = reinterpret_cast<int8_t *>(ws + xq_bytes + sx_bytes);

    sbn_status st = SBN_OK;
    // the decode path derives the quantized activations itself (inside its kernel when it can) unless the
    // caller wants them back in its own buffers
    const bool defer = path == SBN_PATH_GEMV && it.X && !it_in.xq && !it_in.sx;
    it.quantized = !defer;
    if (it.X && !defer) st = launch_act_quant(it.X, it.tokens, it.d_in, it.xq, it.sx, stream);
    if (st != SBN_OK) return st;
    if ((path == SBN_PATH_GEMV || path == SBN_PATH_SMFMAC) && !is24 && sparse_form && !one4_decode) {
        // an instance of 2:4: the dense-weight region of the workspace takes its 2:4 operand form (a quarter of the size)
        st = launch_repack_2of4(it.packed, it.d_out, it.d_in, pat, reinterpret_cast<uint8_t *>(w_dense), stream);
        if (st != SBN_OK) return st;
        it.packed = w_dense;
    }
    if ((path == SBN_PATH_GEMV || path == SBN_PATH_SMFMAC) && !sparse_form && pat.N != pat.M) {
        // no sparse instruction for this pattern: the kernels take dense 2-bit codes (N = M is stored that way already)
        st = launch_repack_dense_codes(it.packed, it.d_out, it.d_in, pat, reinterpret_cast<uint8_t *>(w_dense), stream);
        if (st != SBN_OK) return st;
        it.packed = w_dense;
    }
    switch (path) {
    case SBN_PATH_GEMV: return launch_gemv(1, &it, one4_decode ? GEMV_1OF4 : sparse_form ? GEMV_2OF4 : GEMV_DENSE, stream);
    case SBN_PATH_SMFMAC: return launch_gemm_smfmac(1, &it, !sparse_form, stream);
    case SBN_PATH_DENSE_MFMA: return launch_gemm_dense(it, pat, w_dense, stream);
    case SBN_PATH_GENERIC: return launch_linear_generic(it, pat, stream);
    default: return SBN_EINVAL;
    }
}

sbn_status sbn_sparse_ternary_linear(const void *X, int64_t tokens, int64_t d_in, int64_t d_out, int N, int M,
                                     const void *packed, const float *gamma, const float *bias, float *Y,
                                     int8_t *xq_out, float *sx_out, int32_t *acc_out, sbn_path path, void *workspace,
                                     size_t ws_bytes, void *stream)
{
    Pattern pat;
    if (!packed || !gamma || !Y || !workspace || tokens <= 0) return SBN_EINVAL;
    if (!X && (!xq_out || !sx_out)) return SBN_EINVAL;   // pre-quantized mode needs both inputs
    if (path < SBN_PATH_AUTO || path > SBN_PATH_GENERIC) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    if (tokens * d_out >= (int64_t)1 << 40) return SBN_EUNSUPPORTED;
    if (!aligned(X, 16) || !aligned(packed, 16) || !aligned(Y, 16) || !aligned(workspace, 256)) return SBN_EALIGN;
    if (xq_out && !aligned(xq_out, 16)) return SBN_EALIGN;
    if (acc_out && !aligned(acc_out, 16)) return SBN_EALIGN;
    if (d_in % 8 != 0) return SBN_EUNSUPPORTED;   // bf16 rows are read in 16-byte vectors
    LinearItem it{X, packed, gamma, bias, Y, xq_out, sx_out, acc_out, tokens, d_in, d_out};
    return linear_one(it, pat, path, workspace, ws_bytes, static_cast<hipStream_t>(stream));
}

// ---- the forward call for callers that cannot allocate --------------------------------------------------------
// Scratch of sbn_sparse_ternary_linear_static: int8 activations and per-token scales of one call.  Every GPU the
// library runs on holds its own copy of the array until the process ends.  In host code the array's name is
// only a handle: the device address is looked up once per device (that device current) and kept.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SBN_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
static std::atomic<void *> g_scratch_ptr[STATIC_MAX_DEVICES];

static sbn_status static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_hip_error(e, "hipGetDevice"); return SBN_EHIP; }
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) { g_last_error = "sbn_sparse_ternary_linear_static: device ordinal beyond 63"; return SBN_EUNSUPPORTED; }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy
        if (e != hipSuccess || !p) { set_hip_error(e, "hipGetSymbolAddress(scratch)"); return SBN_EHIP; }
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
    }
    *out = p;
    return SBN_OK;
}

sbn_status sbn_sparse_ternary_linear_static(const void *X, int64_t tokens, int64_t d_in, int64_t d_out, int N, int M,
                                            const void *packed, const float *gamma, const float *bias, float *Y,
                                            int8_t *xq_out, float *sx_out, int32_t *acc_out, sbn_path path, void *stream)
{
    Pattern pat;
    if (!packed || !gamma || !Y || tokens <= 0) return SBN_EINVAL;
    if (!X && (!xq_out || !sx_out)) return SBN_EINVAL;
    if (path < SBN_PATH_AUTO || path > SBN_PATH_GENERIC) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    if (tokens * d_out >= (int64_t)1 << 40) return SBN_EUNSUPPORTED;
    if (!aligned(X, 16) || !aligned(packed, 16) || !aligned(Y, 16)) return SBN_EALIGN;
    if (xq_out && !aligned(xq_out, 16)) return SBN_EALIGN;
    if (acc_out && !aligned(acc_out, 16)) return SBN_EALIGN;
    if (d_in % 8 != 0) return SBN_EUNSUPPORTED;
    const size_t need = align_up((size_t)tokens * d_in, 256) + align_up((size_t)tokens * sizeof(float), 256);
    if (need > STATIC_SCRATCH_BYTES) {
        g_last_error = "sbn_sparse_ternary_linear_static: tokens * d_in + 4 * tokens = " + std::to_string(need) +
                       " bytes of scratch needed, the library's buffer holds " + std::to_string(STATIC_SCRATCH_BYTES);
        return SBN_ESIZE;
    }
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != SBN_OK) return st;
    LinearItem it{X, packed, gamma, bias, Y, xq_out, sx_out, acc_out, tokens, d_in, d_out};
    return linear_one(it, pat, path, ws, STATIC_SCRATCH_BYTES, static_cast<hipStream_t>(stream), true);
}

sbn_status sbn_dense_ternary_linear(const int8_t *xq, const float *sx, int64_t tokens, int64_t d_in, int64_t d_out,
                                    const int8_t *W_eff, const float *gamma, const float *bias, float *Y,
                                    int32_t *acc_out, void *stream)
{
    if (!xq || !sx || !W_eff || !gamma || !Y || tokens <= 0 || d_in <= 0 || d_out <= 0) return SBN_EINVAL;
    if (d_in % 64 != 0 || tokens * d_out >= (int64_t)1 << 40 || d_out * d_in >= (int64_t)1 << 32 ||
        tokens * d_in >= (int64_t)1 << 32)
        return SBN_EUNSUPPORTED;
    if (!aligned(xq, 16) || !aligned(sx, 4) || !aligned(W_eff, 16) || !aligned(Y, 16) || (acc_out && !aligned(acc_out, 16)))
        return SBN_EALIGN;
    LinearItem it{nullptr, nullptr, gamma, bias, Y, const_cast<int8_t *>(xq), const_cast<float *>(sx), acc_out, tokens, d_in, d_out};
    return launch_gemm_dense_expanded(it, W_eff, static_cast<hipStream_t>(stream));
}

sbn_status sbn_sparse_ternary_linear_grouped(int count, const void *const *X, const int64_t *tokens,
                                             const int64_t *d_in, const int64_t *d_out, int N, int M,
                                             const void *const *packed, const float *const *gamma, float *const *Y,
                                             sbn_path path, void *workspace, size_t ws_bytes, void *stream)
{
    if (count <= 0 || count > 4096 || !X || !tokens || !d_in || !d_out || !packed || !gamma || !Y || !workspace)
        return SBN_EINVAL;
    if (path < SBN_PATH_AUTO || path > SBN_PATH_GENERIC) return SBN_EINVAL;
    if (!aligned(workspace, 256)) return SBN_EALIGN;
    Pattern pat;
    size_t need = 0;
    bool all_gemv = true, all_smfmac = true;
    for (int i = 0; i < count; ++i) {
        if (!X[i] || !packed[i] || !gamma[i] || !Y[i] || tokens[i] <= 0) return SBN_EINVAL;
        sbn_status st = check_shape(d_out[i], d_in[i], N, M, pat);
        if (st != SBN_OK) return st;
        if (!aligned(X[i], 16) || !aligned(packed[i], 16) || !aligned(Y[i], 16)) return SBN_EALIGN;
        if (d_in[i] % 8 != 0) return SBN_EUNSUPPORTED;
        need += linear_workspace_bytes(tokens[i], d_out[i], d_in[i]);
        const bool is24 = pat.N == 2 && pat.M == 4;
        const bool one4 = pat.N == 1 && pat.M == 4;
        if (resolve_path(path, tokens[i], d_in[i], pat) != SBN_PATH_GEMV || !(is24 || one4 || pat.N == pat.M) || tokens[i] > 16 ||
            d_in[i] % CHUNK != 0)
            all_gemv = false;   // one launch streams 2:4, 1:4 or dense-code (N = M) weights as stored; other patterns need a rewrite each
        if (resolve_path(path, tokens[i], d_in[i], pat) != SBN_PATH_SMFMAC || !(is24 || pat.N == pat.M) || d_in[i] % CHUNK != 0 ||
            tokens[i] * d_out[i] >= (int64_t)1 << 40)
            all_smfmac = false;
    }
    if (ws_bytes < need) return SBN_ESIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    if (!all_gemv && !all_smfmac) {
        // mixed paths: one enqueue per problem
        for (int i = 0; i < count; ++i) {
            LinearItem it{X[i], packed[i], gamma[i], nullptr, Y[i], nullptr, nullptr, nullptr, tokens[i], d_in[i], d_out[i]};
            const size_t wsz = linear_workspace_bytes(tokens[i], d_out[i], d_in[i]);
            sbn_status st = linear_one(it, pat, path, ws, wsz, s);
            if (st != SBN_OK) return st;
            ws += wsz;
        }
        return SBN_OK;
    }
    static thread_local std::vector<LinearItem> tl_items;   // host-side descriptor list, reused between calls
    tl_items.resize(count);
    for (int i = 0; i < count; ++i) {
        LinearItem &it = tl_items[i];
        it = LinearItem{X[i], packed[i], gamma[i], nullptr, Y[i], nullptr, nullptr, nullptr, tokens[i], d_in[i], d_out[i]};
        it.xq = reinterpret_cast<int8_t *>(ws);
        it.sx = reinterpret_cast<float *>(ws + align_up((size_t)tokens[i] * d_in[i], 256));
        ws += linear_workspace_bytes(tokens[i], d_out[i], d_in[i]);
        // identical X pointers share one quantization
        bool shared = false;
        for (int j = 0; j < i && !shared; ++j)
            if (X[j] == X[i] && tokens[j] == tokens[i] && d_in[j] == d_in[i]) {
                it.xq = tl_items[j].xq;
                it.sx = tl_items[j].sx;
                shared = true;
            }
        it.quantized = !all_gemv;   // the decode path derives the quantized activations itself
        if (!shared && !all_gemv) {
            sbn_status st = launch_act_quant(it.X, it.tokens, it.d_in, it.xq, it.sx, s);
            if (st != SBN_OK) return st;
        }
    }
    return all_gemv ? launch_gemv(count, tl_items.data(), pat.N == pat.M ? GEMV_DENSE : pat.M == 4 && pat.N == 1 ? GEMV_1OF4 : GEMV_2OF4, s)
                    : launch_gemm_smfmac(count, tl_items.data(), pat.N == pat.M, s);
}

sbn_status sbn_sparse_ternary_linear_backward(const void *dY, int64_t tokens, int64_t d_in, int64_t d_out, int N,
                                              int M, const void *packed, const float *gamma, const int8_t *xq,
                                              const float *sx, void *dX, void *dW, int flags, void *workspace,
                                              size_t ws_bytes, void *stream)
{
    Pattern pat;
    if (!dY || !workspace || tokens <= 0 || (!dX && !dW)) return SBN_EINVAL;
    if (dX && (!packed || !gamma)) return SBN_EINVAL;
    if (dW && (!xq || !sx)) return SBN_EINVAL;
    if (flags & ~(SBN_BWD_ACCUMULATE | SBN_BWD_MASK_DW)) return SBN_EINVAL;
    if ((flags & SBN_BWD_MASK_DW) && dW && !packed) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    if (!aligned(dY, 16) || !aligned(workspace, 256)) return SBN_EALIGN;
    if ((dX && !aligned(dX, 16)) || (dW && !aligned(dW, 16)) || (xq && !aligned(xq, 16))) return SBN_EALIGN;
    if (d_in % 8 != 0 || d_out % 8 != 0) return SBN_EUNSUPPORTED;
    if (ws_bytes < backward_workspace_bytes(tokens, d_out, d_in)) return SBN_ESIZE;
    return launch_backward(dY, tokens, d_in, d_out, pat, packed, gamma, xq, sx, dX, dW, flags, workspace,
                           ws_bytes, static_cast<hipStream_t>(stream));
}

sbn_status sbn_sparse_ternary_linear_backward_grouped(int count, const void *const *dY, const int64_t *tokens,
                                                      const int64_t *d_in, const int64_t *d_out, int N, int M,
                                                      const void *const *packed, const float *const *gamma,
                                                      const int8_t *const *xq, const float *const *sx, void *const *dX,
                                                      void *const *dW, int flags, void *workspace, size_t ws_bytes,
                                                      void *stream)
{
    if (count <= 0 || count > SBN_BACKWARD_GROUP_MAX) return SBN_EINVAL;
    if (!dY || !tokens || !d_in || !d_out || !packed || !gamma || !xq || !sx || !dX || !dW || !workspace) return SBN_EINVAL;
    if (flags & ~(SBN_BWD_ACCUMULATE | SBN_BWD_MASK_DW)) return SBN_EINVAL;
    if (!aligned(workspace, 256)) return SBN_EALIGN;
    Pattern pat;
    BackwardItem items[SBN_BACKWARD_GROUP_MAX];
    size_t used = 0;
    for (int i = 0; i < count; ++i) {
        if (!dY[i] || tokens[i] <= 0 || (!dX[i] && !dW[i])) return SBN_EINVAL;
        if (dX[i] && (!packed[i] || !gamma[i])) return SBN_EINVAL;
        if (dW[i] && (!xq[i] || !sx[i])) return SBN_EINVAL;
        if ((flags & SBN_BWD_MASK_DW) && dW[i] && !packed[i]) return SBN_EINVAL;
        sbn_status st = check_shape(d_out[i], d_in[i], N, M, pat);
        if (st != SBN_OK) return st;
        if (!aligned(dY[i], 16) || (dX[i] && !aligned(dX[i], 16)) || (dW[i] && !aligned(dW[i], 16)) || (xq[i] && !aligned(xq[i], 16)))
            return SBN_EALIGN;
        if (d_in[i] % 8 != 0 || d_out[i] % 8 != 0) return SBN_EUNSUPPORTED;
        items[i] = BackwardItem{dY[i], tokens[i], d_in[i], d_out[i], packed[i], gamma[i], xq[i], sx[i], dX[i], dW[i],
                                static_cast<uint8_t *>(workspace) + used};
        used += backward_workspace_bytes(tokens[i], d_out[i], d_in[i]);
        if (used > ws_bytes) return SBN_ESIZE;
    }
    return launch_backward_grouped(count, items, pat, flags, static_cast<hipStream_t>(stream));
}

sbn_status sbn_mask_flips(const void *packed_a, const void *packed_b, int64_t d_out, int64_t d_in, int N, int M,
                          uint64_t *flips_out, void *workspace, size_t ws_bytes, void *stream)
{
    Pattern pat;
    if (!packed_a || !packed_b || !flips_out || !workspace) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    if (!aligned(packed_a, 16) || !aligned(packed_b, 16) || !aligned(flips_out, 8) || !aligned(workspace, 256)) return SBN_EALIGN;
    if (ws_bytes < mask_flips_workspace_bytes(d_out, d_in, M)) return SBN_ESIZE;
    return launch_mask_flips(packed_a, packed_b, d_out, d_in, pat, flips_out, workspace, static_cast<hipStream_t>(stream));
}

sbn_status sbn_convert_packed(const void *packed, int64_t d_out, int64_t d_in, int N, int M, int to_N, int to_M, void *out,
                              void *stream)
{
    Pattern pat, to;
    if (!packed || !out) return SBN_EINVAL;
    sbn_status st = check_shape(d_out, d_in, N, M, pat);
    if (st != SBN_OK) return st;
    st = check_shape(d_out, d_in, to_N, to_M, to);
    if (st != SBN_OK) return st;
    if (!aligned(packed, 16) || !aligned(out, 16)) return SBN_EALIGN;
    if (d_in % CHUNK != 0 || (N == to_N && M == to_M)) return SBN_EUNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (to_N == 2 && to_M == 4 && embeds_in_2of4(pat)) return launch_repack_2of4(packed, d_out, d_in, pat, static_cast<uint8_t *>(out), s);
    if (to_N == to_M) return launch_repack_dense_codes(packed, d_out, d_in, pat, static_cast<uint8_t *>(out), s);
    return SBN_EUNSUPPORTED;
}

}  // extern "C"
