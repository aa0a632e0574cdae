// Ceiling probes: kernels that issue one kind of work and nothing else, so that a benchmark can put
// the rate this board sustains next to the datasheet peak it divides by.  Matrix probes use random
// operands on purpose: with constant operands the same loop runs at a much higher clock (the part is
// power-managed), and the layer's operands are not constant.  Measurement support, not on the path
// of Section 2.2.  Built into libsbn_probe.so, apart from the layer's library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sbn_probe.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

constexpr int PROBE_MMA_PER_ITER = 16;

// KIND 0: v_smfmac_i32_32x32x64_i8 (ternary A, int8 B, random index words); 1: v_mfma_i32_32x32x32_i8;
// 2: v_mfma_f32_32x32x16_bf16.  Four operand sets, four independent accumulators.
template <int KIND>
__global__ void __launch_bounds__(256) probe_mma_kernel(int iters, int *sink)
{
    const uint32_t t = threadIdx.x + blockIdx.x * 256u;
    uint32_t ra[4][8], rb[4][8];
    for (int s = 0; s < 4; ++s)
        for (int i = 0; i < 8; ++i) {
            uint32_t a = mix32(t * 64u + s * 16u + i), b = mix32(t * 64u + s * 16u + 8u + i);
            if (KIND == 0) {   // ternary bytes
                uint32_t o = 0;
                for (int k = 0; k < 4; ++k) {
                    const uint32_t c = ((a >> (8 * k)) & 0xffu) % 3u;
                    o |= (c == 0 ? 0u : c == 1 ? 1u : 0xffu) << (8 * k);
                }
                a = o;
            }
            if (KIND == 2) {   // finite bf16 pairs in [0.5, 1) with random signs
                a = (a & 0x807f807fu) | 0x3f003f00u;
                b = (b & 0x807f807fu) | 0x3f003f00u;
            }
            ra[s][i] = a;
            rb[s][i] = b;
        }
    int acc_fold = 0;
    if constexpr (KIND == 2) {
        v16f c[4] = {};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                v8bf a, b[4];
                __builtin_memcpy(&a, ra[s], 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) __builtin_memcpy(&b[q], rb[(s + q) & 3], 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) c[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[q], c[q], 0, 0, 0);
            }
        }
        for (int q = 0; q < 4; ++q)
            for (int i = 0; i < 16; ++i) acc_fold ^= __float_as_int(c[q][i]);
    } else {
        v16i c[4] = {};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const v4i a = {(int)ra[s][0], (int)ra[s][1], (int)ra[s][2], (int)ra[s][3]};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t *pb = rb[(s + q) & 3];
                    if constexpr (KIND == 0) {
                        const v8i b = {(int)pb[0], (int)pb[1], (int)pb[2], (int)pb[3], (int)pb[4], (int)pb[5], (int)pb[6], (int)pb[7]};
                        c[q] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(a, b, c[q], (int)ra[s][4], 0, 0);
                    } else {
                        const v4i b = {(int)pb[0], (int)pb[1], (int)pb[2], (int)pb[3]};
                        c[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c[q], 0, 0, 0);
                    }
                }
            }
        }
        for (int q = 0; q < 4; ++q)
            for (int i = 0; i < 16; ++i) acc_fold ^= c[q][i];
    }
    if (acc_fold == 0x5a17c0de) *sink = acc_fold;   // keeps the loop alive; practically never taken
}

// contiguous 16-byte loads, eight in flight per lane; every block walks its own slice of the buffer
__global__ void __launch_bounds__(256) probe_read_kernel(const uint4 *buf, int64_t nvec, int *sink)
{
    const int64_t per_block = nvec / gridDim.x;
    const uint4 *p = buf + per_block * blockIdx.x;
    uint4 x = make_uint4(0, 0, 0, 0);
    int64_t i = threadIdx.x;
    for (; i + 7 * 256 < per_block; i += 8 * 256) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[i + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) { x.x ^= v[u].x; x.y ^= v[u].y; x.z ^= v[u].z; x.w ^= v[u].w; }
    }
    for (; i < per_block; i += 256) { const uint4 v = p[i]; x.x ^= v.x; x.y ^= v.y; x.z ^= v.z; x.w ^= v.w; }
    if ((x.x ^ x.y ^ x.z ^ x.w) == 0x5a17c0deu) *sink = 1;
}

__global__ void __launch_bounds__(256) probe_write_kernel(uint4 *buf, int64_t nvec)
{
    const int64_t per_block = nvec / gridDim.x;
    uint4 *p = buf + per_block * blockIdx.x;
    const uint4 v = make_uint4(threadIdx.x, blockIdx.x, 3u, 4u);
    for (int64_t i = threadIdx.x; i < per_block; i += 256) p[i] = v;
}

// 16 LDS reads of 16 bytes per lane and round, consecutive lanes at consecutive addresses (no bank conflicts);
// the addresses move by 16 bytes per round so that no read can be taken out of the loop.  64 KB per block, two blocks
// per multiprocessor = two wavefronts per SIMD, as in the matrix kernels.
constexpr int PROBE_LDS_BYTES = 64 * 1024;
constexpr int PROBE_LDS_READS = 16;
__global__ void __launch_bounds__(256, 2) probe_lds_kernel(int iters, int *sink)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[PROBE_LDS_BYTES];
    for (int i = threadIdx.x; i < PROBE_LDS_BYTES / 16; i += 256)
        reinterpret_cast<uint4 *>(lds)[i] = make_uint4(mix32(i), mix32(i + 77u), blockIdx.x, threadIdx.x);
    __syncthreads();
    uint4 x = make_uint4(0, 0, 0, 0);
    for (int it = 0; it < iters; ++it) {
        uint4 v[PROBE_LDS_READS];
#pragma unroll
        for (int j = 0; j < PROBE_LDS_READS; ++j)
            v[j] = *reinterpret_cast<const uint4 *>(lds + (((threadIdx.x + it) * 16) & 4095) + j * 4096);
#pragma unroll
        for (int j = 0; j < PROBE_LDS_READS; ++j) { x.x ^= v[j].x; x.y ^= v[j].y; x.z ^= v[j].z; x.w ^= v[j].w; }
    }
    if ((x.x ^ x.y ^ x.z ^ x.w) == 0x5a17c0deu) *sink = 1;
}

int multiprocessors()
{
    int dev = 0, cus = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
    return cus > 0 ? cus : 256;
}

}  // namespace

extern "C" int sbn_ceiling_probe(int kind, void *buf, size_t bytes, int iters, double *work_out, void *stream_)
{
    if (!buf || !work_out || kind < SBN_CEIL_SMFMAC_I8 || kind > SBN_CEIL_LDS_READ) return -1;
    if (reinterpret_cast<uintptr_t>(buf) % 256 != 0) return -4;
    const bool streams = kind == SBN_CEIL_HBM_READ || kind == SBN_CEIL_HBM_WRITE;
    if (streams ? bytes < ((size_t)1 << 20) : (iters <= 0 || bytes < 256)) return -1;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    static thread_local int cus = 0;
    if (cus == 0) cus = multiprocessors();
    int *sink = static_cast<int *>(buf);
    if (kind <= SBN_CEIL_MFMA_BF16) {
        const int blocks = 2 * cus;   // two wavefronts per SIMD
        const double per_mma = kind == SBN_CEIL_SMFMAC_I8 ? 2.0 * 32 * 32 * 64 : kind == SBN_CEIL_MFMA_I8 ? 2.0 * 32 * 32 * 32 : 2.0 * 32 * 32 * 16;
        *work_out = per_mma * PROBE_MMA_PER_ITER * (double)iters * 4.0 * blocks;
        if (kind == SBN_CEIL_SMFMAC_I8) hipLaunchKernelGGL(probe_mma_kernel<0>, dim3(blocks), dim3(256), 0, stream, iters, sink);
        else if (kind == SBN_CEIL_MFMA_I8) hipLaunchKernelGGL(probe_mma_kernel<1>, dim3(blocks), dim3(256), 0, stream, iters, sink);
        else hipLaunchKernelGGL(probe_mma_kernel<2>, dim3(blocks), dim3(256), 0, stream, iters, sink);
    } else if (kind == SBN_CEIL_LDS_READ) {
        const int blocks = 2 * cus;
        *work_out = 16.0 * PROBE_LDS_READS * 256.0 * (double)iters * blocks;
        hipLaunchKernelGGL(probe_lds_kernel, dim3(blocks), dim3(256), 0, stream, iters, sink);
    } else {
        const int blocks = 8 * cus;
        const int64_t nvec = (int64_t)((bytes - 256) / 16) / blocks * blocks;
        *work_out = (double)nvec * 16.0;
        uint4 *data = reinterpret_cast<uint4 *>(static_cast<uint8_t *>(buf) + 256);   // the first 256 bytes hold the sink
        if (kind == SBN_CEIL_HBM_READ) hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, stream, data, nvec, sink);
        else hipLaunchKernelGGL(probe_write_kernel, dim3(blocks), dim3(256), 0, stream, data, nvec);
    }
    return hipGetLastError() == hipSuccess ? 0 : -5;
}
