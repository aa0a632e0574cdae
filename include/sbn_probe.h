/*
 * sbn_probe.h - C ABI of libsbn_probe: ceiling probes for the benchmark of libsbn (AMD MI355X, gfx950).
 *
 * Measurement support only, no step of the layer and not part of libsbn: a probe enqueues one kernel that
 * issues a single kind of work at full rate, so that a benchmark can state the rate this board sustains next
 * to the datasheet peak it divides by.  Matrix kinds run `iters` rounds of 16 matrix instructions per
 * wavefront on random operands (with constant operands the same loop runs at a much higher clock: the part
 * is power-managed, and the layer's operands are not constant), two wavefronts per SIMD; stream kinds read
 * or write `bytes` - 256 bytes of `buf` once; the LDS kind runs `iters` rounds of 16 conflict-free 16-byte
 * LDS reads per lane, two wavefronts per SIMD.
 *   buf       device, >= 256 bytes (stream kinds: >= 1 MiB), 256-byte aligned; matrix and LDS kinds touch
 *             only its first word
 *   work_out  HOST, the operations (2 per multiply-add, dense-equivalent for the sparse instruction) or
 *             bytes one call performs
 *   stream    hipStream_t as void*, NULL = the default stream
 * Returns 0, -1 (bad argument: null pointer, unknown kind, iters <= 0, buffer too small), -4 (buf not
 * 256-byte aligned) or -5 (a HIP call failed).  Never allocates or synchronises.
 */
#ifndef SBN_PROBE_H
#define SBN_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SBN_CEIL_SMFMAC_I8 = 0,  /* v_smfmac_i32_32x32x64_i8, ternary A, int8 B */
    SBN_CEIL_MFMA_I8 = 1,    /* v_mfma_i32_32x32x32_i8 */
    SBN_CEIL_MFMA_BF16 = 2,  /* v_mfma_f32_32x32x16_bf16 */
    SBN_CEIL_HBM_READ = 3,
    SBN_CEIL_HBM_WRITE = 4,
    SBN_CEIL_LDS_READ = 5    /* ds_read_b128 */
} sbn_ceiling;

int sbn_ceiling_probe(int kind, void *buf, size_t bytes, int iters, double *work_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SBN_PROBE_H */
