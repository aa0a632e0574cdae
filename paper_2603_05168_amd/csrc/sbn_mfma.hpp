// Register-level helpers for the CDNA4 matrix instructions used by libsbn.
//
// Operand layouts (measured on gfx950 with one-hot operands, then checked with random data):
//   v_mfma_i32_32x32x32_i8 / v_mfma_i32_16x16x64_i8 (R = 32 / 16 rows):
//       A lane l: row l % R, k = 16 * (l / R) + byte;   B lane l: column l % R, same k
//   v_smfmac_i32_32x32x64_i8 / v_smfmac_i32_16x16x128_i8 (A is 2:4 compressed):
//       A lane l: row l % R, 16 kept values of the 32 consecutive k starting at 32 * (l / R);
//                 values 2t and 2t+1 belong to the group of four k = 32*(l/R) + 4t .. +3 and sit at the
//                 positions given by bits [4t, 4t+2) and [4t+2, 4t+4) of the lane's index register
//       B lane l: column l % R; bytes 0..15 = k 16*(l/R) + 0..15, bytes 16..31 = k Khalf + 16*(l/R) + 0..15
//                 with Khalf = 32 (32x32x64) or 64 (16x16x128)
//   accumulators: 16x16: lane l holds column l % 16, rows 4*(l/16) + i;
//                 32x32: lane l holds column l % 32, rows 8*(i/4) + 4*(l/32) + i%4
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// 16 two-bit ternary codes of one code word -> 16 int8 values in 4 registers.  The code of value v
// sits at bits 8*(v%4) + 2*(v/4), so register q is a byte-wise table lookup (v_perm_b32) of the
// bit pairs 2q, 2q+1 of every byte: code 0 -> 0x00, 1 -> 0x01, 3 -> 0xff.
// v_perm_b32 selector bytes: 0..3 pick a byte of the second source, 4..7 of the first, 12 gives
// 0x00 and 13 or more 0xff.  Even q: selector = code (0, 1, 3).  Odd q: selector = code << 2 | 1
// (1, 5, 13), which needs no shift: byte 1 of the second source is 0x00, byte 1 of the first 0x01,
// and 13 is the constant 0xff.  Nine VALU operations per 16 values.
__device__ __forceinline__ v4i expand_codes(uint32_t cw)
{
    const uint32_t lut = 0xff000100u;
    const uint32_t t = cw >> 4;
    v4i a;
    a[0] = (int)__builtin_amdgcn_perm(lut, lut, cw & 0x03030303u);
    a[1] = (int)__builtin_amdgcn_perm(0x00000100u, 0u, (cw & 0x0c0c0c0cu) | 0x01010101u);
    a[2] = (int)__builtin_amdgcn_perm(lut, lut, t & 0x03030303u);
    a[3] = (int)__builtin_amdgcn_perm(0x00000100u, 0u, (t & 0x0c0c0c0cu) | 0x01010101u);
    return a;
}

}  // namespace sbn
