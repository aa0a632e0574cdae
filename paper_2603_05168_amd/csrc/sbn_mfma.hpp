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
// and 13 is the constant 0xff; mask and OR are one v_and_or_b32 (mask in a scalar register,
// 0x01010101 in the vector register `ones`).  Nine VALU operations per 16 values; VALU work does
// not overlap matrix instructions on this part (measured: their times add), so every operation
// saved here is matrix-pipe time gained.
__device__ __forceinline__ uint32_t vgpr_ones()
{
    uint32_t ones;
    asm volatile("v_mov_b32 %0, 0x01010101" : "=v"(ones));   // opaque, so that it stays in a vector register
    return ones;
}

__device__ __forceinline__ v4i expand_codes(uint32_t cw, uint32_t ones)
{
    const uint32_t lut = 0xff000100u;
    const uint32_t t = cw >> 4;
    uint32_t s1, s3;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(s1) : "v"(cw), "s"(0x0c0c0c0cu), "v"(ones));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(s3) : "v"(t), "s"(0x0c0c0c0cu), "v"(ones));
    v4i a;
    a[0] = (int)__builtin_amdgcn_perm(lut, lut, cw & 0x03030303u);
    a[1] = (int)__builtin_amdgcn_perm(0x00000100u, 0u, s1);
    a[2] = (int)__builtin_amdgcn_perm(lut, lut, t & 0x03030303u);
    a[3] = (int)__builtin_amdgcn_perm(0x00000100u, 0u, s3);
    return a;
}

// Two words of dense 2-bit codes (32 consecutive weights = 8 groups of four; weight 16 w + 4 p + b of word w at bits
// [8 b + 2 p, +2)) -> the operands of two sparse matrix instructions: a01 holds positions 0, 1 of every group, a23
// positions 2, 3, in the byte order of expand_codes (group 2 j in bytes 0, 1 of register j, group 2 j + 1 in bytes 2, 3).
__device__ __forceinline__ void expand_dense_codes(uint32_t w0, uint32_t w1, v4i &a01, v4i &a23)
{
    const uint32_t lut = 0xff000100u, m = 0x03030303u;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t w = i ? w1 : w0;
        const uint32_t lo = w & 0xffffu, hi = w >> 16;
        const uint32_t tl = (lo << 14) | lo, th = (hi << 14) | hi;   // bytes 0, 1 of pair p and, 16 bits up, of pair p + 1
        a01[2 * i] = (int)__builtin_amdgcn_perm(lut, lut, tl & m);
        a01[2 * i + 1] = (int)__builtin_amdgcn_perm(lut, lut, (tl >> 4) & m);
        a23[2 * i] = (int)__builtin_amdgcn_perm(lut, lut, th & m);
        a23[2 * i + 1] = (int)__builtin_amdgcn_perm(lut, lut, (th >> 4) & m);
    }
}

// One index word and one code word of the 1:4 packed form (16 slots = 64 consecutive weights: slot s keeps position
// bits [2s, 2s+2) of `iw14` in its group of four and has its code at bits [8(s%4) + 2(s/4), +2) of `cw14`) -> the
// operands of two sparse matrix instructions (32 weights each), built in registers.  A group with one kept weight
// at position p becomes the 2:4 group that keeps the aligned pair holding p - positions (0, 1) or (2, 3), index
// nibble 0x4 or 0xe - with the code in slot p & 1 and code 0 in the other slot, so positions stay ascending.
//   index:  bit 1 of every position selects the nibble (a byte-wise table lookup on pairs of groups);
//   codes:  a mask of the odd positions in the code word's own layout (one 24-bit multiply per byte of positions
//           moves bit 2b of the byte to bit 8b) splits the code word into the codes bound for slot 0 and those
//           bound for slot 1; two byte permutes interleave the two words byte by byte into the order of the
//           instruction's A registers, and the table lookups of expand_codes finish the job.
// About 25 vector operations per instruction against 9 for the 2:4 form.
__device__ __forceinline__ void expand_1of4(uint32_t iw14, uint32_t cw14, uint32_t ones, uint32_t (&iw)[2], v4i (&a)[2])
{
    const uint32_t lut = 0xff000100u;
    const uint32_t odd = iw14 & 0x55555555u;
    // (the multiply is written out: left to itself the compiler folds the later shift into the constant, which then
    // no longer fits 24 bits and costs a full-width multiply at a quarter of the rate)
    uint32_t e1 = 0;
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        uint32_t m;
        asm("v_mul_u32_u24 %0, %1, %2" : "=v"(m) : "s"(0x41041u), "v"((odd >> (8 * f)) & 0x55u));
        e1 |= (m & 0x01010101u) << (2 * f);
    }
    const uint32_t c_odd = cw14 & (e1 | (e1 << 1)), c_even = cw14 ^ c_odd;
    // bytes: (slot-0 codes of groups b, slot-1 codes of groups b) for b = 0, 1 and for b = 2, 3
    const uint32_t y0 = __builtin_amdgcn_perm(c_odd, c_even, 0x05010400u), y1 = __builtin_amdgcn_perm(c_odd, c_even, 0x07030602u);
    const uint32_t hi = (iw14 >> 1) & 0x55555555u;   // a nibble = bit 1 of two positions, at its bits 0 and 2
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        // the four nibbles of this half go to the low halves of four bytes; as selector bytes (0, 1, 4 or 5) they look
        // up the two index nibbles of their groups: 0x4 for the pair (0, 1), 0xe for (2, 3)
        uint32_t x = q ? hi >> 16 : hi & 0xffffu;
        x = (x | (x << 8)) & 0x00ff00ffu;
        x = (x | (x << 4)) & 0x0f0f0f0fu;
        iw[q] = __builtin_amdgcn_perm(0x0000eee4u, 0x00004e44u, x);
        const uint32_t z0 = q ? y0 >> 4 : y0, z1 = q ? y1 >> 4 : y1;
        uint32_t s2, s3;
        asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(s2) : "v"(z0), "s"(0x0c0c0c0cu), "v"(ones));
        asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(s3) : "v"(z1), "s"(0x0c0c0c0cu), "v"(ones));
        a[q][0] = (int)__builtin_amdgcn_perm(lut, lut, z0 & 0x03030303u);
        a[q][1] = (int)__builtin_amdgcn_perm(lut, lut, z1 & 0x03030303u);
        a[q][2] = (int)__builtin_amdgcn_perm(0x00000100u, 0u, s2);
        a[q][3] = (int)__builtin_amdgcn_perm(0x00000100u, 0u, s3);
    }
}

// One LDS-DMA load: lane l of the wavefront fetches 16 bytes at base + voff and the hardware
// deposits them at LDS byte address lds_addr + 16*l (M0 carries the LDS address).  Written as
// inline assembly on purpose: after the compiler's own LDS-DMA builtin every later LDS read is
// preceded by a wait for ALL outstanding vector-memory operations (it cannot tell which LDS bytes
// a DMA writes), which serialises the prefetch ring with the loads it has just issued.  With the
// load opaque to the compiler the kernels that use it count the outstanding DMA operations themselves
// (SBN_WAIT_VMCNT) and order LDS reads against them with the block barrier.
__device__ __forceinline__ void lds_dma16(const void *base, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}

// the same with one dword per lane: lane l deposits its 4 bytes at lds_addr + 4*l
__device__ __forceinline__ void lds_dma4(const void *base, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// wait until at most n vector-memory operations of this wavefront are outstanding (gfx9 encoding:
// vmcnt in bits [3:0] and [15:14]; expcnt and lgkmcnt fields left at "no wait")
#define SBN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | (((n) >> 4) << 14) | 0x0f70)

}  // namespace sbn
