// Device-side helpers shared by the HIP kernels of the verification library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quasar {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTileRows = 16;      // weight rows per packed tile (one MFMA A operand height)
constexpr int kStepBytes = 1024;   // one wave-wide 128-bit load = one packed step
constexpr int kStepK8 = 64;        // k extent of an int8 step (16 rows x 64 k x 1 B)
constexpr int kStepK16 = 32;       // k extent of a bf16 step  (16 rows x 32 k x 2 B)

__device__ __forceinline__ float bf16_bits_to_float(unsigned int b) {
    return __uint_as_float(b << 16);
}

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN
__device__ __forceinline__ unsigned int float_to_bf16_bits(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// Wait for this wave's LDS traffic, then meet the other waves of the workgroup.
// Outstanding global loads stay in flight across the barrier (the weight ring
// must not be drained by a workgroup-scope fence).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Two dwords of int8 codes (8 codes) -> 8 bf16 values, exactly (|code| <= 127 fits 8 bits
// of significand).  One sign-extending byte-select convert per code, then the high
// halves of two fp32 words are merged by a byte permute (truncation is exact).
__device__ __forceinline__ bf16x8 codes_to_bf16x8(unsigned int lo, unsigned int hi) {
    float f0 = (float)(signed char)(lo & 0xff);
    float f1 = (float)(signed char)((lo >> 8) & 0xff);
    float f2 = (float)(signed char)((lo >> 16) & 0xff);
    float f3 = (float)(signed char)(lo >> 24);
    float f4 = (float)(signed char)(hi & 0xff);
    float f5 = (float)(signed char)((hi >> 8) & 0xff);
    float f6 = (float)(signed char)((hi >> 16) & 0xff);
    float f7 = (float)(signed char)(hi >> 24);
    u32x4 r;
    r.x = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
    r.y = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
    r.z = __builtin_amdgcn_perm(__float_as_uint(f5), __float_as_uint(f4), 0x07060302u);
    r.w = __builtin_amdgcn_perm(__float_as_uint(f7), __float_as_uint(f6), 0x07060302u);
    return __builtin_bit_cast(bf16x8, r);
}

// Monotone map fp32 -> u32 (larger float => larger key); -0 and +0 map apart but adjacent.
__device__ __forceinline__ unsigned int float_order_key(float f) {
    unsigned int u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// (value, index) packed so that an unsigned 64-bit max picks the larger value and,
// on equal values, the smaller index.
__device__ __forceinline__ unsigned long long argmax_key(float v, unsigned int idx) {
    return ((unsigned long long)float_order_key(v) << 32) | (unsigned long long)(0xFFFFFFFFu - idx);
}
__device__ __forceinline__ unsigned int argmax_key_index(unsigned long long key) {
    return 0xFFFFFFFFu - (unsigned int)(key & 0xFFFFFFFFull);
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int mask) {
    unsigned int lo = (unsigned int)v, hi = (unsigned int)(v >> 32);
    lo = __shfl_xor(lo, mask, 64);
    hi = __shfl_xor(hi, mask, 64);
    return ((unsigned long long)hi << 32) | lo;
}

// floor(T * b / G) for wave-uniform non-negative operands: where a workgroup's share of T tiles
// begins.  The 64-bit division is a long software routine; it runs only when the product does
// not fit 32 bits.
__device__ __forceinline__ int tile_split(int T, int b, int G) {
    const unsigned long long prod = (unsigned long long)(unsigned int)T * (unsigned int)b;
    if (prod <= 0xFFFFFFFFull) return (int)((unsigned int)prod / (unsigned int)G);
    return (int)(prod / (unsigned long long)(unsigned int)G);
}

// 16 bytes per lane from gbase + lane_offset (gbase wave-uniform) straight into LDS at lds_addr + 16 * lane,
// without passing through registers.  Inline assembly on purpose: when the compiler sees a direct-to-LDS
// load anywhere in a kernel it makes every LDS read wait for ALL outstanding vector memory loads (it
// cannot tell which loads write LDS), which would drain the weight ring at every slot.  The caller waits
// for these loads explicitly (vmcnt(0)) before anybody reads the bytes.
__device__ __forceinline__ void load_to_lds_16(unsigned long long gbase, unsigned int lane_offset, unsigned int lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(gbase), "s"(lds_addr)
                 : "memory");   // (M0 is reserved: the compiler keeps nothing in it across statements)
}
__device__ __forceinline__ unsigned int lds_address_of(const unsigned char *p) {
    return __builtin_amdgcn_readfirstlane(
        (unsigned int)(unsigned long long)((const __attribute__((address_space(3))) unsigned char *)p));
}


}  // namespace quasar
