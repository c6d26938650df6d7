// Vector types and small helpers shared by the bf16 matrix-core kernels (decode and prefill attention).
#pragma once

#include "lckv_internal.h"

namespace lckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float floatx2;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kNegInf = -__builtin_huge_valf();

// Reductions over the four lanes c, c+16, c+32, c+48 that hold one tile column (its four key quads), result in all
// four.  v_permlane16_swap / v_permlane32_swap (new on gfx950) exchange 16- and 32-lane halves of two registers
// inside the vector ALU: with both registers holding x, afterwards one holds x with its odd 16-lane rows replaced
// by the even ones and the other the reverse (then the same for the 32-lane halves) - a butterfly without the LDS
// round trip a ds_bpermute shuffle costs.  Written as inline assembly with both registers as read-write operands:
// the compiler's builtin for it folded max(result0, result1) into result0 (hipcc 7.2), which is wrong; the
// s_nop pads cover the wait states between a vector-ALU write and this instruction's read, which the compiler
// does not insert inside an asm block.
__device__ __forceinline__ void swap_rows16(float &a, float &b) {
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap_halves32(float &a, float &b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float column_max4(float v) {
    float a = v, b = v;
    swap_rows16(a, b);
    a = b = fmaxf(a, b);
    swap_halves32(a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float column_sum4(float v) {
    float a = v, b = v;
    swap_rows16(a, b);
    a = b = a + b;
    swap_halves32(a, b);
    return a + b;
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    floatx2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));  // v_cvt_pk_bf16_f32, RNE
}

template <bool NT>
__device__ __forceinline__ u32x4 load16(const char *p) {
    // NT: the nontemporal hint.  A stream that is read once and is far larger than the caches is fetched
    // measurably faster with it on MI355X (about 7.1 instead of 6.3 TB/s for a pure read).
    return NT ? __builtin_nontemporal_load((const u32x4 *)p) : *(const u32x4 *)p;
}

}  // namespace lckv
