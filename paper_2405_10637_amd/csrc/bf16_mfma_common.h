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

__device__ __forceinline__ float xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask, 64)); }

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
