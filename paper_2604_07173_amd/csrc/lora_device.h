// Device-side helpers shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define LORA_GLOBAL __attribute__((address_space(1)))

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// 16-byte accesses through pointers that are known to be global memory.  A pointer read
// from the unit table has no address space the compiler can see, and a generic ("flat")
// access forces it to drain every outstanding load before the next use; saying "global"
// keeps prefetched loads in flight.
template <bool NT>
__device__ inline u32x4 ld16(const void *p)
{
    const LORA_GLOBAL u32x4 *q = (const LORA_GLOBAL u32x4 *)p;
    return NT ? __builtin_nontemporal_load(q) : *q;
}

template <bool NT>
__device__ inline void st16(void *p, u32x4 v)
{
    LORA_GLOBAL u32x4 *q = (LORA_GLOBAL u32x4 *)p;
    if (NT) __builtin_nontemporal_store(v, q);
    else *q = v;
}

__device__ inline f32x4 ld16f(const float *p) { return *(const LORA_GLOBAL f32x4 *)p; }
__device__ inline void st16f(float *p, f32x4 v) { *(LORA_GLOBAL f32x4 *)p = v; }

// two fp32 -> packed bf16 pair (first argument in bits 15:0), round to nearest even, in
// hardware (v_cvt_pk_bf16_f32)
__device__ inline unsigned pack_bf16_rne(float lo, float hi)
{
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

}  // namespace lora
