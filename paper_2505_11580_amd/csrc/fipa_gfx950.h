// Small gfx950 building blocks shared by the MFMA kernels: vector types, the transposing LDS
// read, direct global -> LDS loads with explicit completion waits, and the fence-free barrier.
#pragma once

#include <utility>

#include "fipa_bf16_common.h"

namespace fipa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// ds_read_b64_tr_b16: within each group of 16 lanes, lane l receives elements
// data[lane 4e + l/4][l%4], e = 0..3, of the 16 x 4 block of 16-bit values the group addresses.
__device__ __forceinline__ bf16x4 lds_read_tr(const char *ptr)
{
    return __builtin_bit_cast(
        bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(ptr)));
}

// Two weights -> one packed bf16 pair (one v_cvt_pk_bf16_f32), and their rounded values added
// to `sum` (one v_dot2c_f32_bf16): sums taken this way add up exactly the numbers the MFMA uses.
__device__ __forceinline__ unsigned pack_pair(float e0, float e1, float &sum)
{
    const bf16x2 b = __builtin_convertvector((f32x2){e0, e1}, bf16x2);
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    sum = __builtin_amdgcn_fdot2_f32_bf16(b, ones, sum, false);
    return __builtin_bit_cast(unsigned, b);
}

// One direct global -> LDS load: 16 bytes per lane, not passing through registers.  Lane l
// fetches base + voff and writes LDS byte (lds_base + LDS_IMM + 16*l); voff is first advanced by
// `step`.  Written as inline assembly so that the compiler neither counts these loads nor
// orders LDS reads after them; completion is awaited explicitly with wait_vmem<N>() before the
// barrier that publishes the data.  (The vector add between the write of m0 and the load also
// covers the wait state the hardware wants between the two.)
template <int LDS_IMM>
__device__ __forceinline__ void dma16(const char *base, int &voff, int step, unsigned lds_base)
{
    asm volatile(
        "s_add_u32 m0, %1, %2\n\t"
        "v_add_u32 %0, %3, %0\n\t"
        "global_load_lds_dwordx4 %0, %4"
        : "+v"(voff)
        : "s"(lds_base), "n"(LDS_IMM), "s"(step), "s"(base)
        : "memory", "m0", "scc");
}

__device__ __forceinline__ unsigned lds_address(const char *ptr)
{
    return (unsigned)(uintptr_t)((__attribute__((address_space(3))) const char *)ptr);
}

// Workgroup barrier without the fence that __syncthreads() adds: for data that arrives by
// direct loads, whose completion each wave awaits itself.
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmem()  // s_waitcnt vmcnt(N) only
{
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// Calls f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}) in order:
// a loop whose index is a constant expression inside the body.
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

}  // namespace fipa
