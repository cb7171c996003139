// LDS accesses written as inline assembly, and a compile-time loop (gfx950).
//
// The compiler orders every LDS access it knows of behind ALL outstanding direct-to-LDS loads
// (global_load_lds): it cannot tell which LDS bytes such a load writes.  A kernel that prefetches
// tiles into a ring of LDS buffers would therefore wait for its whole prefetch before touching the
// tile that has already landed.  Reads issued from inline assembly are invisible to that rule.  The
// price is that the waits are ours: lds_wait<N> holds the named registers until at most N younger
// LDS operations of this wavefront are outstanding (LDS returns data in issue order).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

#define MAGE_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define MAGE_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define MAGE_LDS_ADDR(a) ((__attribute__((address_space(3))) void *)(uintptr_t)(a))   // from a 32-bit LDS byte address

namespace mage {

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

template <int OFF>
__device__ __forceinline__ u32x4_t lds_read_b128(unsigned addr)
{
    u32x4_t r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

// Transposing read: within each 16-lane block, lane i' addresses 4 channels of one key; lane i
// receives channel i of 4 keys.
template <int OFF>
__device__ __forceinline__ u32x2_t lds_read_tr16_b64(unsigned addr)
{
    u32x2_t r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

template <int N>
__device__ __forceinline__ void lds_wait(u32x4_t &r)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r) : "n"(N));
}

template <int N>
__device__ __forceinline__ void lds_wait(u32x2_t &a, u32x2_t &b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}

template <int OFF>
__device__ __forceinline__ float lds_read_f32(unsigned addr)
{
    float r;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

template <int N>
__device__ __forceinline__ void lds_wait(float &r)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r) : "n"(N));
}

// The same idea for a global load into registers whose completion the caller tracks itself:
// vm_wait<N> holds the register until at most N younger vector-memory loads are outstanding.
template <int OFF>
__device__ __forceinline__ u32x4_t global_load_b128(const void *p)
{
    u32x4_t r;
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=&v"(r) : "v"(p), "n"(OFF));
    return r;
}

template <int N>
__device__ __forceinline__ void vm_wait(u32x4_t &r)
{
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N));
}

// Both 32-lane halves of a value, for every lane: lo = x of lane (l % 32), hi = x of lane 32 + l % 32
// (v_permlane32_swap exchanges the upper half of its first register with the lower half of its
// second; started from two copies of x, the first ends up all-lower and the second all-upper).
// Written as assembly: the builtin's two results were merged into one by the optimiser whenever
// they met in a commutative operation.  The wait states cover a vector-ALU write of x right before.
__device__ __forceinline__ void lane_halves(float x, float &lo, float &hi)
{
    lo = x;
    hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
}

// The same across a pair of 16-lane rows: lo = x of the even row of this lane's row pair (rows 0 and 2
// of the wavefront), hi = x of the odd row (rows 1 and 3), same lane within the row
// (v_permlane16_swap exchanges the odd rows of its first register with the even rows of its second).
__device__ __forceinline__ void lane_rows16(float x, float &lo, float &hi)
{
    lo = x;
    hi = x;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
}

__device__ __forceinline__ unsigned lds_addr(const void *p) { return (unsigned)(uintptr_t)MAGE_LDS_PTR(p); }

template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}

template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

}  // namespace mage
