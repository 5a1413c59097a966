// Global loads that are issued and awaited by hand (inline asm), shared by the prefill and the
// decode kernels.  Not part of the public ABI.
#pragma once

#include "internal.h"

namespace mixllm {

// ---- asynchronous global loads, issued and awaited by hand ---------------------------------
// Inside the main loops every global load is an `asm volatile`, for two reasons.  (1) The
// direct-to-LDS load, when the compiler sees it, makes its wait-count bookkeeping fall back to
// waiting for ALL outstanding memory operations before any later dependent instruction, which
// serialises the fragment pipeline.  (2) The vector-memory counter retires in order: with the
// loads hidden in asm the issue order is exactly the program order, so one `s_waitcnt vmcnt(N)`
// ("all but the youngest N loads of this wave have landed") per group covers everything, and
// the youngest loads - the activation tile two groups ahead - stay in flight across it.
// A register filled by such a load is only read after passing through await_*(), which ties
// the register to the wait.  A wait with N smaller than the number of younger loads merely
// waits longer; it is never unsafe.

// 16 bytes per lane, global -> LDS: lane l writes lds_base + 16 l.  lds_base is wave uniform.
static __device__ inline void load_lds16(uint32_t lds_base, uint32_t voff, const void *sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory", "m0");
}
template <int OFF>
static __device__ inline void load_reg16(v4i &dst, uint32_t voff, const void *sbase)
{
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=&v"(dst) : "v"(voff), "s"(sbase), "n"(OFF) : "memory");
}
// the same, marked non-temporal: weights that are read once
template <int OFF>
static __device__ inline void load_reg16_nt(v4i &dst, uint32_t voff, const void *sbase)
{
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt" : "=&v"(dst) : "v"(voff), "s"(sbase), "n"(OFF) : "memory");
}
static __device__ inline void load_reg8(uint2 &dst, uint32_t voff, const void *sbase)
{
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=&v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
static __device__ inline void load_reg_u16(uint32_t &dst, uint32_t voff, const void *sbase)
{
    asm volatile("global_load_ushort %0, %1, %2" : "=&v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
template <int N>
static __device__ inline void await_loads(v4i &a, v4i &b)
{
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
template <int N>
static __device__ inline void await_loads(v4i &a, v4i &b, v4i &c, v4i &d)
{
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}
template <int N>
static __device__ inline void await_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int N>
static __device__ inline void await_loads(uint32_t &a)
{
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}
template <int N>
static __device__ inline void await_loads(uint2 &a, uint32_t &b)
{
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
// Block-wide barrier in the middle of a group, written out instead of __syncthreads(): the
// fence of the latter would wait for every outstanding load and LDS read.  The caller has
// already waited for what must have landed; LDS_WRITES adds this wave's own LDS stores.
template <bool LDS_WRITES>
static __device__ inline void mid_group_barrier()
{
    if (LDS_WRITES)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else
        asm volatile("s_barrier" ::: "memory");
}
static __device__ inline uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}

// fp16 bit pattern (low 16 bits) -> float.  Values that come out of a hand-issued load are taken
// apart with integer operations and this function only: a reinterpreting copy of the loaded
// variable itself (memcpy to an array of halves, a union) makes the compiler keep the variable
// as 16-bit pieces, and it then splits the register right after the load is issued - before the
// data has arrived - and reassembles it for the wait.
static __device__ inline float half_bits_to_float(uint32_t bits)
{
    return (float)__builtin_bit_cast(half_t, (uint16_t)bits);
}

}  // namespace mixllm
