// Asynchronous global -> LDS copies and hand-scheduled memory waits for gfx950.
//
// global_load_lds copies 16 bytes per lane from global memory into LDS without touching
// registers: lane l of the wave writes LDS bytes [M0 + 16*l, M0 + 16*l + 16).  Its
// completion is counted by vmcnt like any load, and loads complete in issue order, so
// "s_waitcnt vmcnt(N)" means: everything except the N youngest memory instructions has
// landed.  That is what lets a wave keep the next chunk's copy in flight while it consumes
// the current one.
//
// The compiler models such a copy as an access to both memory spaces and answers every
// later dependency on a memory counter with a full wait, which would serialise the
// pipeline.  Inside the pipelined loops all vector-memory loads (the copies, the column
// indices, the sparse operand) and the LDS reads of copied data are therefore issued from
// inline assembly, which the compiler does not track, and ordered by explicit waits:
// vm_wait<N>() / lds_wait(), followed by tie() on every register an untracked load wrote,
// so that no use can be scheduled ahead of the wait.  Counters complete in order, so memory
// instructions the compiler does not know about can only make its own waits stricter.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace mcu {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

// 32-bit LDS address of a pointer into a __shared__ array
__device__ __forceinline__ unsigned lds_addr(const void *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

// The same address made wave-uniform (an SGPR value): the base of a copy must be uniform.
__device__ __forceinline__ unsigned lds_addr_uniform(const void *p) { return __builtin_amdgcn_readfirstlane(lds_addr(p)); }

// 16 bytes per lane, global -> LDS; lane l lands at lds_base + 16*l.  lds_base must be a
// wave-uniform value (see lds_addr_uniform).  Untracked: pair with vm_wait<N>().
__device__ __forceinline__ void copy16_to_lds(const void *gsrc, unsigned lds_base)
{
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_base); // no-op for a value already known to be uniform
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(base) : "memory", "m0");
}

// The same with the address split into a wave-uniform base pointer (SGPR pair) and a 32-bit
// per-lane byte offset: no 64-bit address arithmetic per lane.
__device__ __forceinline__ void copy16_to_lds(const void *gbase_uniform, unsigned lane_offset, unsigned lds_base)
{
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_offset), "s"(gbase_uniform), "s"(base)
                 : "memory", "m0");
}

// Untracked 128-bit / 64-bit global loads: the result may be used only after a vm_wait that
// covers the load, followed by tie(result).
__device__ __forceinline__ v4i gload128(const void *gsrc)
{
    v4i d;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(d) : "v"(gsrc) : "memory");
    return d;
}
__device__ __forceinline__ v2i gload64(const void *gsrc)
{
    v2i d;
    asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(d) : "v"(gsrc) : "memory");
    return d;
}

// Transposing 64-bit LDS read of 8-bit elements: inside each group of 16 lanes, lane l
// receives byte (l % 8) of the 8-byte pieces addressed by lanes 2*t + l/8, t = 0..7.
// With lanes 2t and 2t+1 pointing at the two 8-byte halves of a 16-byte row piece, lane l
// ends up with 8 consecutive-row bytes of column l: the MFMA 8-bit operand layout.
template <int OFFSET> __device__ __forceinline__ v2i lds_read_tr8(unsigned addr)
{
    v2i d;
    asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFFSET) : "memory");
    return d;
}

template <int OFFSET> __device__ __forceinline__ v4i lds_read128(unsigned addr)
{
    v4i d;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFFSET) : "memory");
    return d;
}

template <class T> __device__ __forceinline__ void tie(T &r) { asm volatile("" : "+v"(r)); }

// Waits for all LDS reads issued so far; the listed registers (results of lds_read_*) may
// only be used after this call.
template <class... T> __device__ __forceinline__ void lds_wait(T &...regs)
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    (tie(regs), ...);
}

// At most N memory instructions may still be outstanding.
template <int N> __device__ __forceinline__ void vm_wait() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}),
// for bodies that need the counter as a constant (instruction offsets, register arrays).
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

} // namespace mcu
