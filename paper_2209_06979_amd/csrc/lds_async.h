// Asynchronous global -> LDS copies for gfx950.
//
// global_load_lds copies 16 bytes per lane from global memory into LDS without touching
// registers: lane l of the wave writes LDS bytes [M0 + 16*l, M0 + 16*l + 16).  Its
// completion is counted by vmcnt like any load.
//
// The compiler models such a copy (through its builtin) as an access to both memory spaces
// and answers every later dependency on a memory counter with a full wait.  copy16_to_lds
// therefore issues the copy from inline assembly, which the compiler does not track; the
// code that reads the copied rows must call vm_wait<0>() first (and lgkm_wait() before a
// stage is overwritten by a later copy).  Only copies are issued this way: they have no
// register destination.  Every load that returns data in registers stays an ordinary,
// compiler-tracked load -- the compiler is free to move or spill a register right after the
// statement that defines it, which is only safe if it knows when the data arrives.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace mcu {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

// four fp32 values rounded to fp16 (to nearest even; beyond the fp16 range: infinity)
__device__ __forceinline__ v4h to_half4(v4f f) { return (v4h){(_Float16)f.x, (_Float16)f.y, (_Float16)f.z, (_Float16)f.w}; }
typedef __attribute__((address_space(3))) v2i lds_v2i;

// 32-bit LDS address of a pointer into a __shared__ array
__device__ __forceinline__ unsigned lds_addr(const void *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

// The same address made wave-uniform (an SGPR value): the base of a copy must be uniform.
__device__ __forceinline__ unsigned lds_addr_uniform(const void *p) { return __builtin_amdgcn_readfirstlane(lds_addr(p)); }

// 16 bytes per lane, global -> LDS; lane l fetches gbase_uniform + lane_offset and lands at
// lds_base + 16*l.  gbase_uniform (an SGPR pair) and lds_base must be wave-uniform.  The copy
// writes M0; kernels using it contain no other user of M0.
__device__ __forceinline__ void copy16_to_lds(const void *gbase_uniform, unsigned lane_offset, unsigned lds_base)
{
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_base); // no-op for a value already known to be uniform
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_offset), "s"(gbase_uniform), "s"(base)
                 : "memory", "m0");
}

// Transposing 64-bit LDS read of 8-bit elements: inside each group of 16 lanes, lane l
// receives byte (l % 8) of the 8-byte pieces addressed by lanes 2*t + l/8, t = 0..7.
// With lanes 2t and 2t+1 pointing at the two 8-byte halves of a 16-byte row piece, lane l
// ends up with 8 consecutive-row bytes of column l: the MFMA 8-bit operand layout.
__device__ __forceinline__ v2i lds_read_tr8(const void *p) { return __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)p); }

// All memory instructions issued so far (copies included) have completed / at most N remain.
template <int N> __device__ __forceinline__ void vm_wait() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// All LDS reads issued so far have returned (call before a later copy overwrites their source).
__device__ __forceinline__ void lgkm_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

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
