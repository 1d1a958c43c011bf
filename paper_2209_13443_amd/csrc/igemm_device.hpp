// Device helpers shared by the matrix-core convolution kernels (gfx950): asynchronous global -> LDS
// copies, waits, compile-time loops, requantisation arithmetic.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>
#include <utility>

#ifndef EE_FRAG_DISTANCE
#define EE_FRAG_DISTANCE 2      // sub-steps between the read of a fragment and the matrix instructions that use it (pipelined steps)
#endif

namespace ee {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

namespace {

__device__ __forceinline__ unsigned lds_addr(const void* p)
{
    return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// 16 bytes per lane, global -> LDS, asynchronous (counted by vmcnt).  lds_base must be wave-uniform.
__device__ __forceinline__ void dma16(unsigned lds_base, const void* gptr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
__device__ __forceinline__ void dma16(unsigned lds_base, const void* uniform_base, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(uniform_base) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_copies_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// also waits for this wavefront's own LDS reads
template <int N>
__device__ __forceinline__ void wait_all_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// bytes of LDS the ring takes: the stages in use, and never less than the output tile that reuses it
__host__ __device__ constexpr unsigned igemm_ring_bytes(int ns, int nk, int stage_bytes, int tile_o)
{
    const int used = (ns < nk ? ns : nk) * stage_bytes;
    return (unsigned)(used > tile_o ? used : tile_o);
}
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), unrolled at compile time
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    [&]<int... I>(std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }(std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ unsigned fast_div(unsigned m, unsigned d, unsigned magic)   // magic = floor(2^32 / d), d >= 1
{
    unsigned q = __umulhi(m, magic);
    if (m - q * d >= d) ++q;
    return q;
}

__device__ __forceinline__ uint32_t to_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ int clamp_i32(int v, int lo, int hi)       // lo <= hi
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}
// the low bytes of four ints as one dword, q0 lowest
__device__ __forceinline__ unsigned pack4_i8(int q0, int q1, int q2, int q3)
{
    const unsigned lo = __builtin_amdgcn_perm((unsigned)q1, (unsigned)q0, 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm((unsigned)q3, (unsigned)q2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

}  // namespace

}  // namespace ee
